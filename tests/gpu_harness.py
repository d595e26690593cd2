"""Shared plumbing of the GPU parity tests: run the same seeded inputs through the HIP
library (via the C ABI binding) and through the CPU checker, and compare."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from paper_2306_15685_amd import binding as B
from oracle import OracleGraph, OracleChannel


class GpuDecoder:
    """Owns a graph handle and a decoder handle on the current torch stream."""

    def __init__(self, g, channels, beam, max_active=0, max_frames=512, max_context_arcs=1024, lookup_mode=0,
                 hash_log2=12, table_location=0, records_per_frame=0, max_eps_iters=0, graph_handle=None,
                 lds_token_cap=0, max_pool_contexts=0, workgroups_per_cu=0, compact_records_above=0, block_threads=0, frame_code=0,
                 workgroups_per_channel=0):
        import torch
        self.torch = torch
        self.g = g
        self.own_graph = graph_handle is None
        self.gh = graph_handle if graph_handle is not None else B.cbd_graph_load(
            g.num_states, g.num_pdfs, g.start_state, g.row_offsets, g.dst, g.ilabel, g.olabel, g.weight, g.final_cost)
        self.C = channels
        self.dh = B.cbd_decoder_create(self.gh, channels, beam, max_active, max_frames, max_context_arcs, lookup_mode,
                                       hash_log2, max_eps_iters, records_per_frame, table_location, lds_token_cap,
                                       max_pool_contexts, workgroups_per_cu, compact_records_above, block_threads, frame_code,
                                       workgroups_per_channel,
                                       hip_stream=torch.cuda.current_stream().cuda_stream)
        self.all = np.arange(channels, dtype=np.int32)

    def close(self):
        if self.dh is not None:
            B.cbd_decoder_free(self.dh)
            self.dh = None
        if self.own_graph and self.gh is not None:
            B.cbd_graph_free(self.gh)
            self.gh = None

    def reset(self, channels=None):
        B.cbd_reset_channels(self.dh, self.all if channels is None else channels)

    def set_contexts(self, lists, offsets, channels=None):
        B.cbd_set_contexts(self.dh, self.all if channels is None else channels, lists, offsets)

    def advance(self, L, t0, t1, channels=None):
        """L: device tensor [C, T, P] (contiguous); decodes frames [t0, t1) of the listed channels
        (rows of L are taken in list order, so a channel subset needs a matching tensor)."""
        assert L.is_cuda and L.dtype == self.torch.float32 and L.is_contiguous()
        Cc, T, P = L.shape
        ptr = L.data_ptr() + 4 * t0 * P
        B.cbd_advance(self.dh, self.all if channels is None else channels, ptr, T * P, t1 - t0)

    def compact(self, channels=None, min_new_records=0):
        B.cbd_compact_records(self.dh, self.all if channels is None else channels, min_new_records)

    def records(self, c):
        return B.cbd_get_records(self.dh, c)

    def tokens(self, c):
        return B.cbd_get_tokens(self.dh, c)

    def best(self, c, use_final=False):
        return B.cbd_best_path(self.dh, c, use_final)

    def stats(self, c=-1):
        return B.cbd_get_stats(self.dh, c)


def oracle_channels(g, n, beam, max_active=0, max_eps_iters=64, og=None) -> List[OracleChannel]:
    og = og or OracleGraph.from_graph(g)
    return [OracleChannel(og, beam, max_active, max_eps_iters) for _ in range(n)]


def assert_tables_equal(gpu_tab, orc_tab, where=""):
    rc, gs, gc, ga = gpu_tab
    os_, oc, oa = orc_tab
    assert rc == 0, f"{where}: gpu status {rc}"
    assert gs.size == os_.size, f"{where}: table sizes differ gpu {gs.size} vs checker {os_.size}"
    assert np.array_equal(gs, os_), f"{where}: states differ"
    # costs: same bits (value-equal covers -0/+0)
    assert np.array_equal(gc, oc), f"{where}: costs differ, max abs {np.abs(gc - oc).max()}"
    assert np.array_equal(ga, oa), f"{where}: arcs differ"


def assert_best_equal(gpu_best, orc_best, where="", tol=1e-3):
    grc, gw, ga, gcost = gpu_best
    orc, ow, oa, ocost = orc_best
    # the checker's codes are positive, the library's negative
    if orc == 1:
        assert grc == B.CBD_E_NO_TOKENS, f"{where}: checker has no tokens, gpu status {grc}"
        return
    if orc == 2:
        assert grc == B.CBD_E_EPS_DIVERGED, f"{where}: checker diverged, gpu status {grc}"
        return
    assert grc == 0, f"{where}: gpu status {grc}"
    assert np.array_equal(ga, oa), f"{where}: back-pointer paths differ"
    assert np.array_equal(gw, ow), f"{where}: words differ"
    assert abs(gcost - ocost) <= tol, f"{where}: cost {gcost} vs {ocost}"
    assert np.float32(gcost) == np.float32(ocost), f"{where}: cost bits differ {gcost} vs {ocost}"
