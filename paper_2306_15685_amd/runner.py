"""Drives a synthetic workload through the HIP library: the launch configuration that
bench.py times and that the full-size parity tests check.

torch is used for device memory, streams and events only.
"""
from __future__ import annotations

import time
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional

import numpy as np

from . import binding as B
from . import synth


def default_hash_log2(w: synth.Workload) -> int:
    """Device-memory tables (used by the frames that outgrow LDS): 8192 tokens per frame; the
    lexicon-loop workload holds a table entry per word start, so it gets 32768."""
    return 16 if w.name.startswith("e2e") else 14


def default_team(w: synth.Workload) -> int:
    """Workgroups per channel: the lexicon-loop workload's frames (20,000 tokens) are shared by teams of four
    (64 channels x 4 = the 256 compute units); the HCLG-style workloads fit one workgroup's LDS."""
    return 4 if w.name.startswith("e2e") and w.channels * 4 <= 256 else 1


def default_records_per_frame(w: synth.Workload) -> int:
    return 24_576 if w.name.startswith("e2e") else DEFAULT_RECORDS_PER_FRAME


# Back-pointer records reserved per frame and channel (the workloads here average 350-500 tokens a frame).
DEFAULT_RECORDS_PER_FRAME = 1536


@dataclass
class Inputs:
    w: synth.Workload
    g: synth.Graph
    loglikes: list  # per segment: device tensor [C, frames, P]
    contexts: Optional[list]  # per segment: (arc lists, offsets); None until built from `sequences`
    sequences: Optional[list] = None  # per segment: (per-channel lists of word sequences, offsets)
    context_build: Optional[Dict] = None  # host time of Algorithm 1 (filled with `contexts`)


def make_inputs(w: synth.Workload, g: Optional[synth.Graph] = None, device: str = "cuda") -> Inputs:
    """Synthetic inputs of a workload.  A workload whose graph spaces its word labels (word_period) gets its
    biasing lists as word sequences; the arc lists are made of them by the library (contexts_from_words)."""
    g = g if g is not None else synth.graph_for(w)
    L = [synth.make_loglikes(w.channels, w.frames, w.num_pdfs, w.sigma, seed_stream=(w.config_id, s), device=device)
         for s in range(w.segments)]
    if w.word_period > 0:
        return Inputs(w, g, L, None, [synth.make_context_sequences(w, g, segment=s) for s in range(w.segments)])
    ctx = [synth.make_contexts(w, g, segment=s) for s in range(w.segments)]
    return Inputs(w, g, L, ctx)


def contexts_from_words(graph_handle, sequences: list):
    """Algorithm 1 through the library for every channel's list of word sequences (Sec. 4.1) -> the (arc lists,
    offsets) per segment that the decoder takes, and the host time the calls took."""
    out, n, t0 = [], 0, time.perf_counter()
    for per_channel, offs in sequences:
        out.append(([B.cbd_context_from_words(graph_handle, seqs) for seqs in per_channel], offs))
        n += len(per_channel)
    dt = time.perf_counter() - t0
    arcs = sum(int(x.size) for lists, _ in out for x in lists)
    return out, {"lists": n, "ms_per_list": 1e3 * dt / max(n, 1), "arcs_per_list": arcs / max(n, 1), "threads": 1}


class Session:
    """A decoder sized for a workload, bound to torch's current stream."""

    def __init__(self, inp: Inputs, hash_log2: Optional[int] = None, table_location: int = 0,
                 records_per_frame: int = 0, graph_handle=None, biased: bool = True, lds_token_cap: int = 0,
                 context_mode: str = "upload", async_partials: bool = True, workgroups_per_cu: int = 0,
                 compact_records_above: int = 0, record_frames: int = 0, tail_partials: bool = False,
                 block_threads: int = 0, frame_code: int = 0, workgroups_per_channel: int = -1):
        """compact_records_above / record_frames: automatic compaction of the back-pointer records, and the number
        of frames the record buffer is sized for (0: the whole utterance).  tail_partials: partial results through
        cbd_best_tails_begin / _finish (only the part of the path above what the compactions have fixed).
        context_mode: "upload" sends every segment's lists with cbd_set_contexts; "pool" loads all
        segments' lists once with cbd_contexts_create and switches by id (Sec. 4.3)."""
        import torch
        self.torch = torch
        self.inp = inp
        w, g = inp.w, inp.g
        self.w = w
        self.biased = biased
        self.own_graph = graph_handle is None
        self.gh = graph_handle if graph_handle is not None else B.cbd_graph_load(
            g.num_states, g.num_pdfs, g.start_state, g.row_offsets, g.dst, g.ilabel, g.olabel, g.weight, g.final_cost)
        if inp.contexts is None:
            inp.contexts, inp.context_build = contexts_from_words(self.gh, inp.sequences)
        max_ctx = max([w.ctx_max, 1] + [int(x.size) for lists, _ in inp.contexts for x in lists])
        if workgroups_per_channel < 0:
            workgroups_per_channel = default_team(w)
        self.stream = torch.cuda.current_stream()
        self.dh = B.cbd_decoder_create(
            self.gh, w.channels, w.beam, w.max_active, record_frames or w.frames, max_ctx, w.lookup_mode,
            hash_log2 if hash_log2 is not None else default_hash_log2(w), 0,
            records_per_frame or default_records_per_frame(w), table_location, lds_token_cap,
            w.channels * w.segments if context_mode == "pool" else 0, workgroups_per_cu, compact_records_above,
            block_threads, frame_code, workgroups_per_channel, hip_stream=self.stream.cuda_stream)
        self.context_mode = context_mode
        self.async_partials = async_partials   # partial results through cbd_best_paths_begin / _finish
        self.begin_partial = B.cbd_best_tails_begin if tail_partials else B.cbd_best_paths_begin
        self.finish_partial = B.cbd_best_tails_finish if tail_partials else B.cbd_best_paths_finish
        self.sync_partial = B.cbd_best_tails if tail_partials else B.cbd_best_paths
        # contexts packed once: per segment (arc_idx, list_offsets)
        self.packed = [B.pack_lists(lists) for lists, _ in inp.contexts]
        self.pool_ids = None
        if context_mode == "pool":
            self.pool_ids = [B.cbd_contexts_create(self.dh, None, offs, packed=self.packed[s])
                             for s, (_, offs) in enumerate(inp.contexts)]
        self.all = np.arange(w.channels, dtype=np.int32)
        self.capacity = 4 * w.frames + 64
        self.buffers = B.BestPathBuffers(w.channels, self.capacity, want_arcs=True)
        self.advance_events: List = []
        self.time_kernels = False
        self.on_partial: Optional[Callable] = None  # called with (segment, frames_done, best_paths result)
        self.partials: list = []

    def close(self):
        if self.dh is not None:
            B.cbd_decoder_free(self.dh)
            self.dh = None
        if self.own_graph and self.gh is not None:
            B.cbd_graph_free(self.gh)
            self.gh = None

    def _advance(self, L, t0, n):
        C, T, P = L.shape
        if self.time_kernels:
            e0 = self.torch.cuda.Event(enable_timing=True)
            e1 = self.torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)
        B.cbd_advance(self.dh, self.all, L.data_ptr() + 4 * t0 * P, T * P, n)
        if self.time_kernels:
            e1.record(self.stream)
            self.advance_events.append((e0, e1))

    def step(self, keep_results: bool = False, collect_stats: bool = False):
        """One pass of the workload: per segment, upload contexts, start the utterances, advance
        chunk by chunk (with a partial best path per chunk where the workload says so), read the
        final best paths.  With collect_stats the per-utterance counters are summed over the
        segments into self.step_stats (adds a synchronisation per segment)."""
        w = self.w
        finals = []
        pending_final = None   # ticket of the previous utterance's final result, still in flight
        self.step_stats = None
        for s in range(w.segments):
            lists, offs = self.inp.contexts[s]
            if self.biased and self.context_mode == "pool":
                B.cbd_use_contexts(self.dh, self.all, self.pool_ids[s])
            elif self.biased:
                B.cbd_set_contexts(self.dh, self.all, None, offs, packed=self.packed[s])
            elif s == 0:
                B.cbd_set_contexts(self.dh, self.all, [np.zeros(0, np.int32)] * w.channels,
                                   np.zeros(w.channels, np.float32))
            B.cbd_reset_channels(self.dh, self.all)
            L = self.inp.loglikes[s]
            t = 0
            pending = None   # (ticket, frames done) of the partial request still in flight
            while t < w.frames:
                n = min(w.chunk, w.frames - t)
                self._advance(L, t, n)
                t += n
                if pending_final is not None:
                    # the previous utterance's final result: collected now that this utterance's first chunk is
                    # queued behind it, so the GPU is not left idle while the host reads results
                    r = B.cbd_best_paths_finish(self.dh, pending_final, buffers=self.buffers, as_lists=keep_results)
                    pending_final = None
                    if keep_results:
                        finals.append(r)
                if w.partial_every_chunk and t < w.frames:
                    if self.async_partials:
                        # one request in flight: the walk and copy of chunk k overlap the decoding of chunk k+1.
                        # The previous request is collected first: its copies are queued on the side stream and
                        # must not end up behind the walk that is about to be queued there.
                        if pending is not None:
                            r = self.finish_partial(self.dh, pending[0], buffers=self.buffers, as_lists=keep_results)
                            if keep_results:
                                self.partials.append((s, pending[1], r))
                        tk = self.begin_partial(self.dh, self.all, False, self.capacity, want_arcs=keep_results)
                        pending = (tk, t)
                    else:
                        r = self.sync_partial(self.dh, self.all, False, self.capacity, want_arcs=keep_results,
                                              buffers=self.buffers, as_lists=keep_results)
                        if keep_results:
                            self.partials.append((s, t, r))
            if pending is not None:
                r = self.finish_partial(self.dh, pending[0], buffers=self.buffers, as_lists=keep_results)
                if keep_results:
                    self.partials.append((s, pending[1], r))
            if self.async_partials and s + 1 < w.segments and not collect_stats:
                # (the next utterance's reset waits on the device for this walk: it reuses the record buffer)
                pending_final = B.cbd_best_paths_begin(self.dh, self.all, True, self.capacity, want_arcs=keep_results)
            else:
                r = B.cbd_best_paths(self.dh, self.all, True, self.capacity, want_arcs=keep_results,
                                     buffers=self.buffers, as_lists=keep_results)
                if keep_results:
                    finals.append(r)
            if collect_stats:
                st = self.stats(-1)
                if self.step_stats is None:
                    self.step_stats = dict(st)
                else:
                    for k, v in st.items():
                        if k == "status":
                            self.step_stats[k] = self.step_stats[k] or v
                        elif k == "max_tokens":
                            self.step_stats[k] = max(self.step_stats[k], v)
                        else:
                            self.step_stats[k] += v
        return finals

    def stats(self, c: int = -1) -> Dict:
        return B.cbd_get_stats(self.dh, c)

    def kernel_ms(self) -> List[float]:
        self.torch.cuda.synchronize()
        out = [a.elapsed_time(b) for a, b in self.advance_events]
        self.advance_events = []
        return out


# Algorithmic bytes the method must move, per unit of work (HBM side).
BYTES_PER_ACTIVE_TOKEN = 16     # token (state, cost) + the two row offsets of its state
BYTES_PER_ARC = 12              # dst, ilabel, weight of an expanded arc (emitting or epsilon)
BYTES_PER_CANDIDATE = 24        # key probe + 64-bit read-modify-write of the state table
BYTES_PER_TOKEN = 44            # table read, token write, back-pointer write, prune re-read, slot clear


def algorithmic_bytes(st: Dict, w: synth.Workload, ctx_ints: int = 0) -> int:
    """Bytes implied by the counters of cbd_get_stats for the frames they cover."""
    return (BYTES_PER_ACTIVE_TOKEN * st["active_tokens"]
            + BYTES_PER_ARC * (st["emit_arcs"] + st["eps_arcs"])
            + BYTES_PER_CANDIDATE * st["candidates"]
            + BYTES_PER_TOKEN * st["tokens"]
            + 4 * w.num_pdfs * st["frames"]
            + 4 * ctx_ints)
