"""Teams of workgroups per channel (cbd_config.workgroups_per_channel): the same results as one workgroup per
channel, against the checker."""
import numpy as np
import pytest

from paper_2306_15685_amd import synth
from paper_2306_15685_amd import binding as B

import gpu_harness as GH
from oracle import OracleGraph
from test_gpu_parity import run_batch, mid_inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    return torch


@pytest.mark.parametrize("k", [2, 4, 8])
def test_team_random_graph(torch_cuda, k):
    """HCLG-style random graph with epsilon closures up to a few levels deep, ragged chunks, a partial result per
    chunk, contexts per channel."""
    print(f"team of {k}: random graph", flush=True)
    g, L, ctxs, offs = mid_inputs(torch_cuda)
    s = run_batch(torch_cuda, g, L, ctxs, offs, beam=13.0, max_active=0, chunks=[1, 7, 16, 24], hash_log2=16,
                  workgroups_per_channel=k)
    assert s["eps_arcs"] > 0 and s["frames"] == L.shape[0] * L.shape[1]


def test_team_histogram_pruning(torch_cuda):
    print("team of 4: max-active engaged", flush=True)
    g, L, ctxs, offs = mid_inputs(torch_cuda, seed=12)
    s = run_batch(torch_cuda, g, L, ctxs, offs, beam=14.0, max_active=150, chunks=[12, 12, 24], hash_log2=16,
                  workgroups_per_channel=4, use_final=False)
    assert s["max_tokens"] > 150


def test_team_lexicon_loop_long_hub_row(torch_cuda):
    """A hub row of 1,500 arcs (shared out over the team once it has been announced, by one member's waves in the
    frame after the reset), word-end epsilon arcs that all lead back to the hub, max-active engaged."""
    print("team of 4: lexicon loop", flush=True)
    torch = torch_cuda
    g = synth.make_lexicon_graph(24, 1500, seed_stream=(91,))
    C, T = 5, 40
    L = synth.make_loglikes(C, T, g.num_pdfs, 2.0, seed_stream=(91,), device="cuda")
    w = synth.scaled(synth.WORKLOADS["e2e"], channels=C, ctx_min=20, ctx_max=60, config_id=91)
    ctxs, offs = synth.make_contexts(w, g)
    s = run_batch(torch, g, L, ctxs, offs, beam=8.0, max_active=400, chunks=[3, 10, 27], hash_log2=16, lookup_mode=1,
                  workgroups_per_channel=4)
    assert s["max_tokens"] > 400


def test_team_final_costs_swap_and_subset(torch_cuda):
    """Final costs in the best path, a context swap in mid-utterance, and calls on a subset of the channels (the
    grid is then padded with teams that return at once)."""
    print("team of 4: finals, swap, subset", flush=True)
    torch = torch_cuda
    g, L, ctxs, offs = mid_inputs(torch, finals=True, seed=14)
    w2 = synth.scaled(synth.WORKLOADS["large"], channels=L.shape[0], ctx_min=10, ctx_max=40, config_id=77)
    ctxs2, offs2 = synth.make_contexts(w2, g)
    s = run_batch(torch, g, L, ctxs, offs, beam=12.0, max_active=0, chunks=[8, 16, 24], hash_log2=16, use_final=True,
                  swap=(24, ctxs2, offs2), workgroups_per_channel=4)
    assert s["frames"] == L.shape[0] * L.shape[1]
    # a subset of the channels, in another order, results through the asynchronous calls
    C, T, P = L.shape
    sub = np.array([4, 1, 3], np.int32)
    Lsub = L[torch.as_tensor(sub.astype(np.int64), device="cuda")].contiguous()
    dec = GH.GpuDecoder(g, C, 12.0, 0, max_frames=T, hash_log2=16, max_context_arcs=64, workgroups_per_channel=4)
    try:
        orcs = GH.oracle_channels(g, C, 12.0, 0)
        dec.set_contexts([ctxs[c] for c in sub], [offs[c] for c in sub], channels=sub)
        dec.reset(sub)
        Lh = L.cpu().numpy()
        for c in sub:
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset()
        for t0, t1 in ((0, 20), (20, T)):
            dec.advance(Lsub, t0, t1, channels=sub)
            tk = B.cbd_best_paths_begin(dec.dh, sub, False, 4 * T + 16, want_arcs=True)
            st, wl, al, cost, na, nw = B.cbd_best_paths_finish(dec.dh, tk)
            for i, c in enumerate(sub):
                orcs[c].advance(Lh[c, t0:t1])
                GH.assert_best_equal((int(st[i]), wl[i], al[i], float(cost[i])), orcs[c].best_path(False), f"subset t={t1} ch={c}")
    finally:
        dec.close()


def test_team_overflow_parks_the_channel_and_reset_revives_it(torch_cuda):
    """A member's share of the tokens is too small for the frames (hash_capacity_log2 sizes the token arrays): the
    member that runs out marks the failure before the next team barrier, all members leave together, the channel
    reports CBD_E_CAPACITY until it is reset, and other channels are not affected.  Every kernel ends normally."""
    print("team of 4: overflow and reset", flush=True)
    torch = torch_cuda
    g, L, ctxs, offs = mid_inputs(torch, seed=15)
    C, T, P = L.shape
    dec = GH.GpuDecoder(g, C, 16.0, 0, max_frames=T, hash_log2=9, max_context_arcs=64, workgroups_per_channel=4,
                        records_per_frame=64)
    try:
        dec.set_contexts(ctxs, offs)
        dec.reset()
        dec.advance(L, 0, T)
        st = [dec.best(c)[0] for c in range(C)]
        assert all(s == B.CBD_E_CAPACITY for s in st), st       # 64 tokens per member do not hold these frames
        dec.advance(L, 0, 4)                                     # parked: nothing happens, nothing hangs
        assert dec.best(0)[0] == B.CBD_E_CAPACITY
        dec.reset()
        orcs = GH.oracle_channels(g, C, 16.0, 0)
        Lh = L.cpu().numpy()
        dec.advance(L, 0, 1)                                     # one frame from the start fits
        for c in range(C):
            orcs[c].set_context(ctxs[c], offs[c]); orcs[c].reset(); orcs[c].advance(Lh[c, 0:1])
            if orcs[c].stat(3) <= 48:
                GH.assert_best_equal(dec.best(c), orcs[c].best_path(False), f"after reset ch={c}")
    finally:
        dec.close()
