"""cbd_best_paths_static, the entry point that allocates nothing, against cbd_best_paths: same results, to the
bit, on two calls in a row (the second with fewer channels, so that what the first call left in the fixed result
area must not show), then after more decoding, with final costs, and on a request too large for the fixed area."""
import numpy as np
import pytest

from paper_2306_15685_amd import synth
from paper_2306_15685_amd import binding as B

import gpu_harness as GH

pytestmark = pytest.mark.gpu


def same(a, b, where):
    st_a, w_a, arcs_a, cost_a, na_a, nw_a = a
    st_b, w_b, arcs_b, cost_b, na_b, nw_b = b
    assert np.array_equal(st_a, st_b), f"{where}: status"
    assert np.array_equal(na_a, na_b) and np.array_equal(nw_a, nw_b), f"{where}: counts"
    assert cost_a.tobytes() == cost_b.tobytes(), f"{where}: cost bits"
    for i in range(len(w_a)):
        assert np.array_equal(w_a[i], w_b[i]), f"{where}: words of row {i}"
        assert np.array_equal(arcs_a[i], arcs_b[i]), f"{where}: arcs of row {i}"


def test_static_result_area_matches_best_paths():
    import torch
    assert torch.cuda.is_available()
    torch.cuda.set_device(0)
    C, T, S, P = 12, 60, 60_000, 500
    g = synth.make_graph(S, P, 2000, 0.10, seed_stream=(77,), with_finals=True)
    L = synth.make_loglikes(C, T, P, 4.0, seed_stream=(77,), device="cuda")
    w = synth.scaled(synth.WORKLOADS["large"], channels=C, ctx_min=30, ctx_max=60, config_id=77)
    ctxs, offs = synth.make_contexts(w, g)
    dec = GH.GpuDecoder(g, C, 13.0, 300, max_frames=T, max_context_arcs=max(len(x) for x in ctxs))
    try:
        cap = 4 * T + 16
        everyone = np.arange(C, dtype=np.int32)
        some = np.array([7, 2, 9, 4, 0], dtype=np.int32)
        dec.set_contexts(ctxs, offs)
        dec.reset()
        dec.advance(L, 0, 40)
        # two calls in a row, the second with a smaller input
        same(B.cbd_best_paths_static(dec.dh, everyone, False, cap), B.cbd_best_paths(dec.dh, everyone, False, cap),
             "all channels after 40 frames")
        same(B.cbd_best_paths_static(dec.dh, some, False, cap), B.cbd_best_paths(dec.dh, some, False, cap),
             "five channels after 40 frames")
        got = B.cbd_best_paths_static(dec.dh, some, False, cap)
        for i, c in enumerate(some):
            rc, words, arcs, cost = dec.best(int(c))
            assert rc == got[0][i] == 0 and np.array_equal(words, got[1][i]) and np.array_equal(arcs, got[2][i])
            assert np.float32(cost) == got[3][i]
        # one channel restarted, words only, final costs, after more decoding
        B.cbd_reset_channels(dec.dh, np.array([3], np.int32))
        dec.advance(L, 40, T)
        same(B.cbd_best_paths_static(dec.dh, everyone, True, cap), B.cbd_best_paths(dec.dh, everyone, True, cap),
             "all channels, final costs")
        a = B.cbd_best_paths_static(dec.dh, some, True, cap, want_arcs=False)
        b = B.cbd_best_paths(dec.dh, some, True, cap, want_arcs=False)
        assert a[2] is None and b[2] is None
        for i in range(len(some)):
            assert np.array_equal(a[1][i], b[1][i])
        # an output buffer that is too small reports the needed sizes the same way
        small_a = B.cbd_best_paths_static(dec.dh, some, False, 8)
        small_b = B.cbd_best_paths(dec.dh, some, False, 8)
        assert (small_a[0] == B.CBD_E_BUFFER).all() and np.array_equal(small_a[0], small_b[0])
        assert np.array_equal(small_a[4], small_b[4]) and np.array_equal(small_a[5], small_b[5])
        # beyond the fixed area: refused with a clear error, nothing enqueued
        with pytest.raises(B.CbdError) as e:
            B.cbd_best_paths_static(dec.dh, everyone, False, 1 << 20)
        assert e.value.status == B.CBD_E_CAPACITY
        same(B.cbd_best_paths_static(dec.dh, everyone, False, cap), B.cbd_best_paths(dec.dh, everyone, False, cap),
             "after the refused request")
    finally:
        dec.close()
