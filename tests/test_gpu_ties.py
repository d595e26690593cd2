"""GPU parity on the method's tie and edge cases: crafted graphs in which costs are bit-equal, so that the
recombination's tie order, the start token's place in it, the beam's edge, the full bin 0 of the pruning
histogram, signed zeros and zero-weight epsilon cycles are exercised on the device (random fp32 scores never
tie).  Every case runs through the C ABI with the tables in LDS and in device memory and is compared with the
CPU checker frame by frame (whole token table: states, cost bits, arcs), then on the best path."""
import numpy as np
import pytest

from paper_2306_15685_amd import synth
from paper_2306_15685_amd import binding as B

import gpu_harness as GH
from oracle import OracleGraph, OracleChannel

pytestmark = pytest.mark.gpu

LOCATIONS = [1, 2]   # state table in LDS / in device memory


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    torch.cuda.set_device(0)
    return torch


def graph(row, dst, il, ol, wt, num_pdfs=1, finals=None):
    row = np.asarray(row, np.int32)
    return synth.Graph(len(row) - 1, len(dst), num_pdfs, max(max(ol), 1), 0, row, np.asarray(dst, np.int32),
                       np.asarray(il, np.int32), np.asarray(ol, np.int32), np.asarray(wt, np.float32),
                       None if finals is None else np.asarray(finals, np.float32))


def both(torch, g, L, beam, max_active, table_location, ctx=None, offset=0.0, max_eps_iters=0, use_final=False,
         expect_tables=None):
    """Decode L ([T, P] host array) frame by frame on the device and on the checker; compare the table after the
    start and after every frame, then the best path.  Returns the checker's tables as dicts state -> (cost, arc)."""
    T = L.shape[0]
    Ld = torch.tensor(L, dtype=torch.float32, device="cuda").unsqueeze(0).contiguous()
    dec = GH.GpuDecoder(g, 1, beam, max_active, max_frames=max(T, 1), hash_log2=8, table_location=table_location,
                        max_eps_iters=max_eps_iters, max_context_arcs=max(1, 0 if ctx is None else len(ctx)))
    tables = []
    try:
        orc = OracleChannel(OracleGraph.from_graph(g), beam, max_active, max_eps_iters or 64)
        if ctx is not None:
            dec.set_contexts([np.asarray(ctx, np.int32)], [offset])
            orc.set_context(np.asarray(ctx, np.int32), offset)
        dec.reset(); orc.reset()
        if orc.status == 0:
            GH.assert_tables_equal(dec.tokens(0), orc.tokens(), "after the start")
        for t in range(T):
            dec.advance(Ld, t, t + 1)
            orc.advance(L[t:t + 1])
            if orc.status != 0:
                break
            GH.assert_tables_equal(dec.tokens(0), orc.tokens(), f"frame {t}")
            st, co, ar = orc.tokens()
            tables.append({int(s): (np.float32(c), int(a)) for s, c, a in zip(st, co, ar)})
        GH.assert_best_equal(dec.best(0, use_final), orc.best_path(use_final), "best path")
        if orc.status == 0:
            stc = dec.stats(0)
            assert stc["emit_arcs"] == orc.emit_arcs and stc["tokens"] == orc.stat(1)
            assert stc["active_tokens"] == orc.stat(2) and stc["max_tokens"] == orc.stat(3)
        return tables, dec.best(0, use_final), orc.best_path(use_final)
    finally:
        dec.close()


@pytest.mark.parametrize("loc", LOCATIONS)
def test_lower_source_state_then_lower_arc_wins(torch_cuda, loc):
    """Three arcs reach state 2 at cost 1.0: two from state 0, one from state 1 (itself reached through an
    epsilon arc).  The lower source state wins, then the lower arc index."""
    g = graph([0, 3, 4, 6, 6], [1, 2, 2, 2, 3, 3], [0, 1, 1, 1, 0, 1], [0, 1, 2, 3, 4, 5],
              [1.0, 1.0, 1.0, 0.0, 1.0, 1.0])
    L = np.zeros((2, 1), np.float32)
    tables, gpu_best, _ = both(torch_cuda, g, L[:1], 1.0e30, 0, loc)
    assert tables[0][2] == (np.float32(1.0), 1)
    assert tables[0][3] == (np.float32(2.0), 4)
    assert gpu_best[2].tolist() == [1] and gpu_best[1].tolist() == [1]


@pytest.mark.parametrize("loc", LOCATIONS)
def test_emitting_arc_beats_epsilon_arc_of_the_same_state(torch_cuda, loc):
    """An epsilon arc and an emitting arc of one state reach state 1 at equal cost: the emitting arc wins although
    the caller numbered the epsilon arc first."""
    g = graph([0, 3, 3], [1, 0, 1], [0, 1, 1], [0, 0, 0], [1.0, 0.0, 1.0])
    L = np.zeros((1, 1), np.float32)
    tables, _, _ = both(torch_cuda, g, L, 1.0e30, 0, loc)
    assert tables[0][0] == (np.float32(0.0), 1)
    assert tables[0][1] == (np.float32(1.0), 2)


@pytest.mark.parametrize("loc", LOCATIONS)
def test_start_token_loses_a_tie_to_a_real_arc_and_the_walk_is_bounded(torch_cuda, loc):
    """Zero-weight epsilon cycle through the start state: the closure settles (no cost ever drops), the start
    token ties with the arc that returns to the start state and loses (its pseudo arc sorts last), and the
    predecessors then form a cycle, which the walk must leave with the divergence status, as the checker does."""
    g = graph([0, 2, 3], [1, 1, 0], [0, 1, 0], [0, 7, 0], [0.0, 0.5, 0.0])
    L = np.zeros((2, 1), np.float32)
    Ld = torch_cuda.tensor(L, dtype=torch_cuda.float32, device="cuda").unsqueeze(0).contiguous()
    dec = GH.GpuDecoder(g, 1, 10.0, 0, max_frames=4, hash_log2=8, table_location=loc)
    try:
        orc = OracleChannel(OracleGraph.from_graph(g), 10.0, 0)
        dec.reset()
        assert orc.reset() == 0
        st, co, ar = orc.tokens()
        assert st.tolist() == [0, 1] and co.tolist() == [0.0, 0.0] and ar.tolist() == [2, 0]   # not the start token's -1
        GH.assert_tables_equal(dec.tokens(0), orc.tokens(), "after the start")
        orc_best = orc.best_path(False)
        assert orc_best[0] == 2   # the checker's walk meets the predecessor cycle
        assert dec.best(0)[0] == B.CBD_E_EPS_DIVERGED
        # decoding itself goes on normally on both sides
        dec.advance(Ld, 0, 1); orc.advance(L[:1])
        GH.assert_tables_equal(dec.tokens(0), orc.tokens(), "frame 0")
        GH.assert_best_equal(dec.best(0), orc.best_path(False), "after frame 0")
    finally:
        dec.close()


@pytest.mark.parametrize("loc", LOCATIONS)
def test_zero_weight_epsilon_cycle_away_from_the_start(torch_cuda, loc):
    """A zero-weight epsilon cycle between states 1 and 2, entered by an emitting arc: the closure ends, the
    entered state keeps its emitting arc (an emitting arc's source, state 0, is lower), and results match."""
    g = graph([0, 1, 3, 4], [1, 2, 0, 1], [1, 0, 1, 0], [3, 0, 4, 0], [0.25, 0.0, 0.5, 0.0])
    L = np.zeros((4, 1), np.float32)
    tables, gpu_best, orc_best = both(torch_cuda, g, L, 10.0, 0, loc)
    assert tables[0][1] == (np.float32(0.25), 0) and tables[0][2] == (np.float32(0.25), 1)
    assert orc_best[0] == 0 and gpu_best[0] == 0


@pytest.mark.parametrize("loc", LOCATIONS)
def test_token_on_the_beam_edge_and_one_ulp_above(torch_cuda, loc):
    """Beam 4: a token with cost - best == 4 survives the prune and is expanded, one with the next fp32 above
    is not; the same at the frame cutoff (candidate - minimum)."""
    beam = np.float32(4.0)
    above = np.nextafter(beam, np.float32(np.inf), dtype=np.float32)
    # state 0 -> 1 (w 0), 2 (w 4.0: on the edge), 3 (w above: dropped by the frame cutoff)
    # states 1, 2, 3 each go on to their own state 4, 5, 6 at weight 0
    # frame 1: state 1 -> 7 with weight 0 and 1 -> 8 with weight `above` (cut), 2 -> 9 weight 0 (kept: 4 - 0 == beam)
    g = graph([0, 3, 5, 6, 7, 7, 7, 7, 7, 7, 7], [1, 2, 3, 7, 8, 9, 6], [1, 1, 1, 1, 1, 1, 1], [0] * 7,
              [0.0, beam, above, 0.0, above, 0.0, 0.0])
    L = np.zeros((2, 1), np.float32)
    tables, _, _ = both(torch_cuda, g, L, float(beam), 0, loc)
    assert sorted(tables[0]) == [1, 2]          # state 3 fell to the cutoff by one ulp
    assert sorted(tables[1]) == [7, 9]          # 8 is one ulp outside; 9 descends from the token on the edge


@pytest.mark.parametrize("loc", LOCATIONS)
@pytest.mark.parametrize("max_active", [3, 16])
def test_all_costs_equal_with_max_active_below_the_table_size(torch_cuda, loc, max_active):
    """Forty tokens of bit-equal cost and max_active 3: bin 0 alone exceeds the limit, so all of it stays
    (max_active 16 likewise).  Both sides must keep all forty and expand them."""
    n = 40
    row = [0, n] + [n + 1 + i for i in range(n)] + [2 * n] * n
    dst = list(range(1, n + 1)) + list(range(n + 1, 2 * n + 1))
    g = graph(row, dst, [1] * (2 * n), [0] * (2 * n), [0.5] * (2 * n))
    L = np.zeros((2, 1), np.float32)
    tables, _, _ = both(torch_cuda, g, L, 8.0, max_active, loc)
    assert len(tables[0]) == n and len(tables[1]) == n
    assert all(a == s - 1 for s, (c, a) in tables[0].items())


@pytest.mark.parametrize("loc", LOCATIONS)
def test_histogram_cut_drops_whole_bins(torch_cuda, loc):
    """max_active 3 over costs 0, 1, 1.01, 1.02, 5 (beam 8: bin width 1/32): the bin holding the three tokens near
    1 does not fit, so only the best token is expanded in the next frame."""
    costs = [0.0, 1.0, 1.01, 1.02, 5.0]
    n = len(costs)
    row = [0, n] + [n + 1 + i for i in range(n)] + [2 * n] * n
    dst = list(range(1, n + 1)) + list(range(n + 1, 2 * n + 1))
    g = graph(row, dst, [1] * (2 * n), [0] * (2 * n), costs + [0.0] * n)
    L = np.zeros((2, 1), np.float32)
    tables, _, _ = both(torch_cuda, g, L, 8.0, 3, loc)
    assert len(tables[0]) == n and sorted(tables[1]) == [n + 1]


@pytest.mark.parametrize("loc", LOCATIONS)
def test_signed_zeros(torch_cuda, loc):
    """Weights, offsets and log-likelihoods of -0.0: costs compare by value (+0 == -0), ties then go to the arc
    order, and the returned cost equals the checker's."""
    nz = np.float32(-0.0)
    # two arcs into state 1: a0 with weight -0.0 and a1 with weight +0.0 -> equal costs, a0 wins;
    # state 1 -> 2 through an epsilon arc of weight -0.0 and an emitting arc
    g = graph([0, 2, 4, 4], [1, 1, 2, 2], [1, 2, 0, 1], [1, 2, 3, 4], [nz, 0.0, nz, nz], num_pdfs=2)
    L = np.array([[nz, 0.0], [0.0, nz]], np.float32)
    for ctx, off in ((None, 0.0), ([0, 1, 2, 3], float(nz)), ([1], -0.0)):
        tables, gpu_best, orc_best = both(torch_cuda, g, L, 6.0, 0, loc, ctx=ctx, offset=off)
        assert tables[0][1][1] == 0 and tables[0][2][1] == 2
        assert gpu_best[3] == orc_best[3] == 0.0


@pytest.mark.parametrize("loc", LOCATIONS)
def test_equal_keys_from_two_epsilon_parents(torch_cuda, loc):
    """Two epsilon arcs of different states reach state 3 at bit-equal cost in the closure, and a boosted
    epsilon arc ties an unboosted one: the lower source state wins."""
    # 0 -> 1 (emit, w 1), 0 -> 2 (emit, w 1); 1 -eps(0.5)-> 3, 2 -eps(0.5)-> 3; 3 -> 4 (emit)
    g = graph([0, 2, 3, 4, 5, 5], [1, 2, 3, 3, 4], [1, 1, 0, 0, 1], [0, 0, 5, 6, 0], [1.0, 1.0, 0.5, 0.5, 0.0])
    L = np.zeros((2, 1), np.float32)
    tables, gpu_best, _ = both(torch_cuda, g, L, 10.0, 0, loc)
    assert tables[0][3] == (np.float32(1.5), 2)
    assert gpu_best[1].tolist() == [5]
    # with arc 3 boosted by -0.25 and arc 2's weight lowered to match: still a tie, still the lower source
    g2 = graph([0, 2, 3, 4, 5, 5], [1, 2, 3, 3, 4], [1, 1, 0, 0, 1], [0, 0, 5, 6, 0], [1.0, 1.0, 0.25, 0.5, 0.0])
    tables, gpu_best, _ = both(torch_cuda, g2, L, 10.0, 0, loc, ctx=[3], offset=-0.25)
    assert tables[0][3] == (np.float32(1.25), 2)


@pytest.mark.parametrize("loc", LOCATIONS)
def test_final_cost_ties_go_to_the_arc_order(torch_cuda, loc):
    """Two tokens whose cost + final cost are bit-equal: the best path ends in the one with the earlier arc."""
    g = graph([0, 2, 2, 2], [2, 1], [1, 1], [8, 9], [1.0, 0.5], finals=[0.0, 1.0, 0.5])
    L = np.zeros((1, 1), np.float32)
    tables, gpu_best, orc_best = both(torch_cuda, g, L, 10.0, 0, loc, use_final=True)
    assert gpu_best[3] == 1.5 and gpu_best[2].tolist() == [0] and gpu_best[1].tolist() == [8]
