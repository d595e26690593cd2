"""Independent checks used to pin the CPU checker (and, through it, the HIP path).

Nothing here calls the decoder's own routines to produce an expected value:
paths are enumerated by brute force, costs are re-accumulated along returned
paths, frame tables are verified as supported fixed points of the recursion,
and the infinite-beam optimum comes from scipy's shortest-path routine on the
trellis product graph.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32


def f32(x) -> np.float32:
    return np.float32(x)


def biased_w(g, a: int, ctx: set, offset) -> np.float32:
    """Sec. 4.1: boosted weight = original weight + discount, for listed arcs only."""
    w = F32(g.weight[a])
    if a in ctx:
        w = F32(w + F32(offset))
    return w


def arc_order_key(g, a: int) -> Tuple[int, int, int]:
    """Tie-break order of arcs: source state, emitting before epsilon, arc index.
    The start token's pseudo arc (-1) sorts after every real arc."""
    if a < 0:
        return (1 << 40, 0, 0)
    return (int(g.src[a]), int(g.ilabel[a] == 0), int(a))


def key_of(g, cost, a: int):
    return (float(cost), *arc_order_key(g, a))


def enumerate_paths(g, L: np.ndarray, ctx: Iterable[int], offset: float,
                    use_final: bool = False) -> List[Tuple[np.float32, Tuple[int, ...]]]:
    """Every path from the start state that consumes exactly len(L) frames
    (epsilon arcs consume none), with its fp32 cost accumulated in path order."""
    ctx = set(int(x) for x in ctx)
    T = L.shape[0]
    out: List[Tuple[np.float32, Tuple[int, ...]]] = []
    row = g.row_offsets

    def rec(s: int, t: int, c: np.float32, path: Tuple[int, ...]):
        if t == T:
            cc = c
            if use_final and g.final_cost is not None:
                cc = F32(c + F32(g.final_cost[s]))
            out.append((cc, path))
        for a in range(int(row[s]), int(row[s + 1])):
            il = int(g.ilabel[a])
            w = biased_w(g, a, ctx, offset)
            if il == 0:
                rec(int(g.dst[a]), t, F32(c + w), path + (a,))
            elif t < T:
                cand = F32(F32(c + w) - F32(L[t, il - 1]))
                rec(int(g.dst[a]), t + 1, cand, path + (a,))

    rec(int(g.start_state), 0, F32(0.0), ())
    return out


def rescore_path(g, arcs: Sequence[int], L: np.ndarray, ctx_at_frame, offset_at_frame,
                 use_final: bool = False):
    """Walk a returned arc path: check it is connected from the start state and
    re-accumulate its cost in fp32 in path order.

    ctx_at_frame(t) -> set of listed arcs in force while frame t is decoded
    (t = number of emitting arcs already taken; epsilon arcs after the last frame
    use the last frame's context).  Returns (cost, frames consumed, words).
    """
    s = int(g.start_state)
    c = F32(0.0)
    t = 0
    words = []
    T = L.shape[0]
    for a in arcs:
        a = int(a)
        assert g.row_offsets[s] <= a < g.row_offsets[s + 1], "path not connected"
        il = int(g.ilabel[a])
        # an epsilon arc taken after frame t-1 belongs to that frame's closure
        # (t == 0: the closure done at reset, frame index -1)
        tt = t if il != 0 else t - 1
        w = biased_w(g, a, ctx_at_frame(tt), offset_at_frame(tt))
        if il == 0:
            c = F32(c + w)
        else:
            assert t < T
            c = F32(F32(c + w) - F32(L[t, il - 1]))
            t += 1
        if g.olabel[a] != 0:
            words.append(int(g.olabel[a]))
        s = int(g.dst[a])
    if use_final and g.final_cost is not None:
        c = F32(c + F32(g.final_cost[s]))
    return c, t, words, s


def incoming_index(g):
    """dst state -> list of arcs entering it."""
    order = np.argsort(g.dst, kind="stable")
    counts = np.bincount(g.dst, minlength=g.num_states)
    offs = np.zeros(g.num_states + 1, dtype=np.int64)
    np.cumsum(counts, out=offs[1:])
    return order, offs


def check_frame_table(g, inc, prev: Dict[int, Tuple[np.float32, int]], active: set,
                      cur: Dict[int, Tuple[np.float32, int]], Lrow: Optional[np.ndarray],
                      ctx: set, offset: float, beam: float, m_reported: Optional[float] = None):
    """Verify that `cur` is the supported fixed point of one frame of the recursion.

    prev/cur map state -> (cost, arc).  `active` = states of prev that survived
    pruning.  Lrow None means the reset step (cur must be the closure of the
    start token).  Raises AssertionError with a description on any violation.
    """
    order, offs = inc
    beam = F32(beam)

    def cand_emit(a):
        s = int(g.src[a])
        c = prev[s][0]
        return F32(F32(c + biased_w(g, a, ctx, offset)) - F32(Lrow[int(g.ilabel[a]) - 1]))

    def cand_eps(a):
        s = int(g.src[a])
        return F32(cur[s][0] + biased_w(g, a, ctx, offset))

    # emission minimum m over all candidates from active tokens
    if Lrow is None:
        m = F32(0.0)
    else:
        m = None
        for s in active:
            for a in range(int(g.row_offsets[s]), int(g.row_offsets[s + 1])):
                if g.ilabel[a] != 0:
                    c = cand_emit(a)
                    if m is None or c < m:
                        m = c
        if m is None:
            assert len(cur) == 0, "no candidates but table not empty"
            return None
    if m_reported is not None:
        assert F32(m_reported) == m, f"emission minimum {m_reported} != {m}"

    def within(c):
        return not (F32(c - m) > beam)

    # (i) support, (ii) beam
    for d, (c, a) in cur.items():
        assert within(c), f"state {d} cost {c} outside beam of m={m}"
        if a < 0:
            assert Lrow is None and d == g.start_state and c == F32(0.0), "bad start token"
            continue
        assert int(g.dst[a]) == d, f"state {d}: arc {a} does not enter it"
        if g.ilabel[a] == 0:
            assert int(g.src[a]) in cur, f"state {d}: epsilon predecessor missing"
            assert cand_eps(a) == c, f"state {d}: cost {c} != eps candidate {cand_eps(a)}"
        else:
            assert Lrow is not None and int(g.src[a]) in active, f"state {d}: emitting predecessor not active"
            assert cand_emit(a) == c, f"state {d}: cost {c} != emitting candidate {cand_emit(a)}"
    # (iii) minimality, (iv) completeness: look at every arc that could feed any state
    feeders: Dict[int, List[Tuple]] = {}
    if Lrow is not None:
        for s in active:
            for a in range(int(g.row_offsets[s]), int(g.row_offsets[s + 1])):
                if g.ilabel[a] != 0:
                    c = cand_emit(a)
                    if within(c):
                        feeders.setdefault(int(g.dst[a]), []).append(key_of(g, c, a))
    else:
        feeders.setdefault(int(g.start_state), []).append(key_of(g, F32(0.0), -1))
    for s in cur:
        for a in range(int(g.row_offsets[s]), int(g.row_offsets[s + 1])):
            if g.ilabel[a] == 0:
                c = cand_eps(a)
                if within(c):
                    feeders.setdefault(int(g.dst[a]), []).append(key_of(g, c, a))
    assert set(feeders.keys()) == set(cur.keys()), (
        f"table states differ from reachable states: missing {set(feeders) - set(cur)}, "
        f"extra {set(cur) - set(feeders)}")
    for d, ks in feeders.items():
        c, a = cur[d]
        assert min(ks) == key_of(g, c, a), f"state {d}: key {key_of(g, c, a)} is not the minimum {min(ks)}"
    return m


def table_dict(states, costs, arcs) -> Dict[int, Tuple[np.float32, int]]:
    return {int(s): (F32(c), int(a)) for s, c, a in zip(states, costs, arcs)}


def trellis_shortest(g, L: np.ndarray, ctx: Iterable[int], offset: float) -> float:
    """Infinite-beam optimum by scipy's Bellman-Ford on the (frames+1) x states
    trellis in fp64: emitting arcs go one layer down, epsilon arcs stay in a layer."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import bellman_ford

    ctx = np.fromiter((int(x) for x in ctx), dtype=np.int64)
    S, T = g.num_states, L.shape[0]
    w = g.weight.astype(np.float64).copy()
    if ctx.size:
        w[np.unique(ctx)] = (g.weight[np.unique(ctx)] + F32(offset)).astype(np.float64)
    src = g.src.astype(np.int64)
    dst = g.dst.astype(np.int64)
    emit = g.ilabel != 0
    rows, cols, vals = [], [], []
    for t in range(T + 1):
        e = ~emit
        rows.append(t * S + src[e]); cols.append(t * S + dst[e]); vals.append(w[e])
        if t < T:
            rows.append(t * S + src[emit]); cols.append((t + 1) * S + dst[emit])
            vals.append(w[emit] - L[t, g.ilabel[emit] - 1].astype(np.float64))
    rows = np.concatenate(rows); cols = np.concatenate(cols); vals = np.concatenate(vals)
    # parallel arcs: keep the cheapest; shift so that explicit zeros are not dropped
    key = rows * ((T + 1) * S) + cols
    o = np.lexsort((vals, key))
    key, rows, cols, vals = key[o], rows[o], cols[o], vals[o]
    first = np.ones(key.size, dtype=bool)
    first[1:] = key[1:] != key[:-1]
    rows, cols, vals = rows[first], cols[first], vals[first]
    vals = np.where(vals == 0.0, 1e-300, vals)
    n = (T + 1) * S
    mat = csr_matrix((vals, (rows, cols)), shape=(n, n))
    dist = bellman_ford(mat, directed=True, indices=int(g.start_state))
    return float(dist[T * S:].min())
