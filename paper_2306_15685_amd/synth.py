"""Seeded synthetic inputs: decoding graphs, log-likelihoods, biasing contexts.

This module only draws random numbers and lays them out.  It holds none of the
decoder's arithmetic, imports neither the HIP binding nor the CPU checker, and is
the one piece both of them are fed from, so that they always see the same bytes.

The inputs stand in for the paper's online workloads (Sec. 5: 2K clients, 30 ms
frames after one-third subsampling, biasing lists of a few hundred up to 1013
entities, Table 2): random HCLG-like transducers, log-softmax Gaussian scores and
per-channel lists of word-arc indices that lie along connected walks, like the
arc sets Algorithm 1 returns for word sequences.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 230615685

FRAME_SHIFT_S = 0.030  # Sec. 5.2: 10 ms features, one-third frame subsampling


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration (sizes and decoder settings)."""

    name: str
    num_states: int
    num_pdfs: int
    num_words: int
    eps_prob: float
    channels: int
    frames: int  # frames per segment (utterance)
    chunk: int  # frames handed to one advance call
    beam: float
    max_active: int  # 0 = off
    sigma: float  # standard deviation of the pre-softmax scores
    ctx_min: int  # context size range (arcs)
    ctx_max: int
    offset_lo: float  # offset range; lo == hi means fixed
    offset_hi: float
    segments: int = 1  # utterances per channel, each with a fresh context
    ctx_walks: bool = True  # arcs along connected walks (False: independent word arcs)
    lookup_mode: int = 0  # 0 sorted list, 1 hashed bitmap + confirm
    partial_every_chunk: bool = False
    mean_degree: float = 3.0
    word_frac: float = 0.25
    word_period: int = 0  # > 0: word labels every word_period arcs (see make_graph); contexts are word sequences
    config_id: int = 0
    graph_id: int = -1  # seed stream of the decoding graph (-1: config_id); workloads that share a graph share it


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 2_000, 200, 600, 0.15, 1, 100, 100, 10.0, 0, 3.0,
                     20, 20, -3.0, -3.0, ctx_walks=False, config_id=0),
    "medium": Workload("medium", 1_000_000, 3_000, 20_000, 0.10, 32, 333, 333, 13.0, 7_000, 4.0,
                       50, 50, -5.0, -5.0, config_id=1),
    "large": Workload("large", 10_000_000, 6_000, 200_000, 0.10, 256, 500, 50, 15.0, 10_000, 4.0,
                      100, 500, -5.0, -5.0, partial_every_chunk=True, lookup_mode=1, config_id=2),
    "dynamic": Workload("dynamic", 10_000_000, 6_000, 200_000, 0.10, 512, 100, 100, 15.0, 10_000, 4.0,
                        10, 1_000, -8.0, -2.0, segments=20, lookup_mode=1, config_id=3, graph_id=2),
    "stress": Workload("stress", 10_000_000, 6_000, 200_000, 0.10, 2_048, 300, 50, 16.0, 20_000, 4.0,
                       1_000, 1_000, -5.0, -5.0, lookup_mode=1, config_id=4, graph_id=2),
    # contexts given as word sequences and turned into arc lists by Algorithm 1 (Sec. 4.1); the graph keeps its
    # word labels four arcs apart, as a composed decoding graph does, so that the algorithm's search stays local
    "words": Workload("words", 2_000_000, 4_000, 50_000, 0.10, 128, 300, 50, 15.0, 10_000, 4.0,
                      100, 500, -5.0, -5.0, partial_every_chunk=True, lookup_mode=1, word_period=4, config_id=6),
    # second workload: lexicon loop over end-to-end units (dense token activity, a 20,000-arc hub row,
    # max-active pruning engaged); contexts are word-end arcs (unigram boosting)
    "e2e": Workload("e2e", 0, 96, 20_000, 0.0, 64, 200, 50, 10.0, 2_500, 2.0,
                    100, 300, -2.0, -2.0, ctx_walks=False, lookup_mode=1, partial_every_chunk=True, config_id=5),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller test variants)."""
    return replace(w, **kw)


def _rng(*stream: int) -> np.random.Generator:
    """Counter-based generator keyed by (base seed, stream ids)."""
    ss = np.random.SeedSequence([BASE_SEED, *[int(x) & 0xFFFFFFFF for x in stream]])
    return np.random.Generator(np.random.Philox(ss))


@dataclass
class Graph:
    """A transducer in the caller's arc numbering: plain CSR rows over states.

    Arc ``a`` of state ``s`` has ``row_offsets[s] <= a < row_offsets[s+1]``.
    ``ilabel`` 0 marks an epsilon-input arc, otherwise it is pdf id + 1.
    ``olabel`` 0 means no word.  ``weight`` is a cost (-log probability), fp32.
    """

    num_states: int
    num_arcs: int
    num_pdfs: int
    num_words: int
    start_state: int
    row_offsets: np.ndarray  # int32 [S+1]
    dst: np.ndarray  # int32 [A]
    ilabel: np.ndarray  # int32 [A]
    olabel: np.ndarray  # int32 [A]
    weight: np.ndarray  # float32 [A]
    final_cost: Optional[np.ndarray] = None  # float32 [S] or None (all final, cost 0)
    _src: Optional[np.ndarray] = field(default=None, repr=False)

    @property
    def src(self) -> np.ndarray:
        if self._src is None:
            deg = np.diff(self.row_offsets.astype(np.int64))
            self._src = np.repeat(np.arange(self.num_states, dtype=np.int32), deg)
        return self._src


def make_graph(num_states: int, num_pdfs: int, num_words: int, eps_prob: float,
               seed_stream: Tuple[int, ...] = (0,), mean_degree: float = 3.0,
               word_frac: float = 0.25, with_finals: bool = False,
               self_loop_frac: float = 0.0, word_period: int = 0) -> Graph:
    """Random HCLG-like graph.

    Out-degree is Poisson(mean_degree) clipped to at least 1.  Each arc is an
    epsilon-input arc with probability ``eps_prob``; such arcs always lead to a
    higher-numbered state, so the epsilon subgraph is acyclic (the last state has
    none).  Emitting arcs go to a uniformly random state and carry a uniformly
    random pdf.  A fraction ``word_frac`` of all arcs carry a uniformly random
    word.  Weights are -ln U(0.05, 1).  Epsilon and emitting arcs are interleaved
    within a row, in no particular order.

    With ``word_period`` p > 0 the words sit as they do in a composed decoding graph, p arcs apart: state s is at
    position s mod p inside a word, every arc leads to a state at the next position, and exactly the arcs that
    close a word (into position 0) carry a word label, so ``word_frac`` is 1/p.  From any state only a few dozen
    states can be reached without crossing a word label, which is what Algorithm 1's search relies on.
    """
    S = int(num_states)
    rng = _rng(1, *seed_stream)
    deg = np.maximum(rng.poisson(mean_degree, S), 1).astype(np.int64)
    row = np.zeros(S + 1, dtype=np.int64)
    np.cumsum(deg, out=row[1:])
    A = int(row[-1])
    assert A < 2**31 - 1
    src = np.repeat(np.arange(S, dtype=np.int64), deg)
    is_eps = rng.random(A) < eps_prob
    is_eps &= src < S - 1
    dst = rng.integers(0, S, A, dtype=np.int64)
    u = rng.random(A)
    eps_dst = src + 1 + np.floor(u * (S - 1 - src)).astype(np.int64)
    eps_dst = np.minimum(eps_dst, S - 1)
    dst = np.where(is_eps, eps_dst, dst)
    if word_period > 0:
        p = int(word_period)
        want = (src + 1) % p                       # position of the destination inside its word
        moved = dst - (dst % p) + want
        moved = np.where(is_eps & (moved <= src), moved + p, moved)   # epsilon arcs keep leading upwards
        fits = moved < S
        is_eps &= fits                              # (an arc pushed past the last state becomes an emitting arc
        dst = np.where(fits, moved, want)           #  into the first block of states)
    if self_loop_frac > 0.0:
        loop = (~is_eps) & (rng.random(A) < self_loop_frac)
        dst = np.where(loop, src, dst)
    pdf = rng.integers(0, num_pdfs, A, dtype=np.int64)
    ilabel = np.where(is_eps, 0, pdf + 1)
    word = rng.integers(1, num_words + 1, A, dtype=np.int64)
    olabel = np.where(rng.random(A) < word_frac, word, 0)
    if word_period > 0:
        olabel = np.where(dst % int(word_period) == 0, word, 0)
    weight = (-np.log(rng.uniform(0.05, 1.0, A))).astype(np.float32)
    final = None
    if with_finals:
        final = (-np.log(rng.uniform(0.05, 1.0, S))).astype(np.float32)
    return Graph(S, A, int(num_pdfs), int(num_words), 0, row.astype(np.int32),
                 dst.astype(np.int32), ilabel.astype(np.int32), olabel.astype(np.int32),
                 weight, final, src.astype(np.int32))


def make_lexicon_graph(num_units: int, num_words: int, seed_stream: Tuple[int, ...] = (0,),
                       min_len: int = 2, max_len: int = 6) -> Graph:
    """Lexicon loop over end-to-end model units (Sec. 6: decoding with characters or subwords
    instead of words' HMM states).

    State 0 is the word-boundary hub.  Every word is a chain of `min_len..max_len` unit states
    entered from the hub by an emitting arc on its first unit; each chain state has a self-loop
    on its own unit (the unit lasts several frames) and an arc to the next state on the next
    unit; the last state returns to the hub through an epsilon-input arc that carries the word
    label.  So the hub row has `num_words` arcs, chains are dense in tokens, and the epsilon
    arcs alone form no cycle.  Unit u is pdf u; weights are -ln U(0.05, 1).
    """
    rng = _rng(6, *seed_stream)
    lens = rng.integers(min_len, max_len + 1, num_words)
    units = [rng.integers(0, num_units, int(n)) for n in lens]
    first_state = np.zeros(num_words, dtype=np.int64)
    nxt = 1
    for w in range(num_words):
        first_state[w] = nxt
        nxt += int(lens[w])
    S = nxt
    row, dst, il, ol = [0], [], [], []
    for w in range(num_words):                      # hub row
        dst.append(int(first_state[w])); il.append(int(units[w][0]) + 1); ol.append(0)
    row.append(len(dst))
    for w in range(num_words):
        for k in range(int(lens[w])):
            s = int(first_state[w]) + k
            dst.append(s); il.append(int(units[w][k]) + 1); ol.append(0)          # self-loop
            if k + 1 < lens[w]:
                dst.append(s + 1); il.append(int(units[w][k + 1]) + 1); ol.append(0)
            else:
                dst.append(0); il.append(0); ol.append(w + 1)                        # word end, back to the hub
            row.append(len(dst))
    A = len(dst)
    weight = (-np.log(rng.uniform(0.05, 1.0, A))).astype(np.float32)
    return Graph(S, A, int(num_units), int(num_words), 0, np.array(row, np.int32), np.array(dst, np.int32),
                 np.array(il, np.int32), np.array(ol, np.int32), weight, None)


def graph_for(w: Workload, with_finals: bool = False) -> Graph:
    """The workload's decoding graph.  Dynamic and Stress decode over Large's 10M-state graph (same seed stream)."""
    gid = w.graph_id if w.graph_id >= 0 else w.config_id
    if w.name.startswith("e2e"):
        return make_lexicon_graph(w.num_pdfs, w.num_words, seed_stream=(gid,))
    return make_graph(w.num_states, w.num_pdfs, w.num_words, w.eps_prob,
                      seed_stream=(gid,), mean_degree=w.mean_degree,
                      word_frac=w.word_frac, with_finals=with_finals, word_period=w.word_period)


def make_loglikes(channels: int, frames: int, num_pdfs: int, sigma: float,
                  seed_stream: Tuple[int, ...] = (0,), device: str = "cpu"):
    """fp32 tensor [channels, frames, num_pdfs]: log_softmax over pdfs of N(0, sigma^2).

    Drawn with torch's generator for ``device`` (the streams differ between
    devices; whoever consumes the tensor sees the same bytes either way).
    """
    import torch

    seed = int(np.random.SeedSequence([BASE_SEED, 2, *seed_stream]).generate_state(1, np.uint64)[0] >> 1)
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    x = torch.randn((channels, frames, num_pdfs), generator=g, device=device, dtype=torch.float32)
    x.mul_(sigma)
    return torch.log_softmax(x, dim=-1)


def word_arcs(g: Graph) -> np.ndarray:
    return np.nonzero(g.olabel != 0)[0].astype(np.int32)


def context_random_word_arcs(g: Graph, k: int, seed_stream: Tuple[int, ...]) -> np.ndarray:
    """k distinct word-arc indices, uniform over the graph's word arcs."""
    rng = _rng(3, *seed_stream)
    wa = word_arcs(g)
    k = min(k, wa.size)
    return rng.choice(wa, size=k, replace=False).astype(np.int32)


def context_walks(g: Graph, n_walks: int, words_per_walk: int, seed_stream: Tuple[int, ...],
                  rng: Optional[np.random.Generator] = None) -> np.ndarray:
    """Word arcs crossed by random walks through the graph.

    Each walk starts at a uniformly random state and follows uniformly random
    out-arcs until it has crossed ``words_per_walk`` word arcs; the word arcs it
    crossed are returned (all walks concatenated, duplicates removed, any order).
    The arcs of one walk lie on a connected path, like the arc sets found for a
    word sequence (Algorithm 1).
    """
    if rng is None:
        rng = _rng(4, *seed_stream)
    row = g.row_offsets.astype(np.int64)
    cur = rng.integers(0, g.num_states, n_walks, dtype=np.int64)
    need = np.full(n_walks, words_per_walk, dtype=np.int64)
    out: List[np.ndarray] = []
    for _ in range(words_per_walk * 64):
        live = need > 0
        if not live.any():
            break
        s = cur[live]
        deg = row[s + 1] - row[s]
        ok = deg > 0
        pick = row[s] + np.floor(rng.random(s.size) * np.maximum(deg, 1)).astype(np.int64)
        pick = np.minimum(pick, row[s + 1] - 1)
        pick = np.where(ok, pick, 0)
        isw = ok & (g.olabel[pick] != 0)
        out.append(pick[isw].astype(np.int32))
        nxt = np.where(ok, g.dst[pick].astype(np.int64), rng.integers(0, g.num_states, s.size))
        cur[live] = nxt
        nl = need[live]
        nl -= isw.astype(np.int64)
        need[live] = nl
    if not out:
        return np.zeros(0, dtype=np.int32)
    return np.unique(np.concatenate(out)).astype(np.int32)


def make_contexts(w: Workload, g: Graph, segment: int = 0,
                  channels: Optional[int] = None) -> Tuple[List[np.ndarray], np.ndarray]:
    """Per-channel arc-index lists and offsets for one segment of a workload.

    Lists are returned shuffled (the decoder treats them as sets).  Sizes are
    drawn uniformly from [ctx_min, ctx_max]; with ``ctx_walks`` a list is built
    from size/10 walks of 10 word arcs each and cut to size.
    """
    C = w.channels if channels is None else channels
    lists: List[np.ndarray] = []
    offs = np.zeros(C, dtype=np.float32)
    for c in range(C):
        rng = _rng(5, w.config_id, c, segment)
        k = int(rng.integers(w.ctx_min, w.ctx_max + 1))
        if w.offset_lo == w.offset_hi:
            offs[c] = np.float32(w.offset_lo)
        else:
            offs[c] = np.float32(rng.uniform(w.offset_lo, w.offset_hi))
        if w.ctx_walks:
            n_walks = max(1, (k + 9) // 10)
            arcs = context_walks(g, n_walks + 1, 10, (), rng=rng)
            if arcs.size > k:
                arcs = arcs[rng.permutation(arcs.size)[:k]]
        else:
            wa = word_arcs(g)
            arcs = rng.choice(wa, size=min(k, wa.size), replace=False).astype(np.int32)
        arcs = arcs[rng.permutation(arcs.size)].astype(np.int32)
        lists.append(arcs)
    return lists, offs


def word_sequences_on_walks(g: Graph, n_seq: int, words_per_seq: int, rng: np.random.Generator) -> List[List[int]]:
    """Word sequences that occur in the graph: the output labels along random walks.

    Each walk starts at a uniformly random state and follows uniformly random out-arcs until it has crossed
    ``words_per_seq`` word arcs (or 64 x that many arcs); the words it crossed, in order, are one sequence.
    This is input drawing only: which arcs a sequence selects is Algorithm 1's business.
    """
    row = g.row_offsets.astype(np.int64)
    cur = rng.integers(0, g.num_states, n_seq, dtype=np.int64)
    seqs: List[List[int]] = [[] for _ in range(n_seq)]
    need = np.full(n_seq, words_per_seq, dtype=np.int64)
    for _ in range(words_per_seq * 64):
        live = np.nonzero(need > 0)[0]
        if live.size == 0:
            break
        s = cur[live]
        deg = row[s + 1] - row[s]
        ok = deg > 0
        pick = row[s] + np.floor(rng.random(s.size) * np.maximum(deg, 1)).astype(np.int64)
        pick = np.where(ok, np.minimum(pick, row[s + 1] - 1), 0)
        word = np.where(ok, g.olabel[pick], 0)
        for i in np.nonzero(word != 0)[0]:
            seqs[int(live[i])].append(int(word[i]))
        need[live] -= (word != 0).astype(np.int64)
        cur[live] = np.where(ok, g.dst[pick].astype(np.int64), rng.integers(0, g.num_states, s.size))
    return [q for q in seqs if q]


def make_context_sequences(w: Workload, g: Graph, segment: int = 0,
                           channels: Optional[int] = None) -> Tuple[List[List[List[int]]], np.ndarray]:
    """Per-channel biasing lists as WORD SEQUENCES (the form a user supplies, Sec. 4.1) and offsets.

    A channel's list holds sequences of 1 to 3 words; their number is drawn so that the arc lists Algorithm 1 makes
    of them come out near the workload's context sizes (a word labels about word arcs / vocabulary arcs, and every
    arc of a sequence's first word is selected).  Offsets are drawn as in make_contexts.
    """
    C = w.channels if channels is None else channels
    per_word = max(1.0, float(np.count_nonzero(g.olabel)) / max(1, g.num_words))
    out: List[List[List[int]]] = []
    offs = np.zeros(C, dtype=np.float32)
    for c in range(C):
        rng = _rng(6, w.config_id, c, segment)
        k = int(rng.integers(w.ctx_min, w.ctx_max + 1))
        if w.offset_lo == w.offset_hi:
            offs[c] = np.float32(w.offset_lo)
        else:
            offs[c] = np.float32(rng.uniform(w.offset_lo, w.offset_hi))
        n_seq = max(1, int(round(k / (per_word + 2.0))))
        seqs: List[List[int]] = []
        for n_words in (3, 2, 1):
            seqs += word_sequences_on_walks(g, (n_seq + n_words - 1) // 3, n_words, rng)
        out.append(seqs)
    return out, offs
