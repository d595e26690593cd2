"""Pins of the Algorithm 1 checker (word sequence -> arcs to boost) against brute force."""
import itertools

import numpy as np
import pytest

from paper_2306_15685_amd import synth
from oracle import arcs_for_sequence, arcs_for_sequences


def dag(seed, S=9, W=3, word_frac=0.6, deg=2.2):
    """Small acyclic graph (every arc leads to a higher state) with few words, so that all paths can
    be listed."""
    rng = np.random.default_rng(seed)
    row, dst, ol = [0], [], []
    for s in range(S):
        n = 0 if s == S - 1 else max(1, rng.poisson(deg))
        for _ in range(n):
            dst.append(int(rng.integers(s + 1, S)))
            ol.append(int(rng.integers(1, W + 1)) if rng.random() < word_frac else 0)
        row.append(len(dst))
    A = len(dst)
    return synth.Graph(S, A, 2, W, 0, np.array(row, np.int32), np.array(dst, np.int32),
                       np.ones(A, np.int32), np.array(ol, np.int32), np.ones(A, np.float32))


def all_paths(g):
    """Every path (tuple of arcs) of the acyclic graph, from every state."""
    out = []

    def rec(s, path):
        for a in range(int(g.row_offsets[s]), int(g.row_offsets[s + 1])):
            p = path + (a,)
            out.append(p)
            rec(int(g.dst[a]), p)

    for s in range(g.num_states):
        rec(s, ())
    return out


def brute_force(g, words):
    """An arc belongs to the set iff it outputs w_t and ends some path, starting anywhere with an arc
    that outputs w_1, whose output labels (arcs without a label skipped) read exactly w_1 .. w_t."""
    want = set()
    for p in all_paths(g):
        if g.olabel[p[0]] == 0:
            continue
        labels = [int(g.olabel[a]) for a in p if g.olabel[a] != 0]
        if g.olabel[p[-1]] != 0 and len(labels) <= len(words) and labels == list(words[:len(labels)]):
            want.add(p[-1])
    return want


@pytest.mark.parametrize("seed", range(25))
def test_against_path_enumeration(seed):
    g = dag(seed)
    for k in (1, 2, 3):
        for words in itertools.product(range(1, 4), repeat=k):
            got = arcs_for_sequence(g, words)
            want = brute_force(g, words)
            # the listing adds the arcs of a prefix also where the sequence cannot continue, which is
            # what the enumeration of prefixes describes too
            assert got == want, (seed, words, sorted(got), sorted(want))


def test_single_word_is_unigram_boosting(tiny_graph):
    g = tiny_graph
    for w in (1, 17, 300):
        assert arcs_for_sequence(g, [w]) == set(np.nonzero(g.olabel == w)[0].tolist())


def test_labels_and_prefix_monotonicity(tiny_graph):
    """Every returned arc outputs a word of the sequence; a longer sequence returns a superset of
    its prefix's set minus nothing (prefix arcs stay)."""
    g = tiny_graph
    rng = np.random.default_rng(3)
    # words along a real path so that continuations exist
    s, words = 0, []
    while len(words) < 4:
        a = int(rng.integers(g.row_offsets[s], g.row_offsets[s + 1]))
        if g.olabel[a]:
            words.append(int(g.olabel[a]))
        s = int(g.dst[a])
    prev = set()
    for k in range(1, 5):
        cur = arcs_for_sequence(g, words[:k])
        assert all(int(g.olabel[a]) in words[:k] for a in cur)
        assert prev <= cur
        prev = cur
    assert len(prev) >= 4
    both = arcs_for_sequences(g, [words[:2], words[2:]])
    assert set(both.tolist()) == arcs_for_sequence(g, words[:2]) | arcs_for_sequence(g, words[2:])


def test_cycle_of_unlabelled_arcs_terminates():
    # 0 -w1-> 1, 1 <-> 2 without labels, 2 -w2-> 3
    g = synth.Graph(4, 4, 1, 2, 0, np.array([0, 1, 2, 4, 4], np.int32), np.array([1, 2, 1, 3], np.int32),
                    np.ones(4, np.int32), np.array([1, 0, 0, 2], np.int32), np.ones(4, np.float32))
    assert arcs_for_sequence(g, [1, 2]) == {0, 3}
    assert arcs_for_sequence(g, [2, 1]) == {3}


def test_spaced_word_labels_keep_the_search_local():
    """The graph of the word-sequence workload: every arc advances the position inside a word, exactly the arcs
    that close a word carry a label, epsilon arcs still lead upwards.  A sequence read off a walk then selects,
    beyond its first word's arcs (all of them: the sequence may start anywhere), at least one arc per later word,
    and each of those leaves a state within word_period arcs of an arc of the word before."""
    p = 4
    g = synth.make_graph(4000, 50, 300, 0.10, seed_stream=(77,), word_period=p)
    src, dst = g.src.astype(np.int64), g.dst.astype(np.int64)
    assert ((dst % p) == ((src + 1) % p)).all()
    assert ((g.olabel != 0) == (dst % p == 0)).all()
    eps = g.ilabel == 0
    assert eps.any() and (dst[eps] > src[eps]).all()
    rng = np.random.default_rng(5)
    seqs = [q for q in synth.word_sequences_on_walks(g, 40, 3, rng) if len(q) == 3]
    assert len(seqs) > 20
    for q in seqs:
        arcs = arcs_for_sequence(g, q)
        by_word = {w: [a for a in arcs if g.olabel[a] == w] for w in set(q)}
        assert set(int(a) for a in np.nonzero(g.olabel == q[0])[0]) <= arcs
        assert all(by_word[w] for w in q)          # the walk itself is a witness for every word
        assert all(g.olabel[a] in q for a in arcs)


def test_word_period_off_leaves_the_graphs_as_they_were():
    """(the other workloads' graphs are pinned by stored results: the option must not touch their random draws)"""
    a = synth.make_graph(3000, 40, 200, 0.15, seed_stream=(3,))
    b = synth.make_graph(3000, 40, 200, 0.15, seed_stream=(3,), word_period=0)
    assert np.array_equal(a.dst, b.dst) and np.array_equal(a.olabel, b.olabel) and np.array_equal(a.weight, b.weight)
