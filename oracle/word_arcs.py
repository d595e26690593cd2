"""Which arcs to boost for a word sequence (paper Algorithm 1) -- TEST INFRASTRUCTURE.

A plain Python statement of the procedure, in the paper's order and notation, on the caller's
CSR arrays.  Reading taken where the listing is loose:
  - "states that output token w": source states of arcs whose output label is w;
  - DepthFirstSearchSpecial(fst, s_p, w_t): leave s_p through an arc that outputs the previous
    word w_{t-1} (the word s_p is known to output), then follow only arcs without an output
    label; every state met on the way that itself has an arc outputting w_t is reachable;
  - ArcsIndicesWithOutput(s_p, w_{t-1}) is added for every s_p, whether or not the search from it
    found a continuation (as the listing has it);
  - after the loop "w_t" is the last word w_k; the input N is not used by the listing.
The sequence may start anywhere in the graph (Sec. 4.1: the first word may start in the
middle of the utterance).
"""
from __future__ import annotations

from typing import Iterable, List, Sequence, Set

import numpy as np


def _arcs_with_output(g, s: int, w: int) -> List[int]:
    return [a for a in range(int(g.row_offsets[s]), int(g.row_offsets[s + 1])) if int(g.olabel[a]) == w]


def _states_that_output(g, w: int) -> Set[int]:
    src = g.src
    return set(int(src[a]) for a in np.nonzero(g.olabel == w)[0])


def _dfs_special(g, s_p: int, w_prev: int, w_next: int) -> Set[int]:
    reachable: Set[int] = set()
    seen: Set[int] = set()
    stack = [int(g.dst[a]) for a in _arcs_with_output(g, s_p, w_prev)]
    while stack:
        q = stack.pop()
        if q in seen:
            continue
        seen.add(q)
        if _arcs_with_output(g, q, w_next):
            reachable.add(q)
        for a in range(int(g.row_offsets[q]), int(g.row_offsets[q + 1])):
            if int(g.olabel[a]) == 0:
                stack.append(int(g.dst[a]))
    return reachable


def arcs_for_sequence(g, words: Sequence[int]) -> Set[int]:
    """Algorithm 1 for one word sequence w_1 .. w_k -> set of arc indices."""
    words = [int(w) for w in words]
    arcs_indices: Set[int] = set()
    if not words:
        return arcs_indices
    states_reached = _states_that_output(g, words[0])
    for t in range(1, len(words)):          # the listing's t = 2 .. k
        prev_states_reached = states_reached
        states_reached = set()
        for s_p in prev_states_reached:
            states_reached |= _dfs_special(g, s_p, words[t - 1], words[t])
            arcs_indices.update(_arcs_with_output(g, s_p, words[t - 1]))
    for s in states_reached:
        arcs_indices.update(_arcs_with_output(g, s, words[-1]))
    return arcs_indices


def arcs_for_sequences(g, sequences: Iterable[Sequence[int]]) -> np.ndarray:
    """Union over a biasing list of sequences, sorted."""
    out: Set[int] = set()
    for seq in sequences:
        out |= arcs_for_sequence(g, seq)
    return np.array(sorted(out), dtype=np.int32)
