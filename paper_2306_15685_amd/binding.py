"""ctypes binding of libcbdec.so: argument marshalling only.

Function names follow include/cbd.h.  Every decoding step runs in the HIP
library; there is no fallback: if the library has not been built, loading
raises.  torch is used by callers for device memory and streams only; this
module takes raw device pointers.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcbdec.so")

CBD_OK, CBD_E_INVALID, CBD_E_CAPACITY, CBD_E_EPS_DIVERGED = 0, -1, -2, -3
CBD_E_NO_TOKENS, CBD_E_BUFFER, CBD_E_HIP, CBD_E_NOMEM = -4, -5, -6, -7

EXPORTS = [
    "cbd_graph_load", "cbd_graph_free", "cbd_context_from_words", "cbd_decoder_create", "cbd_decoder_free", "cbd_reset_channels",
    "cbd_set_context", "cbd_set_contexts", "cbd_contexts_create", "cbd_context_destroy", "cbd_use_contexts", "cbd_advance", "cbd_compact_records", "cbd_best_path", "cbd_best_paths", "cbd_best_paths_static", "cbd_best_paths_begin", "cbd_best_paths_finish", "cbd_best_tails", "cbd_best_tails_begin", "cbd_best_tails_finish",
    "cbd_get_fixed", "cbd_get_tokens",
    "cbd_get_records", "cbd_get_stats", "cbd_decoder_info", "cbd_synchronize", "cbd_selftest", "cbd_strerror", "cbd_last_error",
]


class cbd_graph_desc(C.Structure):
    _fields_ = [("num_states", C.c_int32), ("num_arcs", C.c_int32), ("num_pdfs", C.c_int32),
                ("start_state", C.c_int32), ("row_offsets", C.c_void_p), ("dst", C.c_void_p),
                ("ilabel", C.c_void_p), ("olabel", C.c_void_p), ("weight", C.c_void_p),
                ("final_cost", C.c_void_p)]


class cbd_config(C.Structure):
    _fields_ = [("num_channels", C.c_int32), ("beam", C.c_float), ("max_active", C.c_int32),
                ("max_frames", C.c_int32), ("max_context_arcs", C.c_int32), ("lookup_mode", C.c_int32),
                ("hash_capacity_log2", C.c_int32), ("max_eps_iters", C.c_int32),
                ("records_per_frame", C.c_int32), ("table_location", C.c_int32), ("lds_token_cap", C.c_int32),
                ("max_pool_contexts", C.c_int32), ("workgroups_per_cu", C.c_int32),
                ("compact_records_above", C.c_int32), ("block_threads", C.c_int32),
                ("frame_code", C.c_int32), ("workgroups_per_channel", C.c_int32)]


class cbd_stats(C.Structure):
    _fields_ = [("frames", C.c_int64), ("active_tokens", C.c_int64), ("emit_arcs", C.c_int64),
                ("eps_arcs", C.c_int64), ("candidates", C.c_int64), ("improvements", C.c_int64),
                ("tokens", C.c_int64), ("eps_rounds", C.c_int64), ("records", C.c_int64),
                ("slow_frames", C.c_int64), ("records_dropped", C.c_int64), ("lean_frames", C.c_int64),
                ("compactions", C.c_int32),
                ("status", C.c_int32), ("max_tokens", C.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with paper_2306_15685_amd/build.py "
                           "(this package has no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    i32, i64, f32, vp = C.c_int32, C.c_int64, C.c_float, C.c_void_p
    L.cbd_graph_load.restype = i32
    L.cbd_graph_load.argtypes = [C.POINTER(cbd_graph_desc), C.POINTER(vp)]
    L.cbd_graph_free.restype = i32
    L.cbd_graph_free.argtypes = [vp]
    L.cbd_context_from_words.restype = i32
    L.cbd_context_from_words.argtypes = [vp, vp, vp, i32, vp, i32, vp]
    L.cbd_decoder_create.restype = i32
    L.cbd_decoder_create.argtypes = [vp, C.POINTER(cbd_config), vp, C.POINTER(vp)]
    L.cbd_decoder_free.restype = i32
    L.cbd_decoder_free.argtypes = [vp]
    L.cbd_reset_channels.restype = i32
    L.cbd_reset_channels.argtypes = [vp, vp, i32]
    L.cbd_set_context.restype = i32
    L.cbd_set_context.argtypes = [vp, i32, vp, i32, f32]
    L.cbd_set_contexts.restype = i32
    L.cbd_set_contexts.argtypes = [vp, vp, i32, vp, vp, vp]
    L.cbd_contexts_create.restype = i32
    L.cbd_contexts_create.argtypes = [vp, i32, vp, vp, vp, vp]
    L.cbd_context_destroy.restype = i32
    L.cbd_context_destroy.argtypes = [vp, i32]
    L.cbd_use_contexts.restype = i32
    L.cbd_use_contexts.argtypes = [vp, vp, vp, i32]
    L.cbd_advance.restype = i32
    L.cbd_advance.argtypes = [vp, vp, i32, vp, i64, i32]
    L.cbd_compact_records.restype = i32
    L.cbd_compact_records.argtypes = [vp, vp, i32, i32]
    L.cbd_best_path.restype = i32
    L.cbd_best_path.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp, vp]
    L.cbd_best_paths.restype = i32
    L.cbd_best_paths.argtypes = [vp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    L.cbd_best_paths_static.restype = i32
    L.cbd_best_paths_static.argtypes = [vp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    L.cbd_best_paths_begin.restype = i32
    L.cbd_best_paths_begin.argtypes = [vp, vp, i32, i32, i32, i32, vp]
    L.cbd_best_paths_finish.restype = i32
    L.cbd_best_paths_finish.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp]
    L.cbd_best_tails.restype = i32
    L.cbd_best_tails.argtypes = [vp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    L.cbd_best_tails_begin.restype = i32
    L.cbd_best_tails_begin.argtypes = [vp, vp, i32, i32, i32, i32, vp]
    L.cbd_best_tails_finish.restype = i32
    L.cbd_best_tails_finish.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    L.cbd_get_fixed.restype = i32
    L.cbd_get_fixed.argtypes = [vp, i32, i32, i32, vp, vp, i32, vp, vp]
    L.cbd_get_tokens.restype = i32
    L.cbd_get_tokens.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    L.cbd_get_records.restype = i32
    L.cbd_get_records.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp]
    L.cbd_get_stats.restype = i32
    L.cbd_get_stats.argtypes = [vp, i32, C.POINTER(cbd_stats)]
    L.cbd_decoder_info.restype = i32
    L.cbd_decoder_info.argtypes = [vp, vp, vp, vp, vp]
    L.cbd_synchronize.restype = i32
    L.cbd_synchronize.argtypes = [vp]
    L.cbd_selftest.restype = i32
    L.cbd_selftest.argtypes = []
    L.cbd_strerror.restype = C.c_char_p
    L.cbd_strerror.argtypes = [i32]
    L.cbd_last_error.restype = C.c_char_p
    L.cbd_last_error.argtypes = []
    _lib = L
    return L


class CbdError(RuntimeError):
    def __init__(self, status: int, where: str):
        L = lib()
        msg = L.cbd_strerror(status).decode()
        detail = L.cbd_last_error().decode() if status in (CBD_E_HIP, CBD_E_INVALID) else ""
        super().__init__(f"{where}: {msg} ({status}) {detail}".rstrip())
        self.status = status


def _check(status: int, where: str):
    if status != CBD_OK:
        raise CbdError(status, where)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


# ---- functions named after the C ABI ------------------------------------------

def cbd_graph_load(num_states, num_pdfs, start_state, row_offsets, dst, ilabel, olabel, weight, final_cost=None):
    keep = [_i32(row_offsets), _i32(dst), _i32(ilabel), _i32(olabel),
            np.ascontiguousarray(weight, dtype=np.float32),
            None if final_cost is None else np.ascontiguousarray(final_cost, dtype=np.float32)]
    desc = cbd_graph_desc(int(num_states), int(keep[1].size), int(num_pdfs), int(start_state),
                          _p(keep[0]), _p(keep[1]), _p(keep[2]), _p(keep[3]), _p(keep[4]), _p(keep[5]))
    h = C.c_void_p()
    _check(lib().cbd_graph_load(C.byref(desc), C.byref(h)), "cbd_graph_load")
    return h


def cbd_graph_free(g):
    _check(lib().cbd_graph_free(g), "cbd_graph_free")


def cbd_context_from_words(g, sequences) -> np.ndarray:
    """Algorithm 1 for a list of word-id sequences -> sorted arc indices."""
    words, offs = pack_lists([np.asarray(x, dtype=np.int32) for x in sequences])
    cap = 1 << 14
    while True:
        arcs = np.zeros(cap, np.int32)
        n = C.c_int32(0)
        rc = lib().cbd_context_from_words(g, _p(words), _p(offs), int(len(sequences)), _p(arcs), cap, C.byref(n))
        if rc == CBD_E_BUFFER:
            cap = n.value
            continue
        _check(rc, "cbd_context_from_words")
        return arcs[:n.value].copy()


def cbd_decoder_create(g, num_channels, beam, max_active, max_frames, max_context_arcs, lookup_mode=0,
                       hash_capacity_log2=14, max_eps_iters=0, records_per_frame=0, table_location=0,
                       lds_token_cap=0, max_pool_contexts=0, workgroups_per_cu=0, compact_records_above=0,
                       block_threads=0, frame_code=0, workgroups_per_channel=0, hip_stream=0):
    cfg = cbd_config(int(num_channels), float(beam), int(max_active), int(max_frames), int(max_context_arcs),
                     int(lookup_mode), int(hash_capacity_log2), int(max_eps_iters), int(records_per_frame),
                     int(table_location), int(lds_token_cap), int(max_pool_contexts), int(workgroups_per_cu),
                     int(compact_records_above), int(block_threads), int(frame_code), int(workgroups_per_channel))
    h = C.c_void_p()
    _check(lib().cbd_decoder_create(g, C.byref(cfg), C.c_void_p(int(hip_stream)), C.byref(h)), "cbd_decoder_create")
    return h


def cbd_decoder_free(d):
    _check(lib().cbd_decoder_free(d), "cbd_decoder_free")


def cbd_reset_channels(d, channels):
    ch = _i32(channels)
    _check(lib().cbd_reset_channels(d, _p(ch), int(ch.size)), "cbd_reset_channels")


def cbd_set_context(d, channel, arc_idx, offset):
    a = _i32(arc_idx)
    _check(lib().cbd_set_context(d, int(channel), _p(a), int(a.size), float(offset)), "cbd_set_context")


def pack_lists(lists: Sequence[np.ndarray]):
    """Concatenates arc-index lists -> (arc_idx int32, list_offsets int32 [n+1])."""
    lo = np.zeros(len(lists) + 1, dtype=np.int32)
    if len(lists):
        np.cumsum([len(x) for x in lists], out=lo[1:])
    cat = _i32(np.concatenate([_i32(x) for x in lists])) if len(lists) and lo[-1] > 0 else np.zeros(1, np.int32)
    return cat, lo


def cbd_set_contexts(d, channels, lists, offsets, packed=None):
    """lists: one arc-index array per channel, or pass packed=(arc_idx, list_offsets) from pack_lists."""
    ch = _i32(channels)
    cat, lo = packed if packed is not None else pack_lists(lists)
    off = np.ascontiguousarray(offsets, dtype=np.float32)
    _check(lib().cbd_set_contexts(d, _p(ch), int(ch.size), _p(cat), _p(lo), _p(off)), "cbd_set_contexts")


def cbd_contexts_create(d, lists, offsets, packed=None) -> np.ndarray:
    """Uploads the lists into the decoder's context pool -> context ids."""
    cat, lo = packed if packed is not None else pack_lists(lists)
    off = np.ascontiguousarray(offsets, dtype=np.float32)
    ids = np.zeros(off.size, dtype=np.int32)
    _check(lib().cbd_contexts_create(d, int(off.size), _p(cat), _p(lo), _p(off), _p(ids)), "cbd_contexts_create")
    return ids


def cbd_context_destroy(d, context_id):
    _check(lib().cbd_context_destroy(d, int(context_id)), "cbd_context_destroy")


def cbd_use_contexts(d, channels, context_ids):
    ch = _i32(channels)
    ids = _i32(context_ids)
    assert ch.size == ids.size
    _check(lib().cbd_use_contexts(d, _p(ch), _p(ids), int(ch.size)), "cbd_use_contexts")


def cbd_advance(d, channels, loglikes_ptr: int, channel_stride: int, n_frames: int):
    """loglikes_ptr: device address (e.g. tensor.data_ptr()) of fp32 rows."""
    ch = _i32(channels)
    _check(lib().cbd_advance(d, _p(ch), int(ch.size), C.c_void_p(int(loglikes_ptr)), int(channel_stride),
                             int(n_frames)), "cbd_advance")


def cbd_compact_records(d, channels, min_new_records=0):
    ch = _i32(channels)
    _check(lib().cbd_compact_records(d, _p(ch), int(ch.size), int(min_new_records)), "cbd_compact_records")


def cbd_best_path(d, channel, use_final=False, capacity=4096) -> Tuple[int, np.ndarray, np.ndarray, float]:
    """-> (status, words, arcs, cost); grows the buffers on CBD_E_BUFFER."""
    while True:
        words = np.zeros(capacity, np.int32)
        arcs = np.zeros(capacity, np.int32)
        nw, na, cost = C.c_int32(0), C.c_int32(0), C.c_float(float("inf"))
        rc = lib().cbd_best_path(d, int(channel), int(bool(use_final)), _p(words), _p(arcs), int(capacity),
                                 C.byref(nw), C.byref(na), C.byref(cost))
        if rc == CBD_E_BUFFER:
            capacity = max(capacity * 2, na.value)
            continue
        if rc in (CBD_E_HIP, CBD_E_INVALID):
            raise CbdError(rc, "cbd_best_path")
        return rc, words[:nw.value].copy(), arcs[:na.value].copy(), float(cost.value)


class BestPathBuffers:
    """Host arrays a caller can reuse across cbd_best_paths calls."""

    def __init__(self, n: int, capacity: int, want_arcs: bool = True):
        self.n, self.capacity = n, capacity
        self.words = np.zeros((n, capacity), np.int32)
        self.arcs = np.zeros((n, capacity), np.int32) if want_arcs else None
        self.n_words = np.zeros(n, np.int32)
        self.n_arcs = np.zeros(n, np.int32)
        self.cost = np.zeros(n, np.float32)
        self.status = np.zeros(n, np.int32)
        self.n_fixed_words = np.zeros(n, np.int32)   # (cbd_best_tails* only)
        self.n_fixed_arcs = np.zeros(n, np.int32)


def _result(b: BestPathBuffers, n: int, want_arcs: bool, as_lists: bool, fixed: bool = False):
    """What the cbd_best_paths* / cbd_best_tails* calls left in `b`, as their common return value:
    (status[n], words, arcs or None, cost[n], n_arcs[n], n_words[n]) and, with `fixed`, n_fixed_words[n] and
    n_fixed_arcs[n] behind them.  as_lists: one array per channel (copies); else the [n, capacity] matrices."""
    st, nw, na = b.status[:n], b.n_words[:n], b.n_arcs[:n]
    extra = (b.n_fixed_words[:n], b.n_fixed_arcs[:n]) if fixed else ()
    if not as_lists:
        return (st, b.words, b.arcs if want_arcs else None, b.cost[:n], na, nw) + extra
    wl = [b.words[i, :nw[i]].copy() if st[i] == CBD_OK else np.zeros(0, np.int32) for i in range(n)]
    al = None
    if want_arcs:
        al = [b.arcs[i, :na[i]].copy() if st[i] == CBD_OK else np.zeros(0, np.int32) for i in range(n)]
    return (st.copy(), wl, al, b.cost[:n].copy(), na.copy(), nw.copy()) + tuple(x.copy() for x in extra)


def cbd_best_paths(d, channels, use_final=False, capacity=4096, want_arcs=True, buffers: Optional[BestPathBuffers] = None,
                   as_lists=True):
    """-> (status[n], words, arcs or None, cost[n], n_arcs[n], n_words[n]).

    With as_lists the words / arcs come back as one array per channel; otherwise as the
    [n, capacity] matrices of `buffers` (rows valid up to n_words / n_arcs)."""
    ch = _i32(channels)
    n = int(ch.size)
    b = buffers if buffers is not None else BestPathBuffers(n, capacity, want_arcs)
    assert b.n >= n and b.capacity == capacity
    _check(lib().cbd_best_paths(d, _p(ch), n, int(bool(use_final)), _p(b.words), _p(b.arcs) if want_arcs else None,
                                int(capacity), _p(b.n_words), _p(b.n_arcs), _p(b.cost), _p(b.status)), "cbd_best_paths")
    return _result(b, n, want_arcs, as_lists)


def cbd_best_paths_static(d, channels, use_final=False, capacity=4096, want_arcs=True,
                          buffers: Optional[BestPathBuffers] = None, as_lists=True):
    """cbd_best_paths through the entry point that allocates nothing; same return value."""
    ch = _i32(channels)
    n = int(ch.size)
    b = buffers if buffers is not None else BestPathBuffers(n, capacity, want_arcs)
    assert b.n >= n and b.capacity == capacity
    _check(lib().cbd_best_paths_static(d, _p(ch), n, int(bool(use_final)), _p(b.words),
                                       _p(b.arcs) if want_arcs else None, int(capacity), _p(b.n_words), _p(b.n_arcs),
                                       _p(b.cost), _p(b.status)), "cbd_best_paths_static")
    return _result(b, n, want_arcs, as_lists)


def cbd_best_paths_begin(d, channels, use_final=False, capacity=4096, want_arcs=True) -> int:
    """Enqueues the request; returns a ticket for cbd_best_paths_finish."""
    ch = _i32(channels)
    t = C.c_int32(0)
    _check(lib().cbd_best_paths_begin(d, _p(ch), int(ch.size), int(bool(use_final)), int(capacity), int(bool(want_arcs)),
                                      C.byref(t)), "cbd_best_paths_begin")
    return (t.value, int(ch.size), int(capacity), bool(want_arcs))


def cbd_best_paths_finish(d, ticket, buffers: Optional[BestPathBuffers] = None, as_lists=True):
    """Waits for the request; same return value as cbd_best_paths."""
    t, n, capacity, want_arcs = ticket
    b = buffers if buffers is not None else BestPathBuffers(n, capacity, want_arcs)
    assert b.n >= n and b.capacity == capacity
    _check(lib().cbd_best_paths_finish(d, t, _p(b.words), _p(b.arcs) if want_arcs else None, int(capacity),
                                       _p(b.n_words), _p(b.n_arcs), _p(b.cost), _p(b.status)), "cbd_best_paths_finish")
    return _result(b, n, want_arcs, as_lists)


def cbd_best_tails(d, channels, use_final=False, capacity=4096, want_arcs=True,
                   buffers: Optional[BestPathBuffers] = None, as_lists=True):
    """Like cbd_best_paths for the part of each path above the fixed part
    -> (status, words, arcs or None, cost, n_arcs, n_words, n_fixed_words, n_fixed_arcs)."""
    ch = _i32(channels)
    n = int(ch.size)
    b = buffers if buffers is not None else BestPathBuffers(n, capacity, want_arcs)
    assert b.n >= n and b.capacity == capacity
    _check(lib().cbd_best_tails(d, _p(ch), n, int(bool(use_final)), _p(b.words), _p(b.arcs) if want_arcs else None,
                                int(capacity), _p(b.n_words), _p(b.n_arcs), _p(b.cost), _p(b.status),
                                _p(b.n_fixed_words), _p(b.n_fixed_arcs)), "cbd_best_tails")
    return _result(b, n, want_arcs, as_lists, fixed=True)


def cbd_best_tails_begin(d, channels, use_final=False, capacity=4096, want_arcs=True):
    ch = _i32(channels)
    t = C.c_int32(0)
    _check(lib().cbd_best_tails_begin(d, _p(ch), int(ch.size), int(bool(use_final)), int(capacity), int(bool(want_arcs)),
                                      C.byref(t)), "cbd_best_tails_begin")
    return (t.value, int(ch.size), int(capacity), bool(want_arcs))


def cbd_best_tails_finish(d, ticket, buffers: Optional[BestPathBuffers] = None, as_lists=True):
    t, n, capacity, want_arcs = ticket
    b = buffers if buffers is not None else BestPathBuffers(n, capacity, want_arcs)
    assert b.n >= n and b.capacity == capacity
    _check(lib().cbd_best_tails_finish(d, t, _p(b.words), _p(b.arcs) if want_arcs else None, int(capacity),
                                       _p(b.n_words), _p(b.n_arcs), _p(b.cost), _p(b.status), _p(b.n_fixed_words),
                                       _p(b.n_fixed_arcs)), "cbd_best_tails_finish")
    return _result(b, n, want_arcs, as_lists, fixed=True)


def cbd_get_fixed(d, channel, from_word=0, from_arc=0):
    """-> (words, arcs) of the channel's fixed part from the given positions on."""
    nw, na = C.c_int32(0), C.c_int32(0)
    _check(lib().cbd_get_fixed(d, int(channel), int(from_word), int(from_arc), None, None, 0, C.byref(nw), C.byref(na)),
           "cbd_get_fixed")
    words = np.zeros(max(nw.value, 1), np.int32)
    arcs = np.zeros(max(na.value, 1), np.int32)
    cap = int(max(words.size, arcs.size))
    words = np.zeros(cap, np.int32)
    arcs = np.zeros(cap, np.int32)
    _check(lib().cbd_get_fixed(d, int(channel), int(from_word), int(from_arc), _p(words), _p(arcs), cap, C.byref(nw),
                               C.byref(na)), "cbd_get_fixed")
    return words[:nw.value].copy(), arcs[:na.value].copy()


def cbd_get_tokens(d, channel):
    """-> (status, states, costs, arcs) sorted by state."""
    n = C.c_int32(0)
    rc = lib().cbd_get_tokens(d, int(channel), None, None, None, 0, C.byref(n))
    if rc in (CBD_E_HIP, CBD_E_INVALID):
        raise CbdError(rc, "cbd_get_tokens")
    k = n.value
    st = np.zeros(max(k, 1), np.int32)
    co = np.zeros(max(k, 1), np.float32)
    ar = np.zeros(max(k, 1), np.int32)
    if rc == CBD_OK and k > 0:
        _check(lib().cbd_get_tokens(d, int(channel), _p(st), _p(co), _p(ar), k, C.byref(n)), "cbd_get_tokens")
    st, co, ar = st[:k], co[:k], ar[:k]
    o = np.argsort(st, kind="stable")
    return rc, st[o], co[o], ar[o]


def cbd_get_records(d, channel):
    """-> (arcs, prev, frame_base, kept_base): the channel's back-pointer records."""
    n, fb, kb = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(lib().cbd_get_records(d, int(channel), None, None, 0, C.byref(n), C.byref(fb), C.byref(kb)),
           "cbd_get_records")
    arcs = np.zeros(max(n.value, 1), np.int32)
    prev = np.zeros(max(n.value, 1), np.int32)
    _check(lib().cbd_get_records(d, int(channel), _p(arcs), _p(prev), int(arcs.size), C.byref(n), C.byref(fb),
                                 C.byref(kb)), "cbd_get_records")
    return arcs[:n.value], prev[:n.value], fb.value, kb.value


def cbd_get_stats(d, channel=-1) -> dict:
    s = cbd_stats()
    _check(lib().cbd_get_stats(d, int(channel), C.byref(s)), "cbd_get_stats")
    return s.as_dict()


def cbd_decoder_info(d) -> dict:
    b, l, t, i = C.c_int64(0), C.c_int32(0), C.c_int32(0), C.c_int32(0)
    _check(lib().cbd_decoder_info(d, C.byref(b), C.byref(l), C.byref(t), C.byref(i)), "cbd_decoder_info")
    return {"device_bytes": b.value, "lds_bytes": l.value, "block_threads": t.value, "lds_token_cap": i.value,
            "tables_in_lds": i.value > 0}


def cbd_synchronize(d):
    _check(lib().cbd_synchronize(d), "cbd_synchronize")


def cbd_selftest():
    _check(lib().cbd_selftest(), "cbd_selftest")


def cbd_strerror(status: int) -> str:
    return lib().cbd_strerror(int(status)).decode()
