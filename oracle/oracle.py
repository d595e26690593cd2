"""ctypes front end of the C checker in cbd_oracle.c -- TEST INFRASTRUCTURE.

Argument marshalling only; every decoding step runs in the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cbd_oracle.c")
# CBD_ORACLE_SANITIZE=1: the checker built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only);
# the process must then have been started with the sanitizer's runtime preloaded (tests/test_oracle_sanitized.py).
SANITIZE = os.environ.get("CBD_ORACLE_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "liboracle_san.so" if SANITIZE else "liboracle.so")

ORC_OK, ORC_NO_TOKENS, ORC_EPS_DIVERGED, ORC_BUFFER, ORC_INVALID = 0, 1, 2, 3, 4

_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the checker with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
               "-Wall", "-Wextra", "-o", _LIB + ".tmp", _SRC, "-lm"]
        if SANITIZE:
            cmd[1:2] = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                        "-fno-omit-frame-pointer"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = C.CDLL(build_oracle())
    i32, i64, f32, vp = C.c_int32, C.c_int64, C.c_float, C.c_void_p
    lib.orc_graph_new.restype = vp
    lib.orc_graph_new.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    lib.orc_graph_free.argtypes = [vp]
    lib.orc_chan_new.restype = vp
    lib.orc_chan_new.argtypes = [vp, f32, i32, i32]
    lib.orc_chan_free.argtypes = [vp]
    lib.orc_set_context.restype = i32
    lib.orc_set_context.argtypes = [vp, vp, i32, f32]
    lib.orc_set_lookup_mode.argtypes = [vp, i32]
    lib.orc_reset.restype = i32
    lib.orc_reset.argtypes = [vp]
    lib.orc_advance.restype = i32
    lib.orc_advance.argtypes = [vp, vp, i32, i64]
    lib.orc_best_path.restype = i32
    lib.orc_best_path.argtypes = [vp, i32, vp, vp, i32, vp, vp, vp]
    lib.orc_get_tokens.restype = i32
    lib.orc_get_tokens.argtypes = [vp, vp, vp, vp, i32]
    lib.orc_stat.restype = i64
    lib.orc_stat.argtypes = [vp, i32]
    lib.orc_last_m.restype = f32
    lib.orc_last_m.argtypes = [vp]
    lib.orc_last_best.restype = f32
    lib.orc_last_best.argtypes = [vp]
    lib.orc_status.restype = i32
    lib.orc_status.argtypes = [vp]
    lib.orc_prune.restype = i32
    lib.orc_prune.argtypes = [vp, i32, f32, i32, vp, vp, vp]
    _lib = lib
    return lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class OracleGraph:
    """Holds the caller's CSR arrays (kept alive here; the C side borrows them)."""

    def __init__(self, num_states, num_pdfs, start_state, row_offsets, dst, ilabel, olabel, weight,
                 final_cost=None):
        lib = _load()
        self.row = np.ascontiguousarray(row_offsets, dtype=np.int32)
        self.dst = np.ascontiguousarray(dst, dtype=np.int32)
        self.ilabel = np.ascontiguousarray(ilabel, dtype=np.int32)
        self.olabel = np.ascontiguousarray(olabel, dtype=np.int32)
        self.weight = np.ascontiguousarray(weight, dtype=np.float32)
        self.final = None if final_cost is None else np.ascontiguousarray(final_cost, dtype=np.float32)
        self.num_states = int(num_states)
        self.num_arcs = int(self.dst.size)
        self.num_pdfs = int(num_pdfs)
        self.h = lib.orc_graph_new(self.num_states, self.num_arcs, self.num_pdfs, int(start_state),
                                   _ptr(self.row), _ptr(self.dst), _ptr(self.ilabel), _ptr(self.olabel),
                                   _ptr(self.weight), _ptr(self.final))
        if not self.h:
            raise ValueError("bad graph")

    @classmethod
    def from_graph(cls, g) -> "OracleGraph":
        return cls(g.num_states, g.num_pdfs, g.start_state, g.row_offsets, g.dst, g.ilabel, g.olabel,
                   g.weight, g.final_cost)

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.orc_graph_free(self.h)
            self.h = None


class OracleChannel:
    """One decoding channel of the checker."""

    def __init__(self, graph: OracleGraph, beam: float, max_active: int = 0, max_eps_iters: int = 64):
        self.lib = _load()
        self.graph = graph
        self.h = self.lib.orc_chan_new(graph.h, float(beam), int(max_active), int(max_eps_iters))

    def __del__(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.orc_chan_free(self.h)
            self.h = None

    def set_context(self, arcs, offset: float) -> int:
        a = np.ascontiguousarray(arcs, dtype=np.int32)
        return self.lib.orc_set_context(self.h, _ptr(a), int(a.size), float(offset))

    def set_lookup_mode(self, mode: int) -> None:
        self.lib.orc_set_lookup_mode(self.h, int(mode))

    def reset(self) -> int:
        return self.lib.orc_reset(self.h)

    def advance(self, loglikes: np.ndarray) -> int:
        """loglikes: float32 [frames, num_pdfs], rows contiguous."""
        L = np.asarray(loglikes)
        assert L.dtype == np.float32 and L.ndim == 2 and L.shape[1] == self.graph.num_pdfs
        assert L.strides[1] == 4
        return self.lib.orc_advance(self.h, _ptr(L), int(L.shape[0]), int(L.strides[0] // 4))

    def best_path(self, use_final: bool = False) -> Tuple[int, np.ndarray, np.ndarray, float]:
        """-> (status, words, arcs, cost)."""
        cap = 1 << 12
        while True:
            words = np.zeros(cap, dtype=np.int32)
            arcs = np.zeros(cap, dtype=np.int32)
            nw, na, cost = C.c_int32(0), C.c_int32(0), C.c_float(0)
            rc = self.lib.orc_best_path(self.h, int(use_final), _ptr(words), _ptr(arcs), cap,
                                        C.byref(nw), C.byref(na), C.byref(cost))
            if rc == ORC_BUFFER:
                cap = max(cap * 2, na.value)
                continue
            return rc, words[:nw.value].copy(), arcs[:na.value].copy(), float(cost.value)

    def tokens(self):
        """Current table as (states, costs, arcs), sorted by state."""
        n = self.lib.orc_get_tokens(self.h, None, None, None, 0)
        st = np.zeros(n, dtype=np.int32)
        co = np.zeros(n, dtype=np.float32)
        ar = np.zeros(n, dtype=np.int32)
        self.lib.orc_get_tokens(self.h, _ptr(st), _ptr(co), _ptr(ar), n)
        o = np.argsort(st, kind="stable")
        return st[o], co[o], ar[o]

    def stat(self, which: int) -> int:
        return int(self.lib.orc_stat(self.h, which))

    @property
    def emit_arcs(self) -> int:
        return self.stat(0)

    @property
    def last_m(self) -> float:
        return float(self.lib.orc_last_m(self.h))

    @property
    def last_best(self) -> float:
        return float(self.lib.orc_last_best(self.h))

    @property
    def status(self) -> int:
        return int(self.lib.orc_status(self.h))


def prune(costs, beam: float, max_active: int):
    """Step 1 on a bare cost list -> (alive mask, best, cut bin or -1)."""
    lib = _load()
    c = np.ascontiguousarray(costs, dtype=np.float32)
    alive = np.zeros(c.size, dtype=np.uint8)
    best, cut = C.c_float(0), C.c_int32(-1)
    lib.orc_prune(_ptr(c), int(c.size), float(beam), int(max_active), _ptr(alive), C.byref(best), C.byref(cut))
    return alive.astype(bool), float(best.value), int(cut.value)
