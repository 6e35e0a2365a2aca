"""ctypes wrapper around the CPU checker (wfst_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The GPU library never imports this package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_DIR, "_libwfst_oracle.so")
NO_ARC = 0xFFFFFFFF
ST_OK, ST_DEAD, ST_BAD_INPUT = 0, 1, 2


def build(force: bool = False) -> str:
    src = os.path.join(_DIR, "wfst_oracle.cpp")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared",
                               "-o", _SO, src])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = C.CDLL(_SO)
        vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        L.oracle_graph_new.restype = vp
        L.oracle_graph_new.argtypes = [i32, i64, i32, i32, vp, vp, vp, vp, vp, vp]
        L.oracle_graph_free.argtypes = [vp]
        L.oracle_decoder_new.restype = vp
        L.oracle_decoder_new.argtypes = [vp, f32, f32, i32, i32]
        L.oracle_decoder_free.argtypes = [vp]
        L.oracle_init.argtypes = [vp]
        L.oracle_advance.argtypes = [vp, vp, i64, i32]
        for name in ("oracle_status", "oracle_num_frames", "oracle_max_tokens_pre_prune", "oracle_max_tokens"):
            getattr(L, name).argtypes = [vp]
            getattr(L, name).restype = i32
        L.oracle_arcs_expanded.argtypes = [vp]
        L.oracle_arcs_expanded.restype = i64
        L.oracle_last_cutoff.argtypes = [vp]
        L.oracle_last_cutoff.restype = f32
        L.oracle_num_tokens.argtypes = [vp, i32]
        L.oracle_num_tokens.restype = i32
        L.oracle_tokens.argtypes = [vp, i32, vp, vp, vp, i32]
        L.oracle_tokens.restype = i32
        L.oracle_num_lattice.argtypes = [vp]
        L.oracle_num_lattice.restype = i64
        L.oracle_lattice.argtypes = [vp, i32, vp, vp, vp, i64]
        L.oracle_lattice.restype = i64
        L.oracle_best_path.argtypes = [vp, i32, vp, i32, vp, vp, i32, vp, vp, vp]
        L.oracle_best_path.restype = i32
        L.oracle_final_lattice.argtypes = [vp, i32, vp, vp, vp, i64, vp, vp]
        L.oracle_final_lattice.restype = i64
        L.oracle_closure.argtypes = [vp, i32, vp, vp, vp, i32, f32]
        L.oracle_closure.restype = i32
        _lib = L
    return _lib


class OracleGraph:
    """Host copy of a CSR WFST for the checker. `g` is any object with the CSR fields
    (num_states, num_arcs, start_state, num_pdfs, row_offsets, ilabel, olabel, weight,
    nextstate, final_cost) as numpy arrays."""

    def __init__(self, g):
        self.g = g
        self._keep = [np.ascontiguousarray(g.row_offsets, np.int64), np.ascontiguousarray(g.ilabel, np.int32),
                      np.ascontiguousarray(g.olabel, np.int32), np.ascontiguousarray(g.weight, np.float32),
                      np.ascontiguousarray(g.nextstate, np.int32), np.ascontiguousarray(g.final_cost, np.float32)]
        self.h = lib().oracle_graph_new(g.num_states, g.num_arcs, g.start_state, g.num_pdfs,
                                        *[a.ctypes.data for a in self._keep])

    def __del__(self):
        if getattr(self, "h", None):
            lib().oracle_graph_free(self.h)
            self.h = None

    def closure(self, states, costs, in_arcs, cutoff: float, cap: int = 1 << 20):
        st = np.zeros(cap, np.int32); st[:len(states)] = states
        co = np.zeros(cap, np.float32); co[:len(states)] = costs
        ia = np.full(cap, NO_ARC, np.uint32); ia[:len(states)] = in_arcs
        n = lib().oracle_closure(self.h, len(states), st.ctypes.data, co.ctypes.data, ia.ctypes.data, cap, cutoff)
        assert n >= 0
        return st[:n].copy(), co[:n].copy(), ia[:n].copy()


class OracleDecoder:
    """One stream decoded by the checker."""

    def __init__(self, graph: OracleGraph, beam: float, lattice_beam: float, max_active: int, lattice_on: bool = True):
        self.graph = graph
        self.h = lib().oracle_decoder_new(graph.h, beam, lattice_beam, max_active, int(lattice_on))
        lib().oracle_init(self.h)

    def __del__(self):
        if getattr(self, "h", None):
            lib().oracle_decoder_free(self.h)
            self.h = None

    def advance(self, rows: np.ndarray) -> None:
        rows = np.ascontiguousarray(rows, np.float32)
        assert rows.ndim == 2
        lib().oracle_advance(self.h, rows.ctypes.data, rows.shape[1], rows.shape[0])

    @property
    def status(self) -> int:
        return lib().oracle_status(self.h)

    @property
    def num_frames(self) -> int:
        return lib().oracle_num_frames(self.h)

    @property
    def arcs_expanded(self) -> int:
        return lib().oracle_arcs_expanded(self.h)

    @property
    def max_tokens_pre_prune(self) -> int:
        return lib().oracle_max_tokens_pre_prune(self.h)

    @property
    def max_tokens(self) -> int:
        return lib().oracle_max_tokens(self.h)

    @property
    def last_cutoff(self) -> float:
        return lib().oracle_last_cutoff(self.h)

    def tokens(self, frame: int = -1):
        """(state int32[], cost float32[], in_arc uint32[]) sorted by state."""
        n = lib().oracle_num_tokens(self.h, frame)
        if n < 0:
            raise IndexError(frame)
        st, co, ia = np.empty(n, np.int32), np.empty(n, np.float32), np.empty(n, np.uint32)
        m = lib().oracle_tokens(self.h, frame, st.ctypes.data, co.ctypes.data, ia.ctypes.data, n)
        assert m == n
        return st, co, ia

    def lattice(self, from_frame: int = 0):
        """(frame int32[], arc uint32[], extra float32[]) sorted by (frame, arc)."""
        cap = lib().oracle_num_lattice(self.h)
        fr, ar, ex = np.empty(cap, np.int32), np.empty(cap, np.uint32), np.empty(cap, np.float32)
        n = lib().oracle_lattice(self.h, from_frame, fr.ctypes.data, ar.ctypes.data, ex.ctypes.data, cap)
        assert n >= 0
        return fr[:n].copy(), ar[:n].copy(), ex[:n].copy()

    def final_lattice(self, use_final: bool = True):
        """Backward-pruned lattice: dict(frame, arc, extra sorted by (frame, arc), best_cost,
        reached_final), or None if there is no token."""
        cap = max(lib().oracle_num_lattice(self.h), 1)
        fr, ar, ex = np.empty(cap, np.int32), np.empty(cap, np.uint32), np.empty(cap, np.float32)
        bc, rf = C.c_float(), C.c_int32()
        n = lib().oracle_final_lattice(self.h, int(use_final), fr.ctypes.data, ar.ctypes.data, ex.ctypes.data, cap,
                                       C.byref(bc), C.byref(rf))
        if n == -1:
            return None
        assert n >= 0
        return dict(frame=fr[:n].copy(), arc=ar[:n].copy(), extra=ex[:n].copy(), best_cost=np.float32(bc.value),
                    reached_final=bool(rf.value))

    def best_path(self, use_final: bool = True):
        """dict(words, arcs, total_cost, reached_final) or None if there is no token."""
        cap = 8 * self.num_frames + 64
        while True:
            words, arcs = np.empty(cap, np.int32), np.empty(cap, np.int64)
            nw, na, rf, tc = C.c_int32(), C.c_int32(), C.c_int32(), C.c_float()
            rc = lib().oracle_best_path(self.h, int(use_final), words.ctypes.data, cap, C.byref(nw),
                                        arcs.ctypes.data, cap, C.byref(na), C.byref(tc), C.byref(rf))
            if rc == -2:
                cap *= 4
                continue
            if rc == -1:
                return None
            if rc != 0:
                raise RuntimeError(f"oracle_best_path: broken trace ({rc})")
            return dict(words=words[:nw.value].copy(), arcs=arcs[:na.value].copy(),
                        total_cost=np.float32(tc.value), reached_final=bool(rf.value))
