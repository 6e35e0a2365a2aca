"""Thin ctypes binding of the wfst_decode C ABI (include/wfst_decode.h).

Argument marshalling only: every step of decoding runs in the library's HIP kernels.
There is no CPU fallback — importing this module fails if the library has not been built
(python -m paper_1910_10032_amd.build, or __graft_entry__.build()).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_DIR, "_libwfst_decode.so")
NO_ARC = 0xFFFFFFFF

WFST_OK = 0
WFST_E_INVALID_ARG, WFST_E_BAD_GRAPH, WFST_E_BAD_CHANNEL, WFST_E_NOT_INIT, WFST_E_CAPACITY = -1, -2, -3, -4, -5
WFST_E_TOKEN_OVERFLOW, WFST_E_LATTICE_OVERFLOW, WFST_E_DEAD_CHANNEL, WFST_E_NAN_INPUT = -6, -7, -8, -9
WFST_E_BROKEN_TRACE, WFST_E_DEVICE, WFST_E_HISTORY_OVERFLOW, WFST_E_SCRATCH_LIMIT = -10, -11, -12, -13

EXPORTS = [
    "wfst_decode_graph_load", "wfst_decode_graph_free", "wfst_decode_graph_bytes", "wfst_decode_create",
    "wfst_decode_destroy", "wfst_decode_state_bytes", "wfst_decode_init_channels", "wfst_decode_free_channels",
    "wfst_decode_advance", "wfst_decode_best_path_batch", "wfst_decode_best_path", "wfst_decode_best_path_arcs",
    "wfst_decode_lattice_arcs", "wfst_decode_lattice_arcs_batch", "wfst_decode_advance_snapshots",
    "wfst_decode_snapshot_wait", "wfst_decode_snapshot_best_path_batch", "wfst_decode_snapshot_lattice_arcs", "wfst_decode_final_lattice", "wfst_decode_final_lattice_batch", "wfst_decode_final_lattice_noalloc", "wfst_decode_tokens", "wfst_decode_stats", "wfst_decode_set_profiling",
    "wfst_decode_profile", "wfst_decode_strerror",
    "wfst_mux_create", "wfst_mux_destroy", "wfst_mux_submit", "wfst_mux_step", "wfst_mux_pending", "wfst_mux_stats",
]


class wfst_csr_t(C.Structure):
    _fields_ = [("num_states", C.c_int32), ("num_arcs", C.c_int64), ("start_state", C.c_int32),
                ("num_pdfs", C.c_int32), ("row_offsets", C.c_void_p), ("ilabel", C.c_void_p),
                ("olabel", C.c_void_p), ("weight", C.c_void_p), ("nextstate", C.c_void_p),
                ("final_cost", C.c_void_p)]


class wfst_config_t(C.Structure):
    _fields_ = [("beam", C.c_float), ("lattice_beam", C.c_float), ("max_active", C.c_int32),
                ("num_channels", C.c_int32), ("max_lanes", C.c_int32), ("max_frames", C.c_int32),
                ("token_capacity", C.c_int32), ("aux_capacity", C.c_int32), ("history_capacity", C.c_int64),
                ("lattice_capacity", C.c_int64), ("lattice_on", C.c_int32), ("snapshot_blocks", C.c_int32),
                ("snapshot_block_capacity", C.c_int64), ("lane_threads", C.c_int32), ("frame_form", C.c_int32), ("approximate", C.c_int32), ("lane_workgroups", C.c_int32)]


class wfst_stats_t(C.Structure):
    _fields_ = [("frames", C.c_int64), ("arcs_expanded", C.c_int64), ("lattice_arcs", C.c_int64),
                ("tokens", C.c_int64), ("max_tokens_pre_prune", C.c_int32), ("max_tokens", C.c_int32),
                ("closure_iters_max", C.c_int32), ("status", C.c_int32)]


class wfst_lattice_info_t(C.Structure):
    _fields_ = [("arcs_in", C.c_int64), ("arcs_kept", C.c_int64), ("frames", C.c_int32),
                ("reached_final", C.c_int32), ("best_cost", C.c_float), ("density", C.c_float)]


LAT_DTYPE = np.dtype([("frame", np.int32), ("arc", np.uint32), ("extra_cost", np.float32)])
TOK_DTYPE = np.dtype([("state", np.int32), ("cost", np.float32), ("in_arc", np.uint32)])

_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1910_10032_amd.build` "
                               "(hipcc, gfx950); there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.wfst_decode_graph_load.argtypes = [C.POINTER(wfst_csr_t), C.POINTER(vp)]
        L.wfst_decode_graph_free.argtypes = [vp]
        L.wfst_decode_graph_free.restype = None
        L.wfst_decode_graph_bytes.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
        L.wfst_decode_create.argtypes = [vp, C.POINTER(wfst_config_t), C.POINTER(vp)]
        L.wfst_decode_destroy.argtypes = [vp]
        L.wfst_decode_destroy.restype = None
        L.wfst_decode_state_bytes.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
        L.wfst_decode_init_channels.argtypes = [vp, vp, i32]
        L.wfst_decode_free_channels.argtypes = [vp, vp, i32]
        L.wfst_decode_advance.argtypes = [vp, vp, i32, vp, vp, vp, vp]
        L.wfst_decode_best_path_batch.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp, vp]
        L.wfst_decode_best_path.argtypes = [vp, i32, i32, vp, i32, C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(i32)]
        L.wfst_decode_best_path_arcs.argtypes = [vp, i32, i32, vp, i32, C.POINTER(i32), C.POINTER(C.c_float), C.POINTER(i32)]
        L.wfst_decode_lattice_arcs.argtypes = [vp, i32, i32, vp, i64, C.POINTER(i64), i32]
        L.wfst_decode_lattice_arcs_batch.argtypes = [vp, vp, i32, vp, i64, vp, i32]
        L.wfst_decode_advance_snapshots.argtypes = [vp, vp, i32, vp, vp, vp, i32, vp, C.POINTER(i64), C.POINTER(i32)]
        L.wfst_decode_snapshot_wait.argtypes = [vp, i64]
        L.wfst_decode_snapshot_best_path_batch.argtypes = [vp, i64, vp, i32, i32, vp, i32, vp, vp, vp, vp]
        L.wfst_decode_snapshot_lattice_arcs.argtypes = [vp, i64, vp, i32, vp, vp, vp, i64, i32, C.POINTER(i64), C.POINTER(vp)]
        L.wfst_decode_final_lattice.argtypes = [vp, i32, i32, vp, i64, C.POINTER(i64), i32, C.POINTER(wfst_lattice_info_t)]
        L.wfst_decode_final_lattice_batch.argtypes = [vp, vp, i32, i32, vp, i64, vp, i32, vp, vp]
        L.wfst_decode_final_lattice_noalloc.argtypes = [vp, i32, i32, vp, i64, C.POINTER(i64), C.POINTER(wfst_lattice_info_t)]
        L.wfst_decode_tokens.argtypes = [vp, i32, i32, vp, i32, C.POINTER(i32)]
        L.wfst_decode_stats.argtypes = [vp, i32, C.POINTER(wfst_stats_t)]
        L.wfst_decode_set_profiling.argtypes = [vp, i32]
        L.wfst_decode_profile.argtypes = [vp, C.POINTER(i64), C.POINTER(C.c_double)]
        L.wfst_decode_strerror.argtypes = [C.c_int]
        L.wfst_decode_strerror.restype = C.c_char_p
        L.wfst_mux_create.argtypes = [vp, C.POINTER(vp)]
        L.wfst_mux_destroy.argtypes = [vp]
        L.wfst_mux_destroy.restype = None
        L.wfst_mux_submit.argtypes = [vp, i32, vp, i32, i32]
        L.wfst_mux_step.argtypes = [vp, vp, C.POINTER(i32)]
        L.wfst_mux_pending.argtypes = [vp]
        L.wfst_mux_pending.restype = i64
        L.wfst_mux_stats.argtypes = [vp, C.POINTER(i64), C.POINTER(i64)]
        _lib = L
    return _lib


class WfstError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lib().wfst_decode_strerror(code).decode()} ({code})")


def _check(code: int, where: str) -> None:
    if code != 0:
        raise WfstError(code, where)


class WfstGraph:
    """wfst_decode_graph_load / _free / _bytes.  `g` carries the CSR fields as numpy arrays."""

    def __init__(self, g):
        self._keep = [np.ascontiguousarray(g.row_offsets, np.int64), np.ascontiguousarray(g.ilabel, np.int32),
                      np.ascontiguousarray(g.olabel, np.int32), np.ascontiguousarray(g.weight, np.float32),
                      np.ascontiguousarray(g.nextstate, np.int32), np.ascontiguousarray(g.final_cost, np.float32)]
        csr = wfst_csr_t(g.num_states, g.num_arcs, g.start_state, g.num_pdfs, *[a.ctypes.data for a in self._keep])
        self.h = C.c_void_p()
        _check(lib().wfst_decode_graph_load(C.byref(csr), C.byref(self.h)), "wfst_decode_graph_load")
        self._keep = None
        self.num_pdfs = g.num_pdfs

    def graph_bytes(self):
        a, b = C.c_int64(), C.c_int64()
        _check(lib().wfst_decode_graph_bytes(self.h, C.byref(a), C.byref(b)), "wfst_decode_graph_bytes")
        return a.value, b.value

    def free(self):
        if self.h:
            lib().wfst_decode_graph_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class WfstDecoder:
    """wfst_decode_create and the per-decoder calls, one method per C entry point."""

    def __init__(self, graph: WfstGraph, beam: float, lattice_beam: float, max_active: int, num_channels: int,
                 max_lanes: int, max_frames: int, token_capacity: int = 0, aux_capacity: int = 0,
                 history_capacity: int = 0, lattice_capacity: int = 0, lattice_on: bool = True,
                 snapshot_blocks: int = 0, snapshot_block_capacity: int = 0, lane_threads: int = 0,
                 frame_form: int = 0, approximate: bool = False, lane_workgroups: int = 0):
        self.graph = graph
        self.cfg = wfst_config_t(beam, lattice_beam, max_active, num_channels, max_lanes, max_frames, token_capacity,
                                 aux_capacity, history_capacity, lattice_capacity, int(lattice_on), snapshot_blocks,
                                 snapshot_block_capacity, lane_threads, frame_form, int(approximate), lane_workgroups)
        self.h = C.c_void_p()
        _check(lib().wfst_decode_create(graph.h, C.byref(self.cfg), C.byref(self.h)), "wfst_decode_create")

    def destroy(self):
        if self.h:
            lib().wfst_decode_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def state_bytes(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib().wfst_decode_state_bytes(self.h, C.byref(a), C.byref(b), C.byref(c)), "wfst_decode_state_bytes")
        return a.value, b.value, c.value

    def init_channels(self, channels) -> None:
        ch = np.ascontiguousarray(channels, np.int32)
        _check(lib().wfst_decode_init_channels(self.h, ch.ctypes.data, len(ch)), "wfst_decode_init_channels")

    def free_channels(self, channels) -> None:
        ch = np.ascontiguousarray(channels, np.int32)
        _check(lib().wfst_decode_free_channels(self.h, ch.ctypes.data, len(ch)), "wfst_decode_free_channels")

    def advance(self, channels, loglikes, n_frames=None, stream=None, snapshot_every: int = 0):
        """loglikes: one 2-D float32 cuda tensor per lane (rows = frames), or a list of
        (device_ptr, stride) pairs together with n_frames.  With snapshot_every > 0 the lanes seal
        a snapshot after every that many frames; returns (first snapshot id, number of snapshots)."""
        ch = np.ascontiguousarray(channels, np.int32)
        n = len(ch)
        ptrs = np.empty(n, np.uint64)
        strides = np.empty(n, np.int32)
        nfr = np.empty(n, np.int32)
        for i, t in enumerate(loglikes):
            if isinstance(t, tuple):
                ptrs[i], strides[i] = t
                nfr[i] = n_frames[i]
            else:
                assert t.is_cuda and t.dim() == 2 and t.stride(1) == 1 and str(t.dtype) == "torch.float32"
                ptrs[i], strides[i] = t.data_ptr(), t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])
                nfr[i] = t.shape[0] if n_frames is None else n_frames[i]
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        return self.advance_ptrs(ch, ptrs, strides, nfr, stream, snapshot_every)

    def advance_ptrs(self, channels: np.ndarray, ptrs: np.ndarray, strides: np.ndarray, n_frames: np.ndarray,
                     stream: int, snapshot_every: int = 0):
        """wfst_decode_advance(_snapshots) with ready-made argument arrays (int32 / uint64 / int32 / int32)."""
        if snapshot_every <= 0:
            _check(lib().wfst_decode_advance(self.h, channels.ctypes.data, len(channels), ptrs.ctypes.data,
                                             strides.ctypes.data, n_frames.ctypes.data, C.c_void_p(stream)),
                   "wfst_decode_advance")
            return None
        first, count = C.c_int64(), C.c_int32()
        _check(lib().wfst_decode_advance_snapshots(self.h, channels.ctypes.data, len(channels), ptrs.ctypes.data,
                                                   strides.ctypes.data, n_frames.ctypes.data, snapshot_every,
                                                   C.c_void_p(stream), C.byref(first), C.byref(count)),
               "wfst_decode_advance_snapshots")
        return first.value, count.value

    def snapshot_wait(self, snapshot_id: int) -> None:
        _check(lib().wfst_decode_snapshot_wait(self.h, snapshot_id), "wfst_decode_snapshot_wait")

    def best_path_batch(self, channels, use_final: bool = True, words_cap: int = 4096, raw: bool = False,
                        snapshot: int = 0):
        """Per channel: dict(status, words, total_cost, reached_final); with raw=True the
        arrays (words [n, cap], n_words, total_cost, reached_final, status) as filled by the call.
        snapshot = id of a sealed snapshot to read instead of the live state."""
        ch = np.ascontiguousarray(channels, np.int32)
        n = len(ch)
        if snapshot:
            def fn(h, *a):
                return lib().wfst_decode_snapshot_best_path_batch(h, snapshot, *a)
        else:
            fn = lib().wfst_decode_best_path_batch
        if raw:
            words = np.empty((n, max(words_cap, 1)), np.int32)
            nw, tc = np.empty(n, np.int32), np.empty(n, np.float32)
            rf, st = np.empty(n, np.int32), np.empty(n, np.int32)
            _check(fn(self.h, ch.ctypes.data, n, int(use_final), words.ctypes.data, words_cap, nw.ctypes.data,
                      tc.ctypes.data, rf.ctypes.data, st.ctypes.data), "wfst_decode_best_path_batch")
            return words, nw, tc, rf, st
        while True:
            words = np.zeros((n, max(words_cap, 1)), np.int32)
            nw, tc = np.zeros(n, np.int32), np.zeros(n, np.float32)
            rf, st = np.zeros(n, np.int32), np.zeros(n, np.int32)
            _check(fn(self.h, ch.ctypes.data, n, int(use_final), words.ctypes.data, words_cap, nw.ctypes.data,
                      tc.ctypes.data, rf.ctypes.data, st.ctypes.data), "wfst_decode_best_path_batch")
            if (st == WFST_E_CAPACITY).any():
                words_cap = int(nw.max())
                continue
            return [dict(status=int(st[i]), words=words[i, :nw[i]].copy() if st[i] == 0 else None,
                         total_cost=np.float32(tc[i]), reached_final=bool(rf[i])) for i in range(n)]

    def best_path(self, channel: int, use_final: bool = True, cap: int = 4096):
        while True:
            words = np.zeros(max(cap, 1), np.int32)
            nw, rf, tc = C.c_int32(), C.c_int32(), C.c_float()
            rc = lib().wfst_decode_best_path(self.h, channel, int(use_final), words.ctypes.data, cap, C.byref(nw),
                                             C.byref(tc), C.byref(rf))
            if rc == WFST_E_CAPACITY:
                cap = nw.value
                continue
            _check(rc, "wfst_decode_best_path")
            return dict(words=words[:nw.value].copy(), total_cost=np.float32(tc.value), reached_final=bool(rf.value))

    def best_path_arcs(self, channel: int, use_final: bool = True, cap: int = 8192):
        while True:
            arcs = np.zeros(max(cap, 1), np.uint32)
            na, rf, tc = C.c_int32(), C.c_int32(), C.c_float()
            rc = lib().wfst_decode_best_path_arcs(self.h, channel, int(use_final), arcs.ctypes.data, cap, C.byref(na),
                                                  C.byref(tc), C.byref(rf))
            if rc == WFST_E_CAPACITY:
                cap = na.value
                continue
            _check(rc, "wfst_decode_best_path_arcs")
            return dict(arcs=arcs[:na.value].copy(), total_cost=np.float32(tc.value), reached_final=bool(rf.value))

    def lattice_arcs(self, channel: int, from_frame: int = 0, cap: int = 1 << 16, out_device=None):
        """Drains the channel's buffered lattice arcs: structured numpy array (host), or the
        count written into the cuda tensor `out_device` (uint8/any dtype, >= 12*cap bytes)."""
        while True:
            n = C.c_int64()
            if out_device is not None:
                cap = out_device.numel() * out_device.element_size() // LAT_DTYPE.itemsize
                rc = lib().wfst_decode_lattice_arcs(self.h, channel, from_frame, out_device.data_ptr(), cap, C.byref(n), 1)
                _check(rc, "wfst_decode_lattice_arcs")
                return n.value
            out = np.zeros(max(cap, 1), LAT_DTYPE)
            rc = lib().wfst_decode_lattice_arcs(self.h, channel, from_frame, out.ctypes.data, cap, C.byref(n), 0)
            if rc == WFST_E_CAPACITY:
                cap = n.value
                continue
            _check(rc, "wfst_decode_lattice_arcs")
            return out[:n.value].copy()

    def lattice_arcs_batch(self, channels, cap: int = 1 << 20, out_device=None):
        """Drains several channels: (records, offsets) on the host, or offsets only when the
        records go into the cuda tensor `out_device`."""
        fn = lib().wfst_decode_lattice_arcs_batch
        ch = np.ascontiguousarray(channels, np.int32)
        offs = np.zeros(len(ch) + 1, np.int64)
        while True:
            if out_device is not None:
                cap = out_device.numel() * out_device.element_size() // LAT_DTYPE.itemsize
                _check(fn(self.h, ch.ctypes.data, len(ch), out_device.data_ptr(), cap, offs.ctypes.data, 1),
                       "wfst_decode_lattice_arcs_batch")
                return offs
            out = np.zeros(max(cap, 1), LAT_DTYPE)
            rc = fn(self.h, ch.ctypes.data, len(ch), out.ctypes.data, cap, offs.ctypes.data, 0)
            if rc == WFST_E_CAPACITY:
                cap = int(offs[-1])
                continue
            _check(rc, "wfst_decode_lattice_arcs_batch")
            return out[:offs[-1]].copy(), offs

    def snapshot_lattice_arcs(self, snapshot: int, channels, out_device=None, copy: bool = True, cap: int = 1 << 20,
                              out_host=None):
        """Lattice arcs of a sealed snapshot: dict(starts, counts, total, block) and, with copy,
        `records`: the snapshot's block on the host, or None when it went into the cuda tensor
        `out_device` or into `out_host` (a CPU tensor, e.g. pinned, that the caller reuses).
        block = device address of the decoder's own block."""
        ch = np.ascontiguousarray(channels, np.int32)
        n = len(ch)
        starts, counts = np.zeros(n, np.int64), np.zeros(n, np.int64)
        total, block = C.c_int64(), C.c_void_p()
        fn = lib().wfst_decode_snapshot_lattice_arcs
        while True:
            out, ptr, dev = None, None, 0
            if copy and out_device is not None:
                cap, ptr, dev = out_device.numel() * out_device.element_size() // LAT_DTYPE.itemsize, out_device.data_ptr(), 1
            elif copy and out_host is not None:
                cap, ptr = out_host.numel() * out_host.element_size() // LAT_DTYPE.itemsize, out_host.data_ptr()
            elif copy:
                out = np.zeros(max(cap, 1), LAT_DTYPE)
                ptr = out.ctypes.data
            rc = fn(self.h, snapshot, ch.ctypes.data, n, starts.ctypes.data, counts.ctypes.data, ptr, cap, dev,
                    C.byref(total), C.byref(block))
            if rc == WFST_E_CAPACITY and out is not None:
                cap = total.value
                continue
            _check(rc, "wfst_decode_snapshot_lattice_arcs")
            return dict(starts=starts, counts=counts, total=total.value, block=block.value,
                        records=None if out is None else out[:total.value].copy())

    def final_lattice(self, channel: int, use_final: bool = True, cap: int = 1 << 16):
        """(kept arcs as a structured array, info dict) of wfst_decode_final_lattice."""
        while True:
            out = np.zeros(max(cap, 1), LAT_DTYPE)
            n, info = C.c_int64(), wfst_lattice_info_t()
            rc = lib().wfst_decode_final_lattice(self.h, channel, int(use_final), out.ctypes.data, cap, C.byref(n), 0,
                                                 C.byref(info))
            if rc == WFST_E_CAPACITY:
                cap = n.value
                continue
            _check(rc, "wfst_decode_final_lattice")
            return out[:n.value].copy(), {k: getattr(info, k) for k, _ in wfst_lattice_info_t._fields_}

    def final_lattice_batch(self, channels, use_final: bool = True, cap: int = 1 << 20):
        """wfst_decode_final_lattice_batch with HOST output: (records, offsets int64[n+1], infos (list of dicts),
        status int32[n])."""
        ch = np.ascontiguousarray(channels, np.int32)
        n = len(ch)
        while True:
            out = np.zeros(max(cap, 1), LAT_DTYPE)
            offs, st = np.zeros(n + 1, np.int64), np.zeros(n, np.int32)
            info = (wfst_lattice_info_t * max(n, 1))()
            rc = lib().wfst_decode_final_lattice_batch(self.h, ch.ctypes.data, n, int(use_final), out.ctypes.data, cap,
                                                       offs.ctypes.data, 0, C.cast(info, C.c_void_p), st.ctypes.data)
            if rc == WFST_E_CAPACITY:
                cap = int(offs[n])
                continue
            _check(rc, "wfst_decode_final_lattice_batch")
            infos = [{k: getattr(info[i], k) for k, _ in wfst_lattice_info_t._fields_} for i in range(n)]
            return out[:offs[n]].copy(), offs, infos, st

    def final_lattice_device(self, channel: int, use_final: bool, out_ptr: int, cap: int, noalloc: bool = False):
        """wfst_decode_final_lattice with DEVICE output (out_ptr: device address of cap records), or its
        allocation-free variant: (number of kept arcs, info dict).  Raises WfstError (also for WFST_E_CAPACITY)."""
        n, info = C.c_int64(), wfst_lattice_info_t()
        if noalloc:
            rc = lib().wfst_decode_final_lattice_noalloc(self.h, channel, int(use_final), out_ptr, cap, C.byref(n), C.byref(info))
        else:
            rc = lib().wfst_decode_final_lattice(self.h, channel, int(use_final), out_ptr, cap, C.byref(n), 1, C.byref(info))
        _check(rc, "wfst_decode_final_lattice_noalloc" if noalloc else "wfst_decode_final_lattice")
        return n.value, {k: getattr(info, k) for k, _ in wfst_lattice_info_t._fields_}

    def tokens(self, channel: int, frame: int = -1, cap: int = 1 << 14):
        while True:
            out = np.zeros(max(cap, 1), TOK_DTYPE)
            n = C.c_int32()
            rc = lib().wfst_decode_tokens(self.h, channel, frame, out.ctypes.data, cap, C.byref(n))
            if rc == WFST_E_CAPACITY:
                cap = n.value
                continue
            _check(rc, "wfst_decode_tokens")
            return out[:n.value].copy()

    def stats(self, channel: int) -> dict:
        s = wfst_stats_t()
        _check(lib().wfst_decode_stats(self.h, channel, C.byref(s)), "wfst_decode_stats")
        return {k: getattr(s, k) for k, _ in wfst_stats_t._fields_}

    def set_profiling(self, on: bool) -> None:
        _check(lib().wfst_decode_set_profiling(self.h, int(on)), "wfst_decode_set_profiling")

    def profile(self):
        n, ms = C.c_int64(), C.c_double()
        _check(lib().wfst_decode_profile(self.h, C.byref(n), C.byref(ms)), "wfst_decode_profile")
        return n.value, ms.value


class WfstMux:
    """wfst_mux_*: the channel-to-lane multiplexer over one decoder, one method per C entry point."""

    def __init__(self, decoder: WfstDecoder):
        self.decoder = decoder                      # keeps the decoder alive
        self.h = C.c_void_p()
        _check(lib().wfst_mux_create(decoder.h, C.byref(self.h)), "wfst_mux_create")

    def destroy(self):
        if self.h:
            lib().wfst_mux_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def submit(self, channel: int, ptr: int, stride: int, n_frames: int) -> None:
        """ptr: device address of the chunk's first row."""
        _check(lib().wfst_mux_submit(self.h, channel, C.c_void_p(ptr), stride, n_frames), "wfst_mux_submit")

    def step(self, stream: int = 0) -> int:
        n = C.c_int32()
        _check(lib().wfst_mux_step(self.h, C.c_void_p(stream), C.byref(n)), "wfst_mux_step")
        return n.value

    def pending(self) -> int:
        return int(lib().wfst_mux_pending(self.h))

    def stats(self):
        a, b = C.c_int64(), C.c_int64()
        _check(lib().wfst_mux_stats(self.h, C.byref(a), C.byref(b)), "wfst_mux_stats")
        return a.value, b.value
