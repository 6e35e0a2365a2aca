"""Seeded synthetic WFST graphs and log-likelihood rows (inputs only, no decoder arithmetic).

Shared by the CPU checker's tests and by the GPU library's tests and benchmark, so that
both decode byte-identical inputs.  The host generator is plain C (wfst_synth.c), loaded
through ctypes; `device_loglikes` fills a torch tensor on the GPU with the same bytes.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_HOST_SO = os.path.join(_DIR, "_libwfst_synth.so")
_DEV_SO = os.path.join(_DIR, "_libwfst_synth_hip.so")


def build_host(force: bool = False) -> str:
    """Compile the host generator with gcc."""
    src = os.path.join(_DIR, "wfst_synth.c")
    if force or not os.path.exists(_HOST_SO) or os.path.getmtime(_HOST_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fPIC", "-shared", "-o", _HOST_SO, src, "-lm"])
    return _HOST_SO


def build_device(force: bool = False) -> str:
    """Compile the device log-likelihood generator and the measurement probes for gfx950."""
    srcs = [os.path.join(_DIR, "loglikes.hip"), os.path.join(_DIR, "probes.hip")]
    if force or not os.path.exists(_DEV_SO) or os.path.getmtime(_DEV_SO) < max(os.path.getmtime(p) for p in srcs):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-ffp-contract=off",
                               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                               "-fPIC", "-shared", "-o", _DEV_SO] + srcs)
    return _DEV_SO


class _Spec(C.Structure):
    _fields_ = [("seed", C.c_uint64), ("num_states", C.c_int32), ("num_emit", C.c_int64),
                ("num_eps", C.c_int64), ("degree_model", C.c_int32), ("deg_param", C.c_double),
                ("deg_max", C.c_int32), ("num_pdfs", C.c_int32), ("vocab", C.c_int32),
                ("weight_max", C.c_float), ("num_final", C.c_int32), ("final_max", C.c_float),
                ("interleave", C.c_int32)]


_host = None
_dev = None


def _lib():
    global _host
    if _host is None:
        if not os.path.exists(_HOST_SO):
            build_host()
        _host = C.CDLL(_HOST_SO)
        _host.synth_graph_num_arcs.argtypes = [C.POINTER(_Spec), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        _host.synth_graph_fill.argtypes = [C.POINTER(_Spec)] + [C.c_void_p] * 6
        _host.synth_stream_length.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        _host.synth_stream_length.restype = C.c_int32
        _host.synth_true_pdf.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32]
        _host.synth_true_pdf.restype = C.c_int32
        _host.synth_loglikes_fill.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                              C.c_float, C.c_float, C.c_float, C.c_void_p, C.c_int64]
    return _host


@dataclass
class Graph:
    """A decoding WFST in CSR form (host numpy arrays)."""
    num_states: int
    num_arcs: int
    start_state: int
    num_pdfs: int
    row_offsets: np.ndarray   # int64 [num_states+1]
    ilabel: np.ndarray        # int32 [num_arcs], 0 = epsilon, else pdf+1
    olabel: np.ndarray        # int32 [num_arcs], 0 = none
    weight: np.ndarray        # float32 [num_arcs]
    nextstate: np.ndarray     # int32 [num_arcs]
    final_cost: np.ndarray    # float32 [num_states], +inf = not final

    @property
    def num_emit(self) -> int:
        return int(np.count_nonzero(self.ilabel))


@dataclass
class GraphSpec:
    seed: int
    num_states: int
    num_emit: int             # 0 = natural total of the degree model
    num_eps: int              # <0 = that fraction (in percent) of the emitting count
    degree_model: str         # "fixed" | "geometric" | "powerlaw"
    deg_param: float
    deg_max: int
    num_pdfs: int
    vocab: int
    weight_max: float
    num_final: int
    final_max: float = 4.0
    interleave: bool = False

    def _c(self, num_eps: int) -> _Spec:
        model = {"fixed": 0, "geometric": 1, "powerlaw": 2}[self.degree_model]
        return _Spec(self.seed, self.num_states, self.num_emit, num_eps, model, self.deg_param,
                     self.deg_max, self.num_pdfs, self.vocab, self.weight_max, self.num_final,
                     self.final_max, int(self.interleave))


def make_graph(spec: GraphSpec) -> Graph:
    lib = _lib()
    ne, na = C.c_int64(), C.c_int64()
    cs = spec._c(0)
    rc = lib.synth_graph_num_arcs(C.byref(cs), C.byref(ne), C.byref(na))
    if rc:
        raise RuntimeError(f"synth_graph_num_arcs failed ({rc})")
    num_eps = spec.num_eps if spec.num_eps >= 0 else (ne.value * (-spec.num_eps)) // 100
    cs = spec._c(num_eps)
    n_arcs = ne.value + num_eps
    off = np.empty(spec.num_states + 1, np.int64)
    il = np.empty(n_arcs, np.int32)
    ol = np.empty(n_arcs, np.int32)
    w = np.empty(n_arcs, np.float32)
    ns = np.empty(n_arcs, np.int32)
    fin = np.empty(spec.num_states, np.float32)
    rc = lib.synth_graph_fill(C.byref(cs), off.ctypes.data, il.ctypes.data, ol.ctypes.data,
                              w.ctypes.data, ns.ctypes.data, fin.ctypes.data)
    if rc:
        raise RuntimeError(f"synth_graph_fill failed ({rc})")
    return Graph(spec.num_states, n_arcs, 0, spec.num_pdfs, off, il, ol, w, ns, fin)


def stream_length(seed: int, stream: int, lo: int, hi: int) -> int:
    return int(_lib().synth_stream_length(seed, stream, lo, hi))


def true_pdf(seed: int, stream: int, frame: int, num_pdfs: int) -> int:
    return int(_lib().synth_true_pdf(seed, stream, frame, num_pdfs))


def host_loglikes(seed: int, stream: int, frame0: int, n_frames: int, num_pdfs: int,
                  mu: float, sigma: float, boost: float = 6.0) -> np.ndarray:
    """float32 [n_frames, num_pdfs] rows of one stream, generated on the host."""
    out = np.empty((n_frames, num_pdfs), np.float32)
    if n_frames:
        rc = _lib().synth_loglikes_fill(seed, stream, frame0, n_frames, num_pdfs, mu, sigma, boost,
                                        out.ctypes.data, num_pdfs)
        if rc:
            raise RuntimeError(f"synth_loglikes_fill failed ({rc})")
    return out


def _devlib():
    global _dev
    if _dev is None:
        if not os.path.exists(_DEV_SO):
            raise RuntimeError("device generator not built: run synth.build_device() (needs hipcc)")
        _dev = C.CDLL(_DEV_SO)
        _dev.synth_loglikes_device.argtypes = [C.c_uint64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                               C.c_float, C.c_float, C.c_float, C.c_void_p, C.c_int64,
                                               C.c_void_p]
        _dev.probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.POINTER(C.c_float)]
        _dev.probe_gather.argtypes = [C.c_void_p, C.c_uint32, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int,
                                      C.c_void_p, C.POINTER(C.c_float)]
    return _dev


def probe_copy_gbs(nbytes: int = 1 << 30, reps: int = 5) -> float:
    """Measured rate of a plain device copy of nbytes (read + written bytes per second, GB/s)."""
    import torch
    src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ms = C.c_float()
    rc = _devlib().probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, reps, torch.cuda.current_stream().cuda_stream, C.byref(ms))
    if rc:
        raise RuntimeError(f"probe_copy failed ({rc})")
    return 2.0 * nbytes / (ms.value * 1e-3) / 1e9


def probe_gather(table_bytes: int, lanes: int, threads: int, inflight: int = 4, steps: int = 64, reps: int = 3) -> dict:
    """12-byte records fetched at random from a table of table_bytes, lanes x threads threads with
    `inflight` independent loads each: records per second and the rate in 64-byte lines."""
    import torch
    n = table_bytes // 12
    table = torch.zeros(n * 3, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    ms = C.c_float()
    rc = _devlib().probe_gather(table.data_ptr(), n, lanes, threads, steps, inflight, sink.data_ptr(), reps,
                                torch.cuda.current_stream().cuda_stream, C.byref(ms))
    if rc:
        raise RuntimeError(f"probe_gather failed ({rc})")
    recs = lanes * threads * steps * max(1, (8 if inflight >= 8 else 4 if inflight >= 4 else 1))
    return dict(records_per_s=recs / (ms.value * 1e-3), line_gbs=recs * 64 / (ms.value * 1e-3) / 1e9,
                record_gbs=recs * 12 / (ms.value * 1e-3) / 1e9)


def device_loglikes(out, seed: int, stream: int, frame0: int, mu: float, sigma: float,
                    boost: float = 6.0) -> None:
    """Fill a contiguous float32 cuda tensor [n_frames, num_pdfs] with the same bytes as
    host_loglikes, on the tensor's device and the current torch stream."""
    import torch
    _devlib()
    assert out.is_cuda and out.dtype == torch.float32 and out.dim() == 2 and out.is_contiguous()
    n_frames, num_pdfs = out.shape
    if n_frames == 0:
        return
    rc = _devlib().synth_loglikes_device(seed, stream, frame0, n_frames, num_pdfs, mu, sigma, boost,
                                    out.data_ptr(), out.stride(0),
                                    torch.cuda.current_stream(out.device).cuda_stream)
    if rc:
        raise RuntimeError(f"synth_loglikes_device failed ({rc})")


@dataclass
class Config:
    """One workload: a graph recipe, decoding hyper-parameters and the stream mix."""
    name: str
    graph: GraphSpec
    beam: float
    max_active: int
    lattice_beam: float
    n_streams: int
    len_lo: int
    len_hi: int
    ll_mu: float
    ll_sigma: float
    chunk: int = 0            # frames per advance call (0 = whole stream at once)
    ll_boost: float = 6.0
    ll_seed: int = field(default=0)

    def __post_init__(self):
        if not self.ll_seed:
            self.ll_seed = self.graph.seed * 1000003 + 17

    def length(self, stream: int) -> int:
        return stream_length(self.ll_seed, stream, self.len_lo, self.len_hi)

    def loglikes(self, stream: int, frame0: int, n_frames: int) -> np.ndarray:
        return host_loglikes(self.ll_seed, stream, frame0, n_frames, self.graph.num_pdfs,
                             self.ll_mu, self.ll_sigma, self.ll_boost)


def configs() -> list[Config]:
    """The five workloads, index-aligned with the repository's benchmark spec.

    "N(m, v)" in the workload descriptions is read as mean m and VARIANCE v (the usual
    notation), so sigma is sqrt(3) for configs 0-1 and 2 for configs 2-4."""
    g0 = GraphSpec(seed=0, num_states=1000, num_emit=0, num_eps=-15, degree_model="fixed", deg_param=4,
                   deg_max=4, num_pdfs=200, vocab=500, weight_max=8.0, num_final=20)
    g1 = GraphSpec(seed=1, num_states=200_000, num_emit=0, num_eps=-15, degree_model="geometric",
                   deg_param=5.0, deg_max=64, num_pdfs=2000, vocab=20_000, weight_max=10.0, num_final=200)
    g2 = GraphSpec(seed=2, num_states=8_000_000, num_emit=20_000_000, num_eps=3_000_000,
                   degree_model="powerlaw", deg_param=2.2, deg_max=2000, num_pdfs=6000, vocab=200_000,
                   weight_max=12.0, num_final=8000)
    g4 = GraphSpec(seed=4, num_states=50_000_000, num_emit=150_000_000, num_eps=20_000_000,
                   degree_model="powerlaw", deg_param=2.2, deg_max=5000, num_pdfs=8000, vocab=500_000,
                   weight_max=14.0, num_final=50_000)
    return [
        Config("cfg0_tiny", g0, beam=12.0, max_active=2000, lattice_beam=6.0, n_streams=1,
               len_lo=300, len_hi=300, ll_mu=-10.0, ll_sigma=3.0 ** 0.5),
        Config("cfg1_mid", g1, beam=15.0, max_active=7000, lattice_beam=8.0, n_streams=1,
               len_lo=1000, len_hi=1000, ll_mu=-10.0, ll_sigma=3.0 ** 0.5),
        Config("cfg2_hclg_offline", g2, beam=15.0, max_active=10000, lattice_beam=8.0, n_streams=100,
               len_lo=500, len_hi=1500, ll_mu=-12.0, ll_sigma=2.0),
        Config("cfg3_hclg_online", g2, beam=13.0, max_active=7000, lattice_beam=6.0, n_streams=500,
               len_lo=2000, len_hi=2000, ll_mu=-12.0, ll_sigma=2.0, chunk=50, ll_seed=3_000_003 + 17),
        Config("cfg4_large_lm", g4, beam=16.0, max_active=15000, lattice_beam=8.0, n_streams=200,
               len_lo=1000, len_hi=3000, ll_mu=-12.0, ll_sigma=2.0),
    ]
