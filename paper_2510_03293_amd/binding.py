"""Thin ctypes binding of liblaser_route.so (the C ABI in include/laser.h).

Argument marshalling only: torch supplies device memory and the stream; every
step of the routing path runs in the library's HIP kernels.  There is no CPU
fallback: if the library has not been built, importing the binding raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblaser_route.so")

DTYPE_F32 = 0
DTYPE_BF16 = 1
TRIM_TOP = 0
TRIM_RANDOM = 1

# include/laser.h
EXPORTS = ("laser_workspace_bytes", "laser_route", "laser_route_batched", "laser_route_stats",
           "laser_route_from_logits", "laser_imbalance", "laser_percentiles", "laser_summary_f32",
           "laser_strerror", "laser_status", "laser_static_workspace_bytes", "laser_route_static",
           "laser_status_static")
# include/laser_bench.h
BENCH_EXPORTS = ("laser_bench_timer_create", "laser_bench_timer_destroy", "laser_bench_route",
                 "laser_bench_timer_read", "laser_bench_event_overhead", "laser_bench_plain_read")

STATUS_COMPLETE = 0
STATUS_TIMEOUT = 1
STATUS_INCONSISTENT = 2


class LaserParams(ctypes.Structure):
    _fields_ = [
        ("struct_bytes", ctypes.c_uint32),
        ("k", ctypes.c_int32),
        ("c", ctypes.c_int32),
        ("eps_high", ctypes.c_float),
        ("t_fix", ctypes.c_float),
        ("trim_mode", ctypes.c_int32),
        ("renormalize", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("seed", ctypes.c_uint64),
        ("token_offset", ctypes.c_uint64),
        ("stream", ctypes.c_uint32),
        ("poll_budget", ctypes.c_uint32),
        ("pipeline_tiles", ctypes.c_uint32),
        ("split_k", ctypes.c_uint32),
    ]


class LaserError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"laser: {text} (code {code})")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -m paper_2510_03293_amd.build "
            "or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    pp = ctypes.POINTER(LaserParams)
    lib.laser_workspace_bytes.argtypes = [i32, i32, i32, pp]
    lib.laser_workspace_bytes.restype = sz
    lib.laser_route.argtypes = [vp, vp, i32, i32, i32, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.laser_route.restype = ctypes.c_int
    lib.laser_route_batched.argtypes = [vp, vp, i32, i32, i32, i32, pp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.laser_route_batched.restype = ctypes.c_int
    lib.laser_route_stats.argtypes = [vp, vp, i32, i32, i32, pp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                      vp, sz, vp]
    lib.laser_route_stats.restype = ctypes.c_int
    lib.laser_imbalance.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.laser_imbalance.restype = ctypes.c_int
    lib.laser_percentiles.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), i32, vp, vp]
    lib.laser_percentiles.restype = ctypes.c_int
    lib.laser_summary_f32.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), i32, vp, vp, vp]
    lib.laser_summary_f32.restype = ctypes.c_int
    lib.laser_route_from_logits.argtypes = [vp, i32, i32, pp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.laser_route_from_logits.restype = ctypes.c_int
    lib.laser_strerror.argtypes = [ctypes.c_int]
    lib.laser_strerror.restype = ctypes.c_char_p
    lib.laser_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.laser_status.restype = ctypes.c_int
    lib.laser_static_workspace_bytes.argtypes = []
    lib.laser_static_workspace_bytes.restype = sz
    lib.laser_route_static.argtypes = [vp, vp, i32, i32, i32, pp, vp, vp, vp, vp, vp, vp, vp]
    lib.laser_route_static.restype = ctypes.c_int
    lib.laser_status_static.argtypes = [vp, ctypes.POINTER(ctypes.c_int32)]
    lib.laser_status_static.restype = ctypes.c_int
    lib.laser_bench_timer_create.argtypes = [i32, ctypes.POINTER(vp)]
    lib.laser_bench_timer_create.restype = ctypes.c_int
    lib.laser_bench_timer_destroy.argtypes = [vp]
    lib.laser_bench_timer_destroy.restype = None
    lib.laser_bench_route.argtypes = [vp] + lib.laser_route.argtypes
    lib.laser_bench_route.restype = ctypes.c_int
    lib.laser_bench_timer_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                           ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
    lib.laser_bench_timer_read.restype = ctypes.c_int
    lib.laser_bench_event_overhead.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
    lib.laser_bench_event_overhead.restype = ctypes.c_int
    lib.laser_bench_plain_read.argtypes = [vp, sz, sz, vp, vp, ctypes.POINTER(ctypes.c_double),
                                           ctypes.POINTER(ctypes.c_int64)]
    lib.laser_bench_plain_read.restype = ctypes.c_int
    return lib


_lib = _load()


def make_params(k: int, c: int, eps_high: float, t_fix: float, dtype: int = DTYPE_BF16,
                renormalize: bool = True, trim_mode: int = TRIM_TOP, seed: int = 0,
                stream: int = 0, token_offset: int = 0, poll_budget: int = 0,
                pipeline_tiles: int = 0, split_k: int = 0) -> LaserParams:
    return LaserParams(ctypes.sizeof(LaserParams), k, c, eps_high, t_fix, trim_mode,
                       1 if renormalize else 0, dtype, seed, token_offset, stream, poll_budget,
                       pipeline_tiles, split_k)


def laser_strerror(code: int) -> str:
    return _lib.laser_strerror(code).decode()


def _check(code: int) -> None:
    if code != 0:
        raise LaserError(code, laser_strerror(code))


def laser_workspace_bytes(T: int, H: int, E: int, params: LaserParams) -> int:
    return int(_lib.laser_workspace_bytes(T, H, E, ctypes.byref(params)))


def _ptr(t: torch.Tensor | None):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def laser_route(hidden, w_gate, T, H, E, params, loads_inout, expert_ids, weights,
                permutation, expert_offsets, logits_out, workspace, stream=None) -> None:
    """Enqueue one layer's routing step; tensors are device tensors (see laser.h)."""
    _check(_lib.laser_route(_ptr(hidden), _ptr(w_gate), T, H, E, ctypes.byref(params),
                            _ptr(loads_inout), _ptr(expert_ids), _ptr(weights), _ptr(permutation),
                            _ptr(expert_offsets), _ptr(logits_out), _ptr(workspace),
                            workspace.numel() * workspace.element_size(), _stream_handle(stream)))


def laser_route_batched(hidden, w_gate, B, T, H, E, params, loads_inout, expert_ids, weights,
                        permutation, expert_offsets, logits_out, workspace, stream=None) -> None:
    """B independent problems of one size in one call; every tensor has a leading dimension B."""
    _check(_lib.laser_route_batched(_ptr(hidden), _ptr(w_gate), B, T, H, E, ctypes.byref(params),
                                    _ptr(loads_inout), _ptr(expert_ids), _ptr(weights),
                                    _ptr(permutation), _ptr(expert_offsets), _ptr(logits_out),
                                    _ptr(workspace),
                                    0 if workspace is None else workspace.numel() * workspace.element_size(),
                                    _stream_handle(stream)))


def laser_route_stats(hidden, w_gate, T, H, E, params, loads_inout, expert_ids, weights,
                      permutation, expert_offsets, logits_out, topk_mass, entropy, pool_size,
                      workspace, stream=None) -> None:
    """laser_route plus per-token top-k mass, entropy and pool size (each may be None)."""
    _check(_lib.laser_route_stats(_ptr(hidden), _ptr(w_gate), T, H, E, ctypes.byref(params),
                                  _ptr(loads_inout), _ptr(expert_ids), _ptr(weights),
                                  _ptr(permutation), _ptr(expert_offsets), _ptr(logits_out),
                                  _ptr(topk_mass), _ptr(entropy), _ptr(pool_size), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(),
                                  _stream_handle(stream)))


def laser_route_from_logits(logits, T, E, params, loads_inout, expert_ids, weights,
                            permutation, expert_offsets, workspace, stream=None) -> None:
    _check(_lib.laser_route_from_logits(_ptr(logits), T, E, ctypes.byref(params),
                                        _ptr(loads_inout), _ptr(expert_ids), _ptr(weights),
                                        _ptr(permutation), _ptr(expert_offsets), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(),
                                        _stream_handle(stream)))


def laser_imbalance(counts, placement=None, layer_weights=None, stream=None):
    """Imbalance metrics of device counts [L,E] (int32): dict of device fp64 tensors."""
    L, E = counts.shape
    G = 0 if placement is None else placement.shape[0]
    dev = counts.device
    out = {"I": torch.empty(L, dtype=torch.float64, device=dev),
           "MV": torch.empty(L, dtype=torch.float64, device=dev),
           "I_gpu": torch.empty(L, dtype=torch.float64, device=dev),
           "agg": torch.empty(2, dtype=torch.float64, device=dev)}
    _check(_lib.laser_imbalance(_ptr(counts), L, E, _ptr(placement), G, _ptr(layer_weights),
                                _ptr(out["I"]), _ptr(out["MV"]), _ptr(out["I_gpu"]),
                                _ptr(out["agg"]), _stream_handle(stream)))
    return out


def laser_percentiles(values, q, stream=None):
    """q-th percentiles (host sequence, each in [0, 100]) of a device fp64 vector; device fp64 [len(q)]."""
    qs = [float(x) for x in q]
    qa = (ctypes.c_double * max(len(qs), 1))(*qs)
    out = torch.empty(len(qs), dtype=torch.float64, device=values.device)
    _check(_lib.laser_percentiles(_ptr(values), values.numel(), qa, len(qs), _ptr(out),
                                  _stream_handle(stream)))
    return out


def laser_summary_f32(values, q, stream=None):
    """(mean, percentiles) of a device fp32 vector: device fp64 scalar and fp64 [len(q)]."""
    qs = [float(x) for x in q]
    qa = (ctypes.c_double * max(len(qs), 1))(*qs)
    mean = torch.empty((), dtype=torch.float64, device=values.device)
    out = torch.empty(len(qs), dtype=torch.float64, device=values.device)
    _check(_lib.laser_summary_f32(_ptr(values), values.numel(), qa, len(qs), _ptr(mean), _ptr(out),
                                  _stream_handle(stream)))
    return mean, out


def laser_status(workspace, stream=None) -> int:
    """STATUS_* of the last call that used `workspace` (waits for the stream)."""
    st = ctypes.c_int32(-1)
    _check(_lib.laser_status(_ptr(workspace), _stream_handle(stream), ctypes.byref(st)))
    return st.value


def laser_static_workspace_bytes() -> int:
    return int(_lib.laser_static_workspace_bytes())


def laser_route_static(hidden, w_gate, T, H, E, params, loads_inout, expert_ids, weights,
                       permutation, expert_offsets, logits_out, stream=None) -> None:
    """laser_route on the library's own per-GPU workspace (nothing is allocated)."""
    _check(_lib.laser_route_static(_ptr(hidden), _ptr(w_gate), T, H, E, ctypes.byref(params),
                                   _ptr(loads_inout), _ptr(expert_ids), _ptr(weights), _ptr(permutation),
                                   _ptr(expert_offsets), _ptr(logits_out), _stream_handle(stream)))


def laser_status_static(stream=None) -> int:
    st = ctypes.c_int32(-1)
    _check(_lib.laser_status_static(_stream_handle(stream), ctypes.byref(st)))
    return st.value


class BenchTimer:
    """Event pool of include/laser_bench.h: times the stages of laser_bench_route calls."""

    def __init__(self, max_calls: int):
        self.capacity = max_calls
        self._h = ctypes.c_void_p()
        _check(_lib.laser_bench_timer_create(max_calls, ctypes.byref(self._h)))

    def route(self, hidden, w_gate, T, H, E, params, loads_inout, expert_ids, weights, permutation,
              expert_offsets, logits_out, workspace, stream=None) -> None:
        _check(_lib.laser_bench_route(self._h, _ptr(hidden), _ptr(w_gate), T, H, E, ctypes.byref(params),
                                      _ptr(loads_inout), _ptr(expert_ids), _ptr(weights),
                                      _ptr(permutation), _ptr(expert_offsets), _ptr(logits_out),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _stream_handle(stream)))

    def read(self):
        """(first_ms, tail_ms): per timed call, projection + analysis and tail kernel (lists)."""
        a = (ctypes.c_double * self.capacity)()
        b = (ctypes.c_double * self.capacity)()
        n = ctypes.c_int64(0)
        _check(_lib.laser_bench_timer_read(self._h, a, b, self.capacity, ctypes.byref(n)))
        return list(a[:n.value]), list(b[:n.value])

    def close(self) -> None:
        if self._h:
            _lib.laser_bench_timer_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def laser_bench_event_overhead(stream=None) -> float:
    """Milliseconds a HIP event pair adds to the kernel it brackets (measured now)."""
    ms = ctypes.c_double(0.0)
    _check(_lib.laser_bench_event_overhead(_stream_handle(stream), ctypes.byref(ms)))
    return ms.value


def laser_bench_plain_read(buf, bytes_per_launch: int, sink, stream=None):
    """(milliseconds, launches) of a plain streaming read of `buf` in pieces."""
    ms = ctypes.c_double(0.0)
    n = ctypes.c_int64(0)
    nbytes = buf.numel() * buf.element_size()
    _check(_lib.laser_bench_plain_read(
        ctypes.c_void_p(buf.data_ptr()), ctypes.c_size_t(nbytes), ctypes.c_size_t(bytes_per_launch),
        ctypes.c_void_p(sink.data_ptr()), _stream_handle(stream), ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


class RouteBuffers:
    """Output and workspace tensors for calls of one size, allocated once."""

    def __init__(self, T: int, H: int, E: int, params: LaserParams, device="cuda",
                 want_logits: bool = False):
        self.T, self.H, self.E, self.k = T, H, E, params.k
        nbytes = laser_workspace_bytes(T, H, E, params)
        if nbytes == 0:
            raise LaserError(-2, "laser_workspace_bytes rejected the arguments")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.expert_ids = torch.empty((T, params.k), dtype=torch.int32, device=device)
        self.weights = torch.empty((T, params.k), dtype=torch.float32, device=device)
        self.permutation = torch.empty(T * params.k, dtype=torch.int32, device=device)
        self.expert_offsets = torch.empty(E + 1, dtype=torch.int32, device=device)
        self.logits = torch.empty((T, E), dtype=torch.float32, device=device) if want_logits else None


def route(hidden, w_gate, params: LaserParams, loads_inout, buffers: RouteBuffers | None = None,
          want_logits: bool = False, stream=None) -> RouteBuffers:
    """Convenience wrapper: shapes from the tensors, buffers allocated if not given."""
    T, H = hidden.shape
    E = w_gate.shape[0]
    if buffers is None:
        buffers = RouteBuffers(T, H, E, params, device=hidden.device, want_logits=want_logits)
    laser_route(hidden, w_gate, T, H, E, params, loads_inout, buffers.expert_ids, buffers.weights,
                buffers.permutation, buffers.expert_offsets, buffers.logits, buffers.workspace,
                stream)
    return buffers


def route_from_logits(logits, params: LaserParams, loads_inout,
                      buffers: RouteBuffers | None = None, stream=None) -> RouteBuffers:
    T, E = logits.shape
    if buffers is None:
        buffers = RouteBuffers(T, 0, E, params, device=logits.device)
    laser_route_from_logits(logits, T, E, params, loads_inout, buffers.expert_ids, buffers.weights,
                            buffers.permutation, buffers.expert_offsets, buffers.workspace, stream)
    return buffers
