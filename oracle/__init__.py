"""ctypes front end of the CPU oracle (oracle/laser_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the GPU package.  This module marshals
numpy arrays and nothing else; every routing step runs in the C file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "laser_oracle.c")
_LIB = os.path.join(_HERE, "liblaser_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: the binary32 decision
    arithmetic must not be fused behind the code's back."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fPIC",
               "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32, f32, f64, vp = ctypes.c_int32, ctypes.c_float, ctypes.c_double, ctypes.c_void_p
        lib.laser_oracle_gate.argtypes = [vp, vp, i32, i32, i32, i32, vp]
        lib.laser_oracle_gate.restype = ctypes.c_int
        lib.laser_oracle_exp.argtypes = [f32]
        lib.laser_oracle_exp.restype = f32
        lib.laser_oracle_tree_sum.argtypes = [vp, i32]
        lib.laser_oracle_tree_sum.restype = f32
        lib.laser_oracle_route.argtypes = [vp, i32, i32, i32, i32, f32, f32, i32,
                                           vp, vp, vp, vp, vp, vp, vp, vp]
        lib.laser_oracle_route.restype = ctypes.c_int
        lib.laser_oracle_route_literal.argtypes = [vp, i32, i32, i32, i32, f64, f64, i32,
                                                   vp, vp, vp, vp, vp, vp, vp, vp]
        lib.laser_oracle_route_literal.restype = ctypes.c_int
        u32, u64 = ctypes.c_uint32, ctypes.c_uint64
        lib.laser_oracle_philox4x32.argtypes = [vp, vp, vp]
        lib.laser_oracle_philox4x32.restype = None
        lib.laser_oracle_sample_ranks.argtypes = [i32, i32, u64, u32, u64, vp]
        lib.laser_oracle_sample_ranks.restype = None
        lib.laser_oracle_route_random.argtypes = [vp, i32, i32, i32, i32, f32, f32, i32, u64, u32, u64,
                                                  vp, vp, vp, vp, vp, vp, vp, vp]
        lib.laser_oracle_route_random.restype = ctypes.c_int
        lib.laser_oracle_token_stats.argtypes = [vp, i32, i32, i32, f32, vp, vp, vp]
        lib.laser_oracle_token_stats.restype = ctypes.c_int
        lib.laser_oracle_imbalance.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp, vp, vp]
        lib.laser_oracle_imbalance.restype = ctypes.c_int
        lib.laser_oracle_percentiles.argtypes = [vp, i32, vp, i32, vp]
        lib.laser_oracle_percentiles.restype = ctypes.c_int
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def gate(hidden: np.ndarray, w_gate: np.ndarray, dtype: int) -> np.ndarray:
    """fp64 logits [T,E].  dtype 0: float32 arrays; 1: uint16 bf16 bit patterns."""
    want = np.uint16 if dtype == 1 else np.float32
    hidden = np.ascontiguousarray(hidden, dtype=want)
    w_gate = np.ascontiguousarray(w_gate, dtype=want)
    T, H = hidden.shape
    E = w_gate.shape[0]
    assert w_gate.shape[1] == H
    out = np.empty((T, E), dtype=np.float64)
    rc = _load().laser_oracle_gate(_ptr(hidden), _ptr(w_gate), T, H, E, dtype, _ptr(out))
    if rc:
        raise ValueError(f"laser_oracle_gate: {rc}")
    return out


def exp_canon(x: float) -> float:
    return float(_load().laser_oracle_exp(np.float32(x)))


def tree_sum(v: np.ndarray) -> float:
    v = np.ascontiguousarray(v, dtype=np.float32)
    return float(_load().laser_oracle_tree_sum(_ptr(v), v.size))


def _route(fn, logits, ldtype, k, c, eps_high, t_fix, loads_in, renormalize):
    logits = np.ascontiguousarray(logits, dtype=ldtype)
    T, E = logits.shape
    loads_in = np.ascontiguousarray(loads_in, dtype=np.int32)
    assert loads_in.shape == (E,)
    out = {
        "loads": np.empty(E, dtype=np.int32),
        "expert_ids": np.empty((T, k), dtype=np.int32),
        "weights": np.empty((T, k), dtype=np.float64),
        "permutation": np.empty(T * k, dtype=np.int32),
        "expert_offsets": np.empty(E + 1, dtype=np.int32),
        "expanded": np.empty(T, dtype=np.uint8),
        "cstar": np.empty(T, dtype=np.int32),
    }
    rc = fn(_ptr(logits), T, E, k, c, eps_high, t_fix, int(bool(renormalize)),
            _ptr(loads_in), _ptr(out["loads"]), _ptr(out["expert_ids"]),
            _ptr(out["weights"]), _ptr(out["permutation"]), _ptr(out["expert_offsets"]),
            _ptr(out["expanded"]), _ptr(out["cstar"]))
    if rc:
        raise ValueError(f"oracle route: bad arguments ({rc})")
    return out


def route(logits, k, c, eps_high, t_fix, loads_in, renormalize=True):
    """Router with binary32 decisions on fp32 logits [T,E]; returns a dict."""
    return _route(_load().laser_oracle_route, logits, np.float32, k, c,
                  float(np.float32(eps_high)), float(np.float32(t_fix)), loads_in, renormalize)


def route_literal(logits, k, c, eps_high, t_fix, loads_in, renormalize=True):
    """Router in fp64 with the paper's formulas as printed, on fp64 logits."""
    return _route(_load().laser_oracle_route_literal, logits, np.float64, k, c,
                  float(eps_high), float(t_fix), loads_in, renormalize)


def philox4x32(ctr, key):
    """Philox4x32-10 block: 4 counter words, 2 key words -> 4 output words."""
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and k.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    _load().laser_oracle_philox4x32(_ptr(c), _ptr(k), _ptr(out))
    return out


def sample_ranks(m, c, seed, stream, token):
    """The c sampled positions of a pool of m (c < m), ascending."""
    assert 0 < c < m <= 256
    out = np.empty(c, dtype=np.int32)
    _load().laser_oracle_sample_ranks(m, c, seed, stream, token, _ptr(out))
    return out


def route_random(logits, k, c, eps_high, t_fix, loads_in, seed, stream=0, token_offset=0,
                 renormalize=True):
    """Router with RANDOM trimming (binary32 decisions); returns a dict as route()."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    loads_in = np.ascontiguousarray(loads_in, dtype=np.int32)
    assert loads_in.shape == (E,)
    out = {
        "loads": np.empty(E, dtype=np.int32),
        "expert_ids": np.empty((T, k), dtype=np.int32),
        "weights": np.empty((T, k), dtype=np.float64),
        "permutation": np.empty(T * k, dtype=np.int32),
        "expert_offsets": np.empty(E + 1, dtype=np.int32),
        "expanded": np.empty(T, dtype=np.uint8),
        "cstar": np.empty(T, dtype=np.int32),
    }
    rc = _load().laser_oracle_route_random(
        _ptr(logits), T, E, k, c, float(np.float32(eps_high)), float(np.float32(t_fix)),
        int(bool(renormalize)), seed, stream, token_offset, _ptr(loads_in), _ptr(out["loads"]),
        _ptr(out["expert_ids"]), _ptr(out["weights"]), _ptr(out["permutation"]),
        _ptr(out["expert_offsets"]), _ptr(out["expanded"]), _ptr(out["cstar"]))
    if rc:
        raise ValueError(f"oracle route_random: bad arguments ({rc})")
    return out


def token_stats(logits, k, t_fix):
    """Per-token top-k mass, Shannon entropy (nats) and pool size from fp32 logits."""
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    out = {"topk_mass": np.empty(T, dtype=np.float64), "entropy": np.empty(T, dtype=np.float64),
           "pool_size": np.empty(T, dtype=np.int32)}
    rc = _load().laser_oracle_token_stats(_ptr(logits), T, E, k, float(np.float32(t_fix)),
                                          _ptr(out["topk_mass"]), _ptr(out["entropy"]),
                                          _ptr(out["pool_size"]))
    if rc:
        raise ValueError(f"oracle token_stats: bad arguments ({rc})")
    return out


def imbalance(counts, placement=None, weights=None):
    """Imbalance factor, max violation, GPU-level imbalance per layer and the aggregates."""
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    L, E = counts.shape
    G = 0
    pl = wt = None
    if placement is not None:
        pl = np.ascontiguousarray(placement, dtype=np.float64)
        G = pl.shape[0]
        assert pl.shape == (G, E)
    if weights is not None:
        wt = np.ascontiguousarray(weights, dtype=np.float64)
        assert wt.shape == (L,)
    out = {"I": np.empty(L), "MV": np.empty(L), "I_gpu": np.empty(L), "agg": np.empty(2)}
    rc = _load().laser_oracle_imbalance(_ptr(counts), L, E, None if pl is None else _ptr(pl), G,
                                        None if wt is None else _ptr(wt), _ptr(out["I"]),
                                        _ptr(out["MV"]), _ptr(out["I_gpu"]), _ptr(out["agg"]))
    if rc:
        raise ValueError(f"oracle imbalance: bad arguments ({rc})")
    return out


def percentiles(values, q):
    """q-th percentiles (q in [0, 100]) of a 1-D array, linear interpolation between ranks."""
    v = np.ascontiguousarray(values, dtype=np.float64).ravel()
    qq = np.ascontiguousarray(q, dtype=np.float64).ravel()
    out = np.empty(len(qq))
    rc = _load().laser_oracle_percentiles(_ptr(v), len(v), _ptr(qq), len(qq), _ptr(out))
    if rc:
        raise ValueError(f"oracle percentiles: bad arguments ({rc})")
    return out


def route_from_hidden(hidden, w_gate, dtype, k, c, eps_high, t_fix, loads_in, renormalize=True):
    """Gate in fp64, rounded once to fp32, then route()."""
    z = gate(hidden, w_gate, dtype)
    out = route(z.astype(np.float32), k, c, eps_high, t_fix, loads_in, renormalize)
    out["logits"] = z
    return out
