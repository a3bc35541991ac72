"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding and
compare with the CPU oracle on the same seeded inputs."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2510_03293_amd import binding as B
from synth import workloads as wl

TOL_LOGIT = {wl.DTYPE_BF16: 2e-3, wl.DTYPE_F32: 1e-5}   # max abs error, logits and weights


def to_device(arr: np.ndarray, dtype: int | None = None) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(arr))
    if arr.dtype == np.uint16:
        t = torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).view(torch.bfloat16)
    return t.cuda()


def run_route(hidden, w_gate, dtype, k, c, eps_high, t_fix, loads_in, renormalize=True,
              pipeline_tiles=0, split_k=0):
    """GPU laser_route on numpy inputs; returns a dict of numpy outputs incl. logits."""
    params = B.make_params(k, c, eps_high, t_fix, dtype=dtype, renormalize=renormalize,
                           pipeline_tiles=pipeline_tiles, split_k=split_k)
    hd, wd = to_device(hidden), to_device(w_gate)
    loads = torch.from_numpy(np.ascontiguousarray(loads_in, dtype=np.int32)).cuda()
    buf = B.route(hd, wd, params, loads, want_logits=True)
    torch.cuda.synchronize()
    return _collect(buf, loads, buf.logits)


def run_route_stats(hidden, w_gate, dtype, k, c, eps_high, t_fix, loads_in, which=(True, True, True),
                    pipeline_tiles=0, split_k=0):
    """GPU laser_route_stats; routing outputs as run_route plus the requested statistics."""
    params = B.make_params(k, c, eps_high, t_fix, dtype=dtype, pipeline_tiles=pipeline_tiles, split_k=split_k)
    hd, wd = to_device(hidden), to_device(w_gate)
    T, H = hd.shape
    E = wd.shape[0]
    loads = torch.from_numpy(np.ascontiguousarray(loads_in, dtype=np.int32)).cuda()
    buf = B.RouteBuffers(T, H, E, params, want_logits=True)
    mass = torch.full((T,), -1.0, dtype=torch.float32, device="cuda") if which[0] else None
    ent = torch.full((T,), -1.0, dtype=torch.float32, device="cuda") if which[1] else None
    pool = torch.full((T,), -1, dtype=torch.int32, device="cuda") if which[2] else None
    B.laser_route_stats(hd, wd, T, H, E, params, loads, buf.expert_ids, buf.weights, buf.permutation,
                        buf.expert_offsets, buf.logits, mass, ent, pool, buf.workspace)
    torch.cuda.synchronize()
    out = _collect(buf, loads, buf.logits)
    out["topk_mass"] = None if mass is None else mass.cpu().numpy()
    out["entropy"] = None if ent is None else ent.cpu().numpy()
    out["pool_size"] = None if pool is None else pool.cpu().numpy()
    return out


def run_route_from_logits(logits, k, c, eps_high, t_fix, loads_in, renormalize=True):
    params = B.make_params(k, c, eps_high, t_fix, renormalize=renormalize)
    ld = torch.from_numpy(np.ascontiguousarray(logits, dtype=np.float32)).cuda()
    loads = torch.from_numpy(np.ascontiguousarray(loads_in, dtype=np.int32)).cuda()
    buf = B.route_from_logits(ld, params, loads)
    torch.cuda.synchronize()
    return _collect(buf, loads, None)


def run_random_from_logits(logits, k, c, eps_high, t_fix, loads_in, seed, stream=0, token_offset=0,
                           renormalize=True):
    params = B.make_params(k, c, eps_high, t_fix, renormalize=renormalize, trim_mode=B.TRIM_RANDOM,
                           seed=seed, stream=stream, token_offset=token_offset)
    ld = torch.from_numpy(np.ascontiguousarray(logits, dtype=np.float32)).cuda()
    loads = torch.from_numpy(np.ascontiguousarray(loads_in, dtype=np.int32)).cuda()
    buf = B.route_from_logits(ld, params, loads)
    torch.cuda.synchronize()
    return _collect(buf, loads, None)


def check_random_from_logits(logits, k, c, eps_high, t_fix, loads_in, seed, stream=0, token_offset=0,
                             renormalize=True, tol=1e-5, label=""):
    gpu = run_random_from_logits(logits, k, c, eps_high, t_fix, loads_in, seed, stream, token_offset,
                                 renormalize)
    ref = oracle.route_random(logits, k, c, eps_high, t_fix, loads_in, seed, stream, token_offset,
                              renormalize)
    assert_discrete_equal(gpu, ref, label)
    if gpu["weights"].size:
        err = np.abs(gpu["weights"].astype(np.float64) - ref["weights"]).max()
        assert err <= tol, f"{label}: weights max abs err {err}"
    return gpu, ref


def _collect(buf, loads, logits):
    # every kernel of the call has reported completion (no bounded wait ran out)
    assert B.laser_status(buf.workspace) == B.STATUS_COMPLETE
    out = {
        "expert_ids": buf.expert_ids.cpu().numpy(),
        "weights": buf.weights.cpu().numpy(),
        "permutation": buf.permutation.cpu().numpy(),
        "expert_offsets": buf.expert_offsets.cpu().numpy(),
        "loads": loads.cpu().numpy(),
    }
    if logits is not None:
        out["logits"] = logits.cpu().numpy()
    return out


def assert_discrete_equal(gpu: dict, ref: dict, label: str = ""):
    """Bit-exact comparison of every integer output."""
    for key in ("expert_ids", "loads", "expert_offsets", "permutation"):
        a, b = gpu[key], ref[key]
        if not np.array_equal(a, b):
            bad = np.argwhere(a != b)
            raise AssertionError(f"{label}: {key} differs at {len(bad)} places, first {bad[0].tolist()}: "
                                 f"gpu {a[tuple(bad[0])]} oracle {b[tuple(bad[0])]}")


def check_from_logits(logits, k, c, eps_high, t_fix, loads_in, renormalize=True, tol=1e-5,
                      label=""):
    gpu = run_route_from_logits(logits, k, c, eps_high, t_fix, loads_in, renormalize)
    ref = oracle.route(logits, k, c, eps_high, t_fix, loads_in, renormalize)
    assert_discrete_equal(gpu, ref, label)
    if gpu["weights"].size:
        err = np.abs(gpu["weights"].astype(np.float64) - ref["weights"]).max()
        assert err <= tol, f"{label}: weights max abs err {err}"
    return gpu, ref


def check_route(hidden, w_gate, dtype, k, c, eps_high, t_fix, loads_in, renormalize=True,
                label="", logit_rows=None, pipeline_tiles=0, split_k=0):
    """Full path.  Logits against the fp64 gate (all rows, or a sample of rows);
    discrete outputs against the oracle routed on the GPU's own fp32 logits."""
    gpu = run_route(hidden, w_gate, dtype, k, c, eps_high, t_fix, loads_in, renormalize,
                    pipeline_tiles, split_k)
    tol = TOL_LOGIT[dtype]
    if logit_rows is None:
        z = oracle.gate(hidden, w_gate, dtype)
        err = np.abs(gpu["logits"].astype(np.float64) - z).max() if z.size else 0.0
    else:
        z = oracle.gate(hidden[logit_rows], w_gate, dtype)
        err = np.abs(gpu["logits"][logit_rows].astype(np.float64) - z).max()
    assert err <= tol, f"{label}: logits max abs err {err} > {tol}"
    ref = oracle.route(gpu["logits"], k, c, eps_high, t_fix, loads_in, renormalize)
    assert_discrete_equal(gpu, ref, label)
    if gpu["weights"].size:
        werr = np.abs(gpu["weights"].astype(np.float64) - ref["weights"]).max()
        assert werr <= tol, f"{label}: weights max abs err {werr} > {tol}"
    return gpu, ref


def run_route_batched(hiddens, w_gates, dtype, k, c, eps_high, t_fix, loads_in, renormalize=True,
                      want_logits=True, trim_mode=None, seed=0, stream=0):
    """GPU laser_route_batched on lists of per-problem numpy inputs; list of output dicts."""
    nb = len(hiddens)
    kw = {} if trim_mode is None else dict(trim_mode=trim_mode, seed=seed, stream=stream)
    params = B.make_params(k, c, eps_high, t_fix, dtype=dtype, renormalize=renormalize, **kw)
    hd = torch.stack([to_device(h) for h in hiddens])
    wd = torch.stack([to_device(w) for w in w_gates])
    T, H = hiddens[0].shape
    E = w_gates[0].shape[0]
    loads = torch.from_numpy(np.ascontiguousarray(np.stack(loads_in), dtype=np.int32)).cuda()
    one = B.laser_workspace_bytes(T, H, E, params)
    ws = torch.empty(nb * one, dtype=torch.uint8, device="cuda")
    ids = torch.full((nb, T, k), -1, dtype=torch.int32, device="cuda")
    wts = torch.full((nb, T, k), -1.0, dtype=torch.float32, device="cuda")
    perm = torch.full((nb, T * k), -1, dtype=torch.int32, device="cuda")
    offs = torch.full((nb, E + 1), -1, dtype=torch.int32, device="cuda")
    logits = torch.full((nb, T, E), -1.0, dtype=torch.float32, device="cuda") if want_logits else None
    B.laser_route_batched(hd, wd, nb, T, H, E, params, loads, ids, wts, perm, offs, logits, ws)
    torch.cuda.synchronize()
    for b in range(nb):
        assert B.laser_status(ws[b * one:]) == B.STATUS_COMPLETE
    out = []
    for b in range(nb):
        d = {"expert_ids": ids[b].cpu().numpy(), "weights": wts[b].cpu().numpy(),
             "permutation": perm[b].cpu().numpy(), "expert_offsets": offs[b].cpu().numpy(),
             "loads": loads[b].cpu().numpy()}
        if logits is not None:
            d["logits"] = logits[b].cpu().numpy()
        out.append(d)
    return out
