"""GPU tests of split calls: a small bf16 batch (up to 64 tiles of 64 tokens) has the
contraction axis of its gate projection cut over eight workgroups per tile (four beyond 32
tiles), whose partial logit tiles meet in the workspace; the workgroup that arrives last
adds them in the order the unsplit kernel uses.  Nothing may depend on the split, the logits included: every case
is compared with the oracle and, bit for bit, with the same call run with `split_k = 1`."""
from __future__ import annotations

import numpy as np
import pytest

from synth import workloads as wl

pytestmark = pytest.mark.gpu


def _util():
    import gpu_util
    return gpu_util


def _gate(seed, T, H, E, flat_frac):
    rng = np.random.default_rng(seed)
    rank_of = rng.permutation(E) + 1
    zipf = (-1.3 * np.log(rank_of)).astype(np.float32)
    flat = rng.random(T) < flat_frac
    bias = np.where(flat[:, None], np.float32(0.0), zipf[None, :]).astype(np.float32)
    natural = 0.02 * np.sqrt(H)
    sigma = np.where(flat, np.float32(0.05 / natural), np.float32(1.0)).astype(np.float32)
    return wl.make_gate(rng, T, H, E, wl.DTYPE_BF16, bias=bias, sigma=sigma)


def _same(a, b, label):
    for key in ("expert_ids", "loads", "expert_offsets", "permutation", "weights", "logits"):
        assert np.array_equal(a[key], b[key]), f"{label}: {key} depends on the split"


CASES = [
    # T, H, E, k, c, share of flat rows
    (1, 2048, 64, 6, 8, 0.0),
    # one tile without a load-dependent token: the fused kernel writes the dispatch tables itself
    (64, 2048, 64, 6, 8, 0.0),
    (37, 512, 8, 2, 4, 0.0),
    (64, 4096, 16, 4, 12, 0.0),
    (50, 1000, 33, 3, 9, 0.0),
    (64, 2048, 64, 6, 8, 0.3),       # the decode shape: one tile, written-out loop of 4 chunks
    (64, 4096, 8, 2, 4, 0.5),        # written-out loop of 8 chunks, one expert block
    (65, 4096, 64, 6, 8, 0.3),       # a second tile of one token
    (200, 512, 64, 6, 8, 0.2),       # one chunk per role
    (200, 256, 64, 6, 8, 0.2),       # four of the eight roles have no chunk
    (130, 64, 16, 4, 12, 0.4),       # a single chunk in all
    (300, 1000, 33, 3, 9, 0.4),      # ragged contraction axis (1000 = 15 chunks + 40), odd expert count
    (257, 40, 8, 2, 4, 1.0),         # no full chunk at all
    (1000, 2048, 64, 6, 8, 0.1),
    (2048, 2048, 64, 6, 8, 0.5),     # 32 tiles: the most that eight workgroups per tile take; window evaluation
    (2048, 4096, 32, 4, 8, 0.3),
    (1500, 768, 24, 5, 16, 0.6),
    # 33 to 64 tiles: four workgroups per tile, two wavefront roles each
    (2049, 2048, 64, 6, 8, 0.3),
    (4096, 2048, 64, 6, 8, 0.2),     # one round of eight chunks per workgroup
    (4096, 4096, 8, 2, 4, 0.4),      # two rounds
    (3000, 512, 16, 4, 12, 0.3),     # one chunk per role
    (2500, 320, 64, 6, 8, 0.3),      # five chunks: roles with one chunk and with none
    (2200, 1000, 33, 3, 9, 0.4),     # ragged contraction axis
    (2100, 40, 32, 4, 8, 0.5),       # no full chunk at all
    (4096, 3000, 64, 6, 8, 0.1),     # six rounds, the last one ragged
]


@pytest.mark.parametrize("T,H,E,k,c,frac", CASES)
def test_split_call_equals_oracle_and_unsplit_call(T, H, E, k, c, frac):
    u = _util()
    hidden, w = _gate(4000 + T + H + E, T, H, E, frac)
    rng = np.random.default_rng(T)
    loads = rng.integers(0, 50, size=E).astype(np.int32)
    gpu, _ = u.check_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, label=f"split T{T} H{H} E{E}")
    whole = u.run_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, split_k=1)
    _same(gpu, whole, f"T{T} H{H} E{E}")


def test_above_the_limit_nothing_changes():
    """65 tiles: the call is not split, with or without the switch."""
    u = _util()
    T, H, E, k, c = 4097, 512, 64, 6, 8
    hidden, w = _gate(77, T, H, E, 0.2)
    loads = np.zeros(E, np.int32)
    gpu, _ = u.check_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, label="65 tiles")
    whole = u.run_route(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, split_k=1)
    _same(gpu, whole, "65 tiles")


def test_calls_in_a_row_on_one_workspace():
    """The arrival counters belong to the workspace's address and go back to zero with every
    call: calls of different sizes in a row on one workspace, split and not, each against
    the oracle fed with the call's own logits."""
    import torch
    import oracle
    from paper_2510_03293_amd import binding as B
    u = _util()
    H, E, k, c = 1024, 64, 6, 8
    sizes = [2048, 64, 4096, 700, 1, 2048, 2500, 130, 64, 64]
    Tmax = max(sizes)
    params = [B.make_params(k, c, 0.40, 0.80, dtype=wl.DTYPE_BF16),
              B.make_params(k, c, 0.40, 0.80, dtype=wl.DTYPE_BF16, split_k=1)]
    buf = B.RouteBuffers(Tmax, H, E, params[0], want_logits=True)
    loads = torch.zeros(E, dtype=torch.int32, device="cuda")
    ref_loads = np.zeros(E, np.int32)
    for n, T in enumerate(sizes):
        hidden, w = _gate(900 + n, T, H, E, 0.3)
        hd, wd = u.to_device(hidden), u.to_device(w)
        B.laser_route(hd, wd, T, H, E, params[n % 3 == 2], loads, buf.expert_ids, buf.weights, buf.permutation,
                      buf.expert_offsets, buf.logits, buf.workspace)
        torch.cuda.synchronize()
        assert B.laser_status(buf.workspace) == B.STATUS_COMPLETE
        z = buf.logits.cpu().numpy().reshape(-1)[:T * E].reshape(T, E)
        ref = oracle.route(z, k, c, 0.40, 0.80, ref_loads)
        got = {"expert_ids": buf.expert_ids.cpu().numpy()[:T], "loads": loads.cpu().numpy(),
               "expert_offsets": buf.expert_offsets.cpu().numpy(),
               "permutation": buf.permutation.cpu().numpy()[:T * k]}
        u.assert_discrete_equal(got, ref, f"call {n} T{T}")
        ref_loads = ref["loads"].astype(np.int32)


def test_split_call_with_statistics():
    u = _util()
    T, H, E, k, c = 900, 2048, 64, 6, 8
    hidden, w = _gate(31, T, H, E, 0.3)
    loads = np.zeros(E, np.int32)
    a = u.run_route_stats(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads)
    b = u.run_route_stats(hidden, w, wl.DTYPE_BF16, k, c, 0.40, 0.80, loads, split_k=1)
    _same(a, b, "statistics")
    for key in ("topk_mass", "entropy", "pool_size"):
        assert np.array_equal(a[key], b[key]), key


def test_a_workspace_for_a_large_batch_serves_small_ones():
    """The room for the partial tiles is part of what laser_workspace_bytes reports for up to
    4096 tokens, but a call does not insist on it: in a workspace sized for 16384 tokens a
    call of 4096 tokens finds too little room and runs without the split, one of 2048 tokens
    splits; both equal the oracle."""
    import torch
    import oracle
    from paper_2510_03293_amd import binding as B
    u = _util()
    H, E, k, c = 512, 64, 6, 8
    params = B.make_params(k, c, 0.40, 0.80, dtype=wl.DTYPE_BF16)
    big = B.RouteBuffers(16384, H, E, params, want_logits=True)
    assert B.laser_workspace_bytes(4096, H, E, params) > big.workspace.numel() > B.laser_workspace_bytes(2048, H, E, params)
    for T in (4096, 2048, 4000, 64):
        hidden, w = _gate(5 + T, T, H, E, 0.3)
        loads = torch.zeros(E, dtype=torch.int32, device="cuda")
        B.laser_route(u.to_device(hidden), u.to_device(w), T, H, E, params, loads, big.expert_ids, big.weights,
                      big.permutation, big.expert_offsets, big.logits, big.workspace)
        torch.cuda.synchronize()
        assert B.laser_status(big.workspace) == B.STATUS_COMPLETE
        z = big.logits.cpu().numpy().reshape(-1)[:T * E].reshape(T, E)
        ref = oracle.route(z, k, c, 0.40, 0.80, np.zeros(E, np.int32))
        got = {"expert_ids": big.expert_ids.cpu().numpy()[:T], "loads": loads.cpu().numpy(),
               "expert_offsets": big.expert_offsets.cpu().numpy(),
               "permutation": big.permutation.cpu().numpy()[:T * k]}
        u.assert_discrete_equal(got, ref, f"T{T} in a workspace for 16384 tokens")
        assert np.abs(z.astype(np.float64) - oracle.gate(hidden, w, wl.DTYPE_BF16)).max() <= u.TOL_LOGIT[wl.DTYPE_BF16]


@pytest.mark.parametrize("T,E,k,c,trim", [(900, 32, 4, 6, "random"), (3000, 64, 6, 8, "random"),
                                          (700, 64, 4, 40, "wide"), (2500, 64, 6, 64, "wide"),
                                          (640, 16, 4, 4, "random c = k")])
def test_split_call_with_random_or_wide_trimming(T, E, k, c, trim):
    """RANDOM trimming and trimming sizes above 16 run other kernels behind the fused one;
    the split of the fused one changes nothing for them either."""
    import torch
    import oracle
    from paper_2510_03293_amd import binding as B
    u = _util()
    H = 512
    hidden, w = wl.make_gate(np.random.default_rng(T + E), T, H, E, wl.DTYPE_BF16)
    hd, wd = u.to_device(hidden), u.to_device(w)
    extra = dict(trim_mode=B.TRIM_RANDOM, seed=11, stream=2, token_offset=50) if trim.startswith("random") else {}
    outs = []
    for split_k in (0, 1):
        params = B.make_params(k, c, 2.0, 0.05, dtype=wl.DTYPE_BF16, split_k=split_k, **extra)
        loads = torch.zeros(E, dtype=torch.int32, device="cuda")
        buf = B.route(hd, wd, params, loads, want_logits=True)
        torch.cuda.synchronize()
        assert B.laser_status(buf.workspace) == B.STATUS_COMPLETE
        outs.append({"expert_ids": buf.expert_ids.cpu().numpy(), "weights": buf.weights.cpu().numpy(),
                     "permutation": buf.permutation.cpu().numpy(), "expert_offsets": buf.expert_offsets.cpu().numpy(),
                     "loads": loads.cpu().numpy(), "logits": buf.logits.cpu().numpy()})
    _same(outs[0], outs[1], trim)
    z = outs[0]["logits"]
    if trim.startswith("random"):
        ref = oracle.route_random(z, k, c, 2.0, 0.05, np.zeros(E, np.int32), 11, 2, 50)
    else:
        ref = oracle.route(z, k, c, 2.0, 0.05, np.zeros(E, np.int32))
    u.assert_discrete_equal(outs[0], ref, trim)
