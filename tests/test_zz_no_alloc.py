"""The entry point that allocates nothing (laser_route_static: the workspace is an array
inside the library) against laser_route with a caller's workspace: every output bit for
bit, on two calls in a row, the second smaller (the shared array keeps the first call's
contents), and against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from synth import workloads as wl  # noqa: E402


def _pair(T, H, E, k, c, eps, tfix, seed, dtype=wl.DTYPE_BF16):
    import torch
    from paper_2510_03293_amd import binding as B
    from tests import gpu_util as u
    rng = np.random.default_rng(seed)
    h, w = wl.make_gate(rng, T, H, E, dtype)
    loads_in = rng.integers(0, 100, size=E).astype(np.int32)
    params = B.make_params(k, c, eps, tfix, dtype=dtype)
    hd, wd = u.to_device(h), u.to_device(w)
    # the existing entry point, caller's workspace
    ref = u.run_route(h, w, dtype, k, c, eps, tfix, loads_in)
    # the same call on the library's array; outputs pre-filled so that nothing stale passes
    loads = torch.from_numpy(loads_in.copy()).cuda()
    ids = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    wts = torch.full((T, k), -1.0, dtype=torch.float32, device="cuda")
    perm = torch.full((T * k,), -1, dtype=torch.int32, device="cuda")
    offs = torch.full((E + 1,), -1, dtype=torch.int32, device="cuda")
    logits = torch.full((T, E), -1.0, dtype=torch.float32, device="cuda")
    B.laser_route_static(hd, wd, T, H, E, params, loads, ids, wts, perm, offs, logits)
    assert B.laser_status_static() == B.STATUS_COMPLETE
    got = {"expert_ids": ids.cpu().numpy(), "weights": wts.cpu().numpy(), "permutation": perm.cpu().numpy(),
           "expert_offsets": offs.cpu().numpy(), "loads": loads.cpu().numpy(), "logits": logits.cpu().numpy()}
    u.assert_discrete_equal(got, ref, f"static T{T}")
    assert np.array_equal(got["weights"].view(np.int32), ref["weights"].view(np.int32))
    assert np.array_equal(got["logits"].view(np.int32), ref["logits"].view(np.int32))
    import oracle
    orc = oracle.route(got["logits"], k, c, eps, tfix, loads_in)
    u.assert_discrete_equal(got, orc, f"static vs oracle T{T}")
    return got


def test_static_workspace_calls_in_a_row():
    from paper_2510_03293_amd import binding as B
    assert B.laser_static_workspace_bytes() >= B.laser_workspace_bytes(16384, 2048, 64, B.make_params(6, 8, 0.4, 0.8))
    # a large call with many load-dependent tokens, then a smaller one, then a tiny
    # decode-sized one with other parameters: each on what the call before left behind
    _pair(5000, 2048, 64, 6, 8, 2.0, 0.05, seed=1)
    _pair(1300, 2048, 64, 6, 8, 0.4, 0.8, seed=2)
    _pair(64, 512, 8, 2, 4, 0.7, 0.6, seed=3)
    _pair(700, 256, 64, 6, 40, 2.0, 1e-30, seed=4)      # records of 64 candidates


def test_static_workspace_rejects_what_does_not_fit():
    import ctypes
    from paper_2510_03293_amd import binding as B
    p = B.make_params(6, 8, 0.4, 0.8)
    fake = ctypes.c_void_p(0x1000)
    T = 1 << 20
    assert B.laser_workspace_bytes(T, 2048, 64, p) > B.laser_static_workspace_bytes()
    rc = B._lib.laser_route_static(fake, fake, T, 2048, 64, ctypes.byref(p), fake, fake, fake, fake, fake, None, None)
    assert rc == -4
    assert "workspace" in B.laser_strerror(rc)
