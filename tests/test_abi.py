"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "laser.h")
BENCH_HEADER = os.path.join(ROOT, "include", "laser_bench.h")


@pytest.fixture(scope="module")
def B():
    from paper_2510_03293_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding


def _declared_functions(header):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(laser_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    lib = ctypes.CDLL(B.LIB_PATH)
    for header, listed in ((HEADER, B.EXPORTS), (BENCH_HEADER, B.BENCH_EXPORTS)):
        names = _declared_functions(header)
        assert set(names) == set(listed), header
        for n in names:
            assert hasattr(lib, n), n


def test_product_header_holds_no_benchmark_helpers(B):
    """Calls that create events, synchronise for timing or launch probe kernels live in
    laser_bench.h; laser.h declares the routing path only."""
    assert not [n for n in _declared_functions(HEADER) if "bench" in n or "profile" in n]


def test_strerror_and_struct_size(B):
    assert B.laser_strerror(0) == "ok"
    assert "NULL" in B.laser_strerror(-1)
    # 8 x 4 bytes, then seed, token_offset, stream, poll_budget, pipeline_tiles, split_k
    assert ctypes.sizeof(B.LaserParams) == 64


def test_workspace_query(B):
    p = B.make_params(6, 8, 0.4, 0.8)
    small = B.laser_workspace_bytes(64, 2048, 64, p)
    big = B.laser_workspace_bytes(16384, 2048, 64, p)
    assert 0 < small < big < 64 << 20
    assert B.laser_workspace_bytes(0, 2048, 64, p) > 0
    assert B.laser_workspace_bytes(-1, 2048, 64, p) == 0
    assert B.laser_workspace_bytes(64, 2048, 65, p) == 0          # E above the limit
    wide = B.make_params(6, 64, 0.4, 0.8)                          # records of 64 candidates
    assert B.laser_workspace_bytes(16384, 2048, 64, wide) > big
    assert B.laser_workspace_bytes(16384, 2048, 64, B.make_params(6, 16, 0.4, 0.8)) == big


def test_status_query_rejects_null(B):
    st = ctypes.c_int32(0)
    assert B._lib.laser_status(None, None, ctypes.byref(st)) == -1
    assert B._lib.laser_status(ctypes.c_void_p(0x1000), None, None) == -1


def test_argument_errors_before_any_device_work(B):
    """Fake non-null addresses are safe: validation fails before anything is enqueued."""
    fake = ctypes.c_void_p(0x1000)
    ws = ctypes.c_void_p(0x10000)
    lib = B._lib

    def route(p, T=64, H=2048, E=64, hidden=fake, wsz=1 << 30, wsp=ws):
        return lib.laser_route(hidden, fake, T, H, E, ctypes.byref(p), fake, fake, fake, fake, fake,
                               None, wsp, wsz, None)

    ok = dict(k=6, c=8, eps_high=0.4, t_fix=0.8)
    assert route(B.make_params(**{**ok, "k": 0})) == -2
    assert route(B.make_params(**{**ok, "c": 5})) == -2             # c < k
    assert route(B.make_params(**{**ok, "c": 65})) == -2            # c > E
    assert route(B.make_params(**{**ok, "eps_high": 0.0})) == -2
    assert route(B.make_params(**{**ok, "t_fix": 1.5})) == -2
    assert route(B.make_params(**{**ok, "t_fix": 0.0})) == -2
    assert route(B.make_params(**ok), T=-1) == -2
    assert route(B.make_params(k=6, c=8, eps_high=.4, t_fix=.8), E=65) == -5
    assert route(B.make_params(k=17, c=17, eps_high=.4, t_fix=.8), E=64) == -5  # k > 16
    assert route(B.make_params(k=2, c=64, eps_high=.4, t_fix=.8), E=64, wsz=1024) == -4  # (c up to E is valid)
    assert route(B.make_params(**ok, trim_mode=2)) == -2            # neither TOP nor RANDOM
    assert route(B.make_params(**ok), H=2044) == -3                 # bf16 rows need H % 8 == 0
    assert route(B.make_params(**ok), hidden=ctypes.c_void_p(0x1008)) == -3
    assert route(B.make_params(**ok), hidden=None) == -1
    assert route(B.make_params(**ok), wsz=1024) == -4
    assert route(B.make_params(**ok), wsp=ctypes.c_void_p(0x10010)) == -3
    bad = B.make_params(**ok)
    bad.struct_bytes = 12
    assert route(bad) == -6
    assert route(B.make_params(**ok, dtype=7)) == -2


def test_binding_raises_on_error(B):
    with pytest.raises(B.LaserError):
        B._check(-4)


def test_header_is_plain_c_and_links(B, tmp_path):
    """The header compiles as C99 on its own, and a C program that includes it links
    against the library and calls the host-only entry points (no GPU needed)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_laser.c"
    src.write_text(
        '#include "laser.h"\n'
        '#include "laser_bench.h"\n'
        '#include <stdio.h>\n'
        'int main(void) {\n'
        '  laser_params_t p = {0};\n'
        '  p.struct_bytes = (uint32_t)sizeof p; p.k = 6; p.c = 8; p.eps_high = 0.4f; p.t_fix = 0.8f;\n'
        '  p.trim_mode = LASER_TRIM_TOP; p.renormalize = 1; p.dtype = LASER_DTYPE_BF16;\n'
        '  printf("%zu %s %d\\n", laser_workspace_bytes(16384, 2048, 64, &p), laser_strerror(LASER_E_WORKSPACE),\n'
        '         laser_route(0, 0, 64, 2048, 64, &p, 0, 0, 0, 0, 0, 0, 0, 0, 0));\n'
        '  return 0;\n'
        '}\n')
    exe = tmp_path / "use_laser"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-llaser_route", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == B.laser_workspace_bytes(16384, 2048, 64, B.make_params(6, 8, 0.4, 0.8))
    assert out[-1] == "-1"                     # NULL pointers are refused before any device work
