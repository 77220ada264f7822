"""Host-side checks that need no GPU: the C-ABI library exports what include/tslt.h declares, argument
errors are reported before anything is launched, and the fp64 exp used by the inverse-CDF kernels is
accurate (its header compiles for the host too)."""
import ctypes
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2512_16273_amd", "libtslt.so")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tslt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tslt_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2512_16273_amd import build
        build.build_library(verbose=False)
    return ctypes.CDLL(LIB)


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert {"tslt_truncate", "tslt_sample", "tslt_verify", "tslt_verify_tree"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2512_16273_amd import tslt
    assert set(tslt.EXPORTS) == set(names)


def test_workspace_sizes_and_version(lib):
    lib.tslt_workspace_bytes.restype = ctypes.c_size_t
    lib.tslt_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32]
    assert lib.tslt_version() >= 100
    assert lib.tslt_workspace_bytes(0, 2048, 0, 128256, 256) == 0          # truncate needs none
    small = lib.tslt_workspace_bytes(2, 16, 8, 32000, 64)
    big = lib.tslt_workspace_bytes(2, 256, 8, 128256, 256)
    assert 0 < small < big < 64 << 20 and big % 256 == 0
    assert lib.tslt_workspace_bytes(2, 0, 8, 32000, 64) == 0


def test_argument_errors_are_found_on_the_host(lib):
    """Bad arguments return a negative code and a message; nothing touches the (absent) GPU."""
    lib.tslt_last_error.restype = ctypes.c_char_p
    vp, i32, i64, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t
    lib.tslt_truncate.restype = ctypes.c_int
    lib.tslt_truncate.argtypes = [vp, ctypes.c_int, i64, i64, i64, f32, i32, f32, i32, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp,
                                  sz, vp]
    fake = ctypes.c_void_p(0x1000)
    def call(dt=1, rows=4, V=1000, stride=1000, T=1.0, k=4, p=0.0, cap=4, ptr=fake, payload=0):
        return lib.tslt_truncate(ptr, dt, rows, V, stride, T, k, p, cap, payload, fake, fake, None, fake, None, None, None,
                                 0, None)
    assert call(T=0.0) == -1 and b"temperature" in lib.tslt_last_error()
    assert call(dt=7) == -1
    assert call(stride=10) == -1
    assert call(cap=0) == -2 and call(cap=5000) == -2
    assert call(k=-1) == -1
    assert call(ptr=None) == -1
    assert call(ptr=ctypes.c_void_p(0x1001)) == -1                          # bf16 row at an odd address
    assert call(rows=0) == 0                                                 # empty batch: nothing to do
    assert call(payload=5) == -1 and b"payload" in lib.tslt_last_error()
    # wire format: sizes and argument checks
    lib.tslt_pack_bound_words.restype = i64
    lib.tslt_pack_bound_words.argtypes = [i64, i32, i64]
    assert lib.tslt_pack_bound_words(3, 256, 128256) == 3 * ((16 + 256 * (17 + 16) + 31) // 32)
    assert lib.tslt_pack_bound_words(1, 1, 1) == 1 and lib.tslt_pack_bound_words(1, 1024, 2 ** 31 - 1) == (16 + 1024 * 47 + 31) // 32
    lib.tslt_pack.restype = ctypes.c_int
    lib.tslt_pack.argtypes = [vp, vp, vp, i64, i32, i64, ctypes.c_int, vp, i64, vp, vp]
    assert lib.tslt_pack(fake, fake, fake, 4, 16, 1000, 0, fake, 10 ** 6, fake, None) == -1      # fp32 is not a wire format
    assert lib.tslt_pack(fake, fake, fake, 4, 16, 1000, 1, fake, 3, fake, None) == -3            # too little room
    lib.tslt_unpack.restype = ctypes.c_int
    lib.tslt_unpack.argtypes = [vp, vp, i64, i32, i64, ctypes.c_int, vp, vp, vp, vp]
    assert lib.tslt_unpack(fake, fake, 4, 4096, 1000, 2, fake, fake, fake, None) == -2
    assert lib.tslt_unpack(None, fake, 4, 16, 1000, 2, fake, fake, fake, None) == -1
    lib.tslt_sample.restype = ctypes.c_int
    lib.tslt_sample.argtypes = [vp, vp, vp, i64, i32, vp, i32, i32, vp, vp, vp]
    assert lib.tslt_sample(fake, fake, fake, 4, 2048, fake, 1, 0, fake, None, None) == -2
    assert lib.tslt_sample(None, fake, fake, 4, 16, fake, 1, 0, fake, None, None) == -1
    # verification: shapes, workspace, the staged call's extra argument
    verify_args = [vp, ctypes.c_int, i64, i32, i64, i64, f32, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.tslt_verify.restype = ctypes.c_int
    lib.tslt_verify.argtypes = verify_args
    lib.tslt_verify_staged.restype = ctypes.c_int
    lib.tslt_verify_staged.argtypes = verify_args + [i32]
    lib.tslt_workspace_bytes.restype = ctypes.c_size_t
    lib.tslt_workspace_bytes.argtypes = [ctypes.c_int, i64, i64, i64, i32]
    need = lib.tslt_workspace_bytes(2, 4, 8, 1000, 16)
    ws = ctypes.c_void_p(0x10000)
    def verify(fn, B=4, gamma=8, V=1000, stride=1000, T=1.0, cap=16, ws=ws, ws_bytes=need, extra=()):
        return fn(fake, 1, B, gamma, V, stride, T, fake, fake, fake, cap, fake, fake, fake, fake, fake, None, None, None,
                  ws, ws_bytes, None, *extra)
    assert verify(lib.tslt_verify, gamma=0) == -1
    assert verify(lib.tslt_verify, T=-1.0) == -1
    assert verify(lib.tslt_verify, cap=2000) == -2
    assert verify(lib.tslt_verify, ws_bytes=need - 1) == -3 and b"workspace" in lib.tslt_last_error()
    assert verify(lib.tslt_verify, ws=ctypes.c_void_p(0x10010)) == -3       # workspace not aligned to 256 bytes
    assert verify(lib.tslt_verify, B=0) == 0
    assert verify(lib.tslt_verify_staged, extra=(-1,)) == -1 and b"first_stage" in lib.tslt_last_error()
    assert verify(lib.tslt_verify_staged, B=0, extra=(2,)) == 0


def test_exp64_header_matches_libm(tmp_path):
    """The kernels' fp64 exp, compiled for the host, against libm's long-double exp."""
    exe = tmp_path / "exp64_check"
    subprocess.run(["g++", "-O2", "-ffp-contract=off", "-mfma", "-I", os.path.join(ROOT, "paper_2512_16273_amd", "csrc"),
                    "-o", str(exe), os.path.join(ROOT, "tests", "exp64_check.cpp")], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    m = re.search(r"max_ulp ([0-9.]+) edge (\d)", out)
    assert m and float(m.group(1)) < 1.5 and m.group(2) == "1", out


def test_bench_refuses_more_than_one_gpu():
    """This build measures one GPU; asked for more, bench.py says so and exits before it touches a device."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
