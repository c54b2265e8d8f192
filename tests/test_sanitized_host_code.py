"""The CPU-side code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU needed):
  - the oracle, rebuilt with both sanitizers, runs its pin tests in a subprocess that preloads the sanitizer runtime;
  - the library's host-only mask code (build at gamma_max, slices, release) is compiled with the host compiler's
    sanitizers and driven through the C ABI over many trees, compared with the oracle's masks.
Any finding aborts the subprocess."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _preload(env, runtime):
    old = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = runtime + (":" + old if old else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1"          # the interpreter itself is not leak-clean
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    return env


def test_oracle_pins_under_sanitizers(oracle):
    oracle.build(sanitize=True)
    env = _preload(dict(os.environ, MCSD_ORACLE_SANITIZED="1", OMP_NUM_THREADS="4"), oracle.sanitizer_runtime())
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_mask.py",
                        "tests/test_oracle_attention.py", "tests/test_oracle_verify.py", "tests/test_oracle_commit.py",
                        "tests/test_oracle_fp8kv.py", "tests/test_oracle_decision.py"],
                       cwd=ROOT, capture_output=True, text=True, env=env)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail


DRIVER = r"""
import ctypes as C, sys
import numpy as np
sys.path.insert(0, {root!r})
import oracle
lib = C.CDLL({lib!r})
class View(C.Structure):
    _fields_ = [("gamma", C.c_int32), ("n_nodes", C.c_int32), ("gamma_max", C.c_int32), ("n_nodes_max", C.c_int32),
                ("words_per_row", C.c_int32), ("device", C.c_int32), ("bits_host", C.POINTER(C.c_uint64)),
                ("bits_dev", C.c_void_p), ("parent_host", C.POINTER(C.c_int32)), ("parent_dev", C.c_void_p),
                ("level_host", C.POINTER(C.c_int32)), ("level_off_host", C.POINTER(C.c_int32)),
                ("branching_host", C.POINTER(C.c_int32))]
lib.mcsd_build_mask.argtypes = [C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_void_p)]
lib.mcsd_slice_mask.argtypes = [C.c_void_p, C.c_int32, C.POINTER(View)]
lib.mcsd_free_mask.argtypes = [C.c_void_p]
trees = [(2, 2, 2), (4, 2, 2, 1), (3, 2, 2, 1, 1, 1, 1, 1), (8, 2, 2, 1, 1), (2, 4, 3, 1, 1), (1,), (64,), (64, 63), (1,) * 32,
         (16, 1, 1, 1, 1), (63, 1), (4, 4, 4, 4, 4), (2,) * 11]
for br in trees:
    arr = (C.c_int32 * len(br))(*br)
    h = C.c_void_p()
    assert lib.mcsd_build_mask(arr, len(br), C.byref(h)) == 0, br
    full = oracle.build_mask(br) if sum(np.cumprod(br)) <= 1100 else None
    for g in range(1, len(br) + 1):
        v = View()
        assert lib.mcsd_slice_mask(h, g, C.byref(v)) == 0
        n, W = v.n_nodes, v.words_per_row
        words = np.ctypeslib.as_array(v.bits_host, shape=(v.n_nodes_max * W,)).reshape(v.n_nodes_max, W)
        assert n == int(sum(np.cumprod(br[:g])))
        if full is not None:
            got = np.zeros((n, n), dtype=np.uint8)
            for j in range(n):
                got[:, j] = (words[:n, j >> 6] >> np.uint64(j & 63)) & np.uint64(1)
            assert np.array_equal(got, full[:n, :n]), (br, g)
        else:                                   # large trees: popcount of row i is its level
            lv = np.ctypeslib.as_array(v.level_host, shape=(v.n_nodes_max,))
            pop = np.array([sum(bin(int(x)).count("1") for x in words[i]) for i in range(0, n, 97)])
            assert np.array_equal(pop, lv[0:n:97]), (br, g)
    bad = View()
    assert lib.mcsd_slice_mask(h, len(br) + 1, C.byref(bad)) == -1 and lib.mcsd_slice_mask(h, 0, C.byref(bad)) == -1
    lib.mcsd_free_mask(h)
for br in [(0,), (65,), (2,) * 33, (64, 64, 2)]:
    arr = (C.c_int32 * len(br))(*br)
    h = C.c_void_p()
    assert lib.mcsd_build_mask(arr, len(br), C.byref(h)) < 0 and not h.value, br
lib.mcsd_free_mask(None)
print("host mask code clean")
"""


def test_host_mask_code_under_sanitizers(oracle, tmp_path):
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not available")
    csrc = os.path.join(ROOT, "paper_2409_10644_amd", "csrc")
    lib = str(tmp_path / "libmcsd_mask_san.so")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-x", "hip", "-I",
           os.path.join(ROOT, "include"), "-I", csrc, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all", "-shared-libsan", os.path.join(csrc, "mask.cpp"), "-o", lib]
    subprocess.run(cmd, check=True, capture_output=True)
    rt = subprocess.run([os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "llvm", "bin", "clang"),
                         "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.exists(rt):
        pytest.skip("the host compiler's sanitizer runtime is not installed")
    env = _preload(dict(os.environ), rt)
    r = subprocess.run([sys.executable, "-c", DRIVER.format(root=ROOT, lib=lib)], capture_output=True, text=True, env=env)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0 and "host mask code clean" in r.stdout, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
