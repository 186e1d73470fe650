"""Host-only: the oracle and the library's host dispatch code under the address and
undefined-behaviour sanitizers (heap and stack bounds, use after free, signed overflow, shifts,
misaligned access, float-to-int range) on small awkward shapes.  Nothing here touches a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_is_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    # the sanitizer runtime is linked statically: it must not depend on its place in the
    # loader's list of preloaded libraries
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", os.path.join(ROOT, "oracle", "dabnn_oracle.c"),
           os.path.join(ROOT, "tests", "host", "oracle_sanitize_main.c"), "-o", exe, "-lm"]
    subprocess.run(cmd, check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    sys.stdout.write(out.stdout)
    sys.stderr.write(out.stderr)
    assert out.returncode == 0 and "oracle sanitizer run ok" in out.stdout


def _library_objects():
    import glob
    import pytest
    build_dir = os.path.join(ROOT, "paper_1908_05858_amd", "_build")
    objs = [o for o in glob.glob(os.path.join(build_dir, "*.o")) if not o.endswith("dabnn_api.o")]
    if len(objs) < 5:
        pytest.skip("the library's object files are not in the tree (run build() first)")
    return objs


def test_host_dispatch_is_clean_under_asan_and_ubsan(tmp_path):
    """csrc/dabnn_api.hip rebuilt with both sanitizers on the HOST side only, linked with the
    library's other objects and a C++ driver (tests/host/dispatch_sanitize_main.cpp) into one
    executable with the static sanitizer runtime, and run without a GPU."""
    objs = _library_objects()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    if not os.path.exists(clangxx):
        import pytest
        pytest.skip("no clang++ next to hipcc")
    api_o, drv_o, exe = (str(tmp_path / n) for n in ("api.o", "driver.o", "dispatch_sanitize"))
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops"] + [x for f in san for x in ("-Xarch_host", f)]
    subprocess.run([hipcc] + flags + ["-c", os.path.join(ROOT, "paper_1908_05858_amd", "csrc", "dabnn_api.hip"),
                                      "-o", api_o], check=True, capture_output=True)
    subprocess.run([clangxx] + san + ["-O1", "-g", "-std=c++17", "-c",
                                      os.path.join(ROOT, "tests", "host", "dispatch_sanitize_main.cpp"), "-o", drv_o],
                   check=True, capture_output=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-fsanitize=address,undefined", "-fno-gpu-sanitize", drv_o, api_o]
                   + objs + ["-o", exe], check=True, capture_output=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    sys.stdout.write(out.stdout)
    sys.stderr.write(out.stderr[-2000:])
    assert out.returncode == 0 and "host dispatch sanitizer run ok" in out.stdout


def test_host_dispatch_is_clean_under_ubsan(tmp_path):
    """The library's host code (argument validation, dispatch, the batch-norm threshold helper)
    rebuilt with the undefined-behaviour sanitizer on the HOST side only and driven through the
    C ABI without a GPU: every call here must be refused or computed on the host."""
    import glob
    objs = _library_objects()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    api_o = str(tmp_path / "dabnn_api_ubsan.o")
    lib = str(tmp_path / "libdabnn_ubsan.so")
    flags = ["--offload-arch=gfx950", "-O1", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
             "-packed-fp32-ops", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=all"]
    subprocess.run([hipcc] + flags + ["-c", os.path.join(ROOT, "paper_1908_05858_amd", "csrc", "dabnn_api.hip"),
                                      "-o", api_o], check=True, capture_output=True)
    # a shared object does not pull in the sanitizer runtime by itself: link the shared runtime
    # that ships with the compiler and let the loader find it through an rpath
    rt = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.ubsan_standalone-x86_64.so")
    if not rt:
        import pytest
        pytest.skip("no shared UBSan runtime next to hipcc")
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", api_o] + objs +
                   [rt[0], "-Wl,-rpath," + os.path.dirname(rt[0]), "-o", lib], check=True, capture_output=True)
    driver = r"""
import ctypes, sys
import numpy as np
lib = ctypes.CDLL(sys.argv[1])
P = ctypes.c_void_p
a, w, y = P(0x10000), P(0x20000), P(0x30000)
assert lib.dabnn_bconv2d(a, w, y, 1, 4, 4, 64, 64, 3, 3, 1, 3, None) == 2
assert lib.dabnn_bconv2d(a, w, y, 2**31 - 1, 2**15, 2**15, 64, 64, 3, 3, 1, 1, None) == 2
assert lib.dabnn_bconv2d(a, w, P(0x30002), 1, 4, 4, 64, 64, 3, 3, 1, 1, None) == 3
lib.dabnn_bconv2d_pick_algo.restype = ctypes.c_int
for shape in [(256, 56, 56, 64, 64, 3, 3, 1, 1), (1, 7, 7, 512, 512, 3, 3, 2, 1), (3, 9, 9, 100, 7, 5, 5, 3, 2),
              (2, 6, 6, 128, 64, 1, 1, 1, 0)]:
    assert lib.dabnn_bconv2d_pick_algo(*shape) in (1, 2, 3, 4)
lib.dabnn_bgemm.argtypes = [P, P, P, ctypes.c_int64] + [ctypes.c_int] * 4 + [P]
assert lib.dabnn_bgemm(a, w, y, 2**40, 16, 1, 64, 0, None) == 2
lib.dabnn_bitpack.argtypes = [P, P, ctypes.c_int64, ctypes.c_int, ctypes.c_int, P]
assert lib.dabnn_bitpack(a, w, 2**41, 2**10, 0, None) == 2
lib.dabnn_bn_thresholds.argtypes = [P] * 4 + [ctypes.c_float, ctypes.c_int, ctypes.c_int, P, P]
C, K = 300, 4608
rng = np.random.default_rng(3)
g = rng.uniform(-3, 3, C).astype(np.float32); g[::5] = 0; g[1] = 1e-38; g[2] = -3e38
b = rng.normal(0, 2, C).astype(np.float32); b[3] = 3e38; b[4] = -3e38
m = rng.normal(0, 500, C).astype(np.float32); m[6] = 3e38
v = rng.uniform(0, 50, C).astype(np.float32); v[7] = 0; v[8] = 3e38
thr = np.empty(C, np.int32); flip = np.empty((C + 63) // 64, np.uint64)
ptr = lambda x: P(x.ctypes.data)
assert lib.dabnn_bn_thresholds(ptr(g), ptr(b), ptr(m), ptr(v), ctypes.c_float(1e-5), C, K, ptr(thr), ptr(flip)) == 0
assert np.all(np.abs(thr.astype(np.int64)) <= 2**30)
print("host dispatch ubsan run ok")
"""
    out = subprocess.run([sys.executable, "-c", driver, lib], capture_output=True, text=True, timeout=300)
    sys.stdout.write(out.stdout)
    sys.stderr.write(out.stderr[-2000:])
    assert out.returncode == 0 and "host dispatch ubsan run ok" in out.stdout
