"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU call is made):

  * the C scoring oracle, built with gcc -fsanitize=address,undefined, must run clean on ragged shapes of both
    element types and both reductions, and give bit for bit what the regular build gives;
  * libilre's host pass (argument validation, the scoring plan, the selection layout and workspace carving),
    built with hipcc's host compiler under the same sanitizers, must size workspaces over a sweep of shapes and
    refuse every bad call without touching a pointer it was handed.
"""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

import inputs
import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests", "sanitize")
OUT = os.path.join(ROOT, "_build", "sanitize")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


@pytest.fixture(scope="module")
def oracle_driver():
    os.makedirs(OUT, exist_ok=True)
    exe = os.path.join(OUT, "oracle_driver")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
           "-o", exe, os.path.join(HERE, "oracle_driver.c"), os.path.join(ROOT, "oracle", "ilre_oracle.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return exe


@pytest.mark.parametrize("L,Lq,Hq,Hkv,d,dtype,mode", [
    (257, 3, 4, 2, 128, "bf16", oracle.MODE_SUM),
    (100, 5, 6, 3, 16, "f32", oracle.MODE_MAX),
    (1, 1, 2, 2, 8, "bf16", oracle.MODE_SUM),
])
def test_oracle_runs_clean_under_sanitizers(oracle_driver, tmp_path, L, Lq, Hq, Hkv, d, dtype, mode):
    inp = inputs.custom(L=L, Lq=Lq, Hq=Hq, Hkv=Hkv, d=d, dtype=dtype, n_spans=0, seed=L + d)
    rows = np.array(sorted({0, Hq * Lq - 1, (Hq * Lq) // 2}), dtype=np.int32)
    scale = 0.37
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("<8q", 1 if dtype == "bf16" else 0, L, Lq, Hq, Hkv, d, mode, rows.size))
        f.write(struct.pack("<d", scale))
        f.write(np.ascontiguousarray(inp.q).tobytes())
        f.write(np.ascontiguousarray(inp.k).tobytes())
        f.write(rows.tobytes())
    env = dict(SAN_ENV, OMP_NUM_THREADS="3")
    run = subprocess.run([oracle_driver, str(src), str(dst)], env=env, capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stderr[-2000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-2000:]
    got = np.fromfile(dst, dtype=np.float64)
    R = Hq * Lq
    score, rmax, rsum = oracle.scores(inp.q, inp.k, scale=scale, mode=mode)
    smax, ssum = oracle.row_stats(inp.q, inp.k, rows, scale=scale)
    want = np.concatenate([score, rmax, rsum, smax, ssum])
    assert got.size == L + 2 * R + 2 * rows.size
    assert np.array_equal(got, want)


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_library_host_code_runs_clean_under_sanitizers():
    from concurrent.futures import ThreadPoolExecutor

    from paper_2508_17892_amd import build as hip_build

    os.makedirs(OUT, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]

    def compile_one(src):
        obj = os.path.join(OUT, src.replace(".hip", ".o"))
        subprocess.run(["hipcc", *hip_build.FLAGS, *san, "-c", os.path.join(hip_build.CSRC, src), "-o", obj], check=True,
                       capture_output=True)
        return obj

    with ThreadPoolExecutor(max_workers=len(hip_build.SOURCES)) as pool:
        objs = list(pool.map(compile_one, hip_build.SOURCES))
    lib = os.path.join(OUT, "libilre_san.so")
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-fno-gpu-sanitize",
                    "-shared-libsan", "-o", lib, *objs], check=True, capture_output=True)
    clang = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    exe = os.path.join(OUT, "abi_driver")
    subprocess.run([clang, "-O1", "-g", "-std=c11", "-Wall", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-shared-libsan", "-I" + os.path.join(ROOT, "include"), "-o", exe, os.path.join(HERE, "abi_driver.c"),
                    lib, "-Wl,-rpath," + OUT], check=True, capture_output=True)
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    rt_dir = os.path.dirname(os.path.realpath(rt))
    env = dict(SAN_ENV, ASAN_OPTIONS=SAN_ENV["ASAN_OPTIONS"] + ":detect_leaks=0:verify_asan_link_order=0",
               LD_LIBRARY_PATH=rt_dir + os.pathsep + os.environ.get("LD_LIBRARY_PATH", ""))
    run = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, (run.stdout[-3000:], run.stderr[-3000:])
    assert "0 failures" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-3000:]
