"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU, no GPU sanitizer).

Two sanitizer builds, each exercised in a child process that preloads the sanitizer runtime:
  * the C oracle (gcc -fsanitize=address,undefined) on ragged shapes through every entry point it has;
  * the host side of the C-ABI library (api.hip compiled with the sanitizers for the host pass only, linked with
    the ordinary device objects) through the argument checks of tests/test_abi.py.
A sanitizer report ends the child with a nonzero status.
"""
import glob
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
           PYTHONPATH=ROOT + os.pathsep + os.path.join(ROOT, "tests"))

ORACLE_CASES = r"""
import numpy as np
import oracle
rng = np.random.default_rng(5)
for (B, H, N, d, w) in [(1, 1, 1, 8, 1), (2, 3, 37, 16, 5), (1, 2, 70, 64, 200), (1, 1, 129, 128, 64)]:
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    alpha = -np.abs(rng.standard_normal((B, H, N)))
    c = oracle.gate_prefix(alpha)
    O, L = oracle.forward_from_c(Q, K, V, c, w, d ** -0.5)
    g = oracle.backward_from_c(Q, K, V, c, dO, w, d ** -0.5, return_dS=True)
    g2 = oracle.backward_from_c(Q, K, V, c, dO, w, d ** -0.5, O_saved=O.astype(np.float32))
    g3 = oracle.backward(Q, K, V, alpha, dO, w, d ** -0.5)
    da = oracle.dalpha_direct(g["dS"], w)
    for x in (O, L, da) + tuple(g.values()) + tuple(g2.values()) + tuple(g3.values()):
        assert np.isfinite(np.asarray(x)).all()
h, beta = rng.standard_normal((2, 3, 50)), rng.standard_normal((2, 3, 50))
a = oracle.gate_activation(h, beta, 1e-6)
dh, db = oracle.gate_activation_backward(h, beta, 1e-6, rng.standard_normal((2, 3, 50)))
assert np.isfinite(a).all() and np.isfinite(dh).all() and np.isfinite(db).all()
print("oracle under sanitizers: ok")
"""


def run(cmd, **kw):
    return subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)


def test_oracle_under_asan_ubsan(tmp_path):
    lib = str(tmp_path / "libgfwa_oracle_san.so")
    r = run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fsanitize=address,undefined",
             "-fno-sanitize-recover=all", "-o", lib, os.path.join(ROOT, "oracle", "gfwa_oracle.c"), "-lm"])
    assert r.returncode == 0, r.stdout
    asan = run(["gcc", "-print-file-name=libasan.so"]).stdout.strip()
    if not os.path.isabs(asan):
        pytest.skip("gcc has no shared AddressSanitizer runtime")
    env = dict(ENV, LD_PRELOAD=asan, GFWA_ORACLE_LIB=lib, OMP_NUM_THREADS="2")
    r = run([sys.executable, "-c", ORACLE_CASES], env=env, cwd=ROOT, timeout=600)
    assert r.returncode == 0 and "oracle under sanitizers: ok" in r.stdout, r.stdout[-4000:]


def test_abi_host_side_under_asan_ubsan(tmp_path):
    objdir = os.path.join(ROOT, "paper_2512_07782_amd", "_build")
    others = [o for o in glob.glob(os.path.join(objdir, "*.o")) if os.path.basename(o) not in ("api.o", "fwd_bf16_pipe.o")]
    if len(others) < 6:
        pytest.skip("the library's object files are not built here")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    rt = glob.glob("/opt/rocm/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    if not os.path.exists(hipcc) or not rt:
        pytest.skip("no hipcc or no shared AddressSanitizer runtime of its clang")
    obj, lib = str(tmp_path / "api_san.o"), str(tmp_path / "libgfwa_san.so")
    csrc = os.path.join(ROOT, "paper_2512_07782_amd", "csrc")
    r = run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-Xclang", "-target-feature",
             "-Xclang", "-packed-fp32-ops", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=all", "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
             "-c", os.path.join(csrc, "api.hip"), "-o", obj], timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    r = run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan", "-fsanitize=address", "-fsanitize=undefined",
             "-fno-gpu-sanitize", "-o", lib, obj] + others, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    env = dict(ENV, LD_PRELOAD=rt[0], GFWA_LIB=lib)
    r = run([sys.executable, "-m", "pytest", "-q", "-x", "-p", "no:cacheprovider", os.path.join(ROOT, "tests", "test_abi.py")],
            env=env, cwd=ROOT, timeout=600)
    assert r.returncode == 0 and " passed" in r.stdout, r.stdout[-4000:]
