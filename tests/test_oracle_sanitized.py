"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the source
is compiled a second time with -fsanitize=address,undefined and a small set of its pins runs
through that build in a child process (the sanitizer runtime must be loaded before anything else,
hence LD_PRELOAD in the child only).  Any out-of-bounds access, signed overflow or misaligned
access in the oracle's loops aborts the child and fails the test."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SOURCE = os.path.join(ROOT, "oracle", "bigcn_oracle.c")

CHILD = textwrap.dedent("""
    import ctypes, sys
    import numpy as np
    sys.path.insert(0, {root!r})
    import oracle.reference as ref
    ref._LIB = None
    ref._build.LIBRARY = {lib!r}              # the sanitized build instead of the regular one
    import oracle
    rng = np.random.default_rng(3)
    # +-1 dot product against numpy, K on both sides of a word
    for k in (1, 63, 64, 65, 130):
        f = rng.choice(np.array([-1, 1], dtype=np.int8), size=(9, k))
        b = rng.choice(np.array([-1, 1], dtype=np.int8), size=(5, k))
        assert np.array_equal(oracle.sign_matmul(f, b), f.astype(np.int32) @ b.astype(np.int32).T)
    # sign / scale of a hand-written row, zeros count as +1
    s, beta = oracle.binarize_rows(np.array([[0.5, -2.0, 0.0, -0.0, 3.5]], dtype=np.float32))
    assert s.tolist() == [[1, -1, 1, 1, 1]] and abs(beta[0] - 6.0 / 5) < 1e-12
    # normalised adjacency of K4 with self-loops: every coefficient 1/4; aggregation of ones = ones
    row_ptr = np.arange(0, 17, 4, dtype=np.int64)
    col_idx = np.tile(np.arange(4, dtype=np.int32), 4)
    a = oracle.gcn_norm(row_ptr, col_idx)
    assert np.allclose(a, 0.25)
    assert np.allclose(oracle.aggregate(row_ptr, col_idx, a, np.ones((4, 3))), 1.0)
    # a whole two-layer forward on a 150-node graph (every loop of the library runs)
    from workloads import chung_lu_csr
    rp, ci = chung_lu_csr(150, 400, 2.5, 2.0, seed=1)
    x = rng.standard_normal((150, 70)).astype(np.float32)
    ws = [rng.uniform(-1, 1, size=(70, 33)).astype(np.float32), rng.uniform(-1, 1, size=(33, 4)).astype(np.float32)]
    out, _ = oracle.forward(rp, ci, x, ws, calibrate=[True, True])
    assert out.shape == (150, 4) and np.isfinite(out).all()
    labels, probs = oracle.predict(out)
    assert np.allclose(probs.sum(axis=1), 1.0)
    assert {lib!r} in open("/proc/self/maps").read(), "the sanitized library was not the one loaded"
    print("sanitized pins ok")
""")


def _runtime(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not available")
def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    asan, ubsan = _runtime("libasan.so"), _runtime("libubsan.so")
    if asan is None or ubsan is None:
        pytest.skip("gcc's sanitizer runtimes are not installed")
    lib = str(tmp_path / "libbigcn_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-omit-frame-pointer",
                    "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", lib, SOURCE, "-lm"],
                   check=True)
    env = dict(os.environ, LD_PRELOAD=f"{asan}:{ubsan}", ASAN_OPTIONS="detect_leaks=0:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1", OMP_NUM_THREADS="2")
    run = subprocess.run([sys.executable, "-c", CHILD.format(root=ROOT, lib=lib)], env=env, capture_output=True,
                         text=True, timeout=300)
    assert run.returncode == 0 and "sanitized pins ok" in run.stdout, run.stdout[-2000:] + run.stderr[-4000:]
