"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer (host code only) and driven through
every exported routine in a child process: empty, tiny and ragged inputs, carried states, all boundary rules.
A memory error or undefined behaviour in the oracle aborts the child and fails the test."""
import os
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
import ctypes, sys
import numpy as np
lib = ctypes.CDLL(sys.argv[1])
dp = ctypes.POINTER(ctypes.c_double); fp = ctypes.POINTER(ctypes.c_float); ip = ctypes.POINTER(ctypes.c_int32)
P = lambda a: None if a is None else a.ctypes.data_as(dp)
rng = np.random.default_rng(0)
for (B, Hh, n, d, W, start, mode) in ((1, 1, 0, 2, 3, 0, 0), (1, 2, 1, 1, 1, 0, 0), (2, 2, 7, 3, 3, 2, 1), (1, 3, 9, 4, 4, 5, 2)):
    gam = rng.uniform(0.3, 1.0, Hh).astype(np.float32)
    lam32 = np.empty((Hh, n), np.float32); cum = np.empty(n + 1, np.int32)
    assert lib.lasad_oracle_decay_factors(gam.ctypes.data_as(fp), Hh, 4, W, start, n, mode, lam32.ctypes.data_as(fp), cum.ctypes.data_as(ip)) == 0
    lam = lam32.astype(np.float64)
    q, k, v, g = (np.ascontiguousarray(rng.standard_normal((B, Hh, n, d))) for _ in range(4))
    s0, h = (np.ascontiguousarray(rng.standard_normal((B, Hh, d, d))) for _ in range(2))
    o = np.empty_like(q); s1 = np.empty_like(s0)
    for name in ("lasad_oracle_forward_fullmask", "lasad_oracle_recurrent"):
        assert getattr(lib, name)(P(q), P(k), P(v), P(lam), ctypes.c_double(0.7), P(s0), P(o), P(s1), B, Hh, n, d) == 0
        assert getattr(lib, name)(P(q), P(k), P(v), P(lam), ctypes.c_double(0.7), None, P(o), None, B, Hh, n, d) == 0
    if n:
        st = s0.copy(); o1 = np.empty((B, Hh, d))
        lt = np.ascontiguousarray(lam[:, 0])
        assert lib.lasad_oracle_decode_step(P(np.ascontiguousarray(q[:, :, 0])), P(np.ascontiguousarray(k[:, :, 0])),
                                            P(np.ascontiguousarray(v[:, :, 0])), P(lt), ctypes.c_double(1.0), P(st), P(o1), B, Hh, d) == 0
        ob = np.empty((n, d))
        assert lib.lasad_oracle_bruteforce(P(np.ascontiguousarray(q[0, 0])), P(np.ascontiguousarray(k[0, 0])), P(np.ascontiguousarray(v[0, 0])),
                                           P(np.ascontiguousarray(lam[0])), ctypes.c_double(1.0), P(ob), n, d) == 0
    dq, dk, dv = np.empty_like(q), np.empty_like(q), np.empty_like(q)
    dlam = np.empty((B, Hh, n)); ds0 = np.empty_like(s0); dgam = np.empty(Hh)
    assert lib.lasad_oracle_backward(P(q), P(k), P(v), P(lam), ctypes.c_double(0.7), P(g), P(dq), P(dk), P(dv), P(dlam), B, Hh, n, d) == 0
    assert lib.lasad_oracle_backward_carried(P(q), P(k), P(v), P(lam), ctypes.c_double(0.7), P(g), P(s0), P(h),
                                             P(dq), P(dk), P(dv), P(dlam), P(ds0), B, Hh, n, d) == 0
    assert lib.lasad_oracle_dgamma(P(dlam), B, Hh, n, W, start, mode, P(dgam)) == 0
    gate = np.ascontiguousarray(rng.uniform(0.2, 1.0, (B, Hh, n, d)))
    for key in (None, k):
        assert lib.lasad_oracle_gated_recurrent(P(q), P(gate), P(key), P(v), ctypes.c_double(1.1), P(s0), P(o), P(s1), B, Hh, n, d, W, start, mode) == 0
        dkk = None if key is None else dk
        assert lib.lasad_oracle_gated_backward(P(q), P(gate), P(key), P(v), ctypes.c_double(1.1), P(g), P(dq), P(o), P(dkk), P(dv),
                                               B, Hh, n, d, W, start, mode) == 0
        assert lib.lasad_oracle_gated_backward_carried(P(q), P(gate), P(key), P(v), ctypes.c_double(1.1), P(g), P(s0), P(h),
                                                       P(dq), P(o), P(dkk), P(dv), P(ds0), B, Hh, n, d, W, start, mode) == 0
        if n:
            ob = np.empty((n, d))
            kk = None if key is None else np.ascontiguousarray(key[0, 0])
            assert lib.lasad_oracle_gated_bruteforce(P(np.ascontiguousarray(q[0, 0])), P(np.ascontiguousarray(gate[0, 0])), P(kk),
                                                     P(np.ascontiguousarray(v[0, 0])), ctypes.c_double(1.0), P(ob), n, d, W, start, mode) == 0
assert lib.lasad_oracle_num_threads() >= 1
print("SANITIZED RUN OK")
"""


def test_oracle_under_address_and_undefined_behaviour_sanitizers():
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    asan = subprocess.run([gcc, "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("this gcc has no libasan")
    with tempfile.TemporaryDirectory() as tmp:
        so = os.path.join(tmp, "liblasad_oracle_san.so")
        subprocess.run([gcc, "-O1", "-g", "-fPIC", "-shared", "-fopenmp", "-fsanitize=address,undefined",
                        "-fno-sanitize-recover=all", os.path.join(ROOT, "oracle", "lasad_oracle.c"), "-o", so, "-lm"], check=True)
        env = dict(os.environ, LD_PRELOAD=asan + (":" + os.environ["LD_PRELOAD"] if os.environ.get("LD_PRELOAD") else ""),
                   ASAN_OPTIONS="detect_leaks=0", OMP_NUM_THREADS="2")
        r = subprocess.run([sys.executable, "-c", DRIVER, so], env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "SANITIZED RUN OK" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
