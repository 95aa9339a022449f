"""The CPU oracle and the library's host-only arithmetic under AddressSanitizer and
UndefinedBehaviorSanitizer (no GPU code is involved; GPU sanitizers are not available).

Two small drivers under tests/sanitize/ are compiled with -fsanitize=address,undefined together
with the sources they exercise and run as child processes.  A sanitizer report makes the child
exit with an error; beyond that, what the sanitized build returns must equal what the ordinary
build returns, byte for byte.
"""
import os
import subprocess

import numpy as np
import pytest

from oracle import oracle

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:exitcode=97",
           UBSAN_OPTIONS="halt_on_error=1:exitcode=98", OMP_NUM_THREADS="4")
ENV.pop("LD_PRELOAD", None)       # ASan insists on being the first library loaded


@pytest.fixture(scope="module")
def oracle_driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_driver")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", "-Wall", "-Wextra"] + SAN +
                   [os.path.join(HERE, "sanitize", "oracle_driver.c"), os.path.join(ROOT, "oracle", "atk_oracle.c"),
                    "-o", exe, "-lm"], check=True)
    return exe


@pytest.fixture(scope="module")
def host_driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "host_driver")
    csrc = os.path.join(ROOT, "paper_2506_04165_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                   [os.path.join(HERE, "sanitize", "host_driver.cpp"), os.path.join(csrc, "recall.cpp"),
                    os.path.join(csrc, "select_params.cpp"), "-o", exe, "-lm"], check=True)
    return exe


def _values(rng, dtype, rows, N, stride, style):
    """Raw input array [rows, stride] of the given oracle element type, trimmed to end at the
    last row's N-th element."""
    if dtype in (oracle.I32, oracle.U32):
        lo, hi = (-(1 << 31), 1 << 31) if style == 0 else (-3, 3)
        a = rng.integers(lo, hi, (rows, stride), dtype=np.int64)
        a = (a & 0xffffffff).astype(np.uint32) if dtype == oracle.U32 else a.astype(np.int32)
    else:
        f = rng.standard_normal((rows, stride)).astype(np.float32)
        if style == 1:
            f = np.round(f * 2) / 2                  # dense ties, both zeros
            f[f == 0] *= np.where(rng.random(f.shape) < 0.5, -1.0, 1.0)[f == 0]
        elif style == 2:
            f[rng.random(f.shape) < 0.7] = -np.inf
        if dtype == oracle.F32:
            a = f
        elif dtype == oracle.F16:
            a = f.astype(np.float16)
        else:
            a = (f.view(np.uint32) >> 16).astype(np.uint16)      # bf16 by truncation
    return a


def _library_call(op, a, rows, N, stride, K, Kp, B):
    """The ordinary build on the same (strided) input, through oracle.py's own loader."""
    lib = oracle._load()
    _, code = oracle._prep(a[:, :1])
    if op == 2:
        ov = np.empty((rows, Kp, B), dtype=a.dtype)
        oi = np.empty((rows, Kp, B), dtype=np.int32)
        rc = lib.atk_oracle_stage1(a.ctypes.data, code, rows, N, stride, Kp, B, ov.ctypes.data, oi.ctypes.data)
    else:
        ov = np.empty((rows, K), dtype=a.dtype)
        oi = np.empty((rows, K), dtype=np.int32)
        if op == 0:
            rc = lib.atk_oracle_approx_topk(a.ctypes.data, code, rows, N, stride, K, Kp, B, ov.ctypes.data, oi.ctypes.data)
        else:
            rc = lib.atk_oracle_topk(a.ctypes.data, code, rows, N, stride, K, ov.ctypes.data, oi.ctypes.data)
    return rc, ov, oi


def test_oracle_is_clean_under_asan_and_ubsan(oracle_driver):
    rng = np.random.default_rng(42)
    dtypes = [oracle.F32, oracle.BF16, oracle.F16, oracle.I32, oracle.U32]
    shapes = [(1, 1, 1, 1, 1), (3, 64, 64, 1, 64), (2, 60, 6, 10, 60), (5, 4096, 64, 4, 32),
              (4, 1000, 125, 1, 100), (3, 210, 7, 30, 210), (7, 96, 1, 96, 96), (2, 14336, 128, 4, 287),
              (0, 128, 8, 2, 5), (6, 512, 512, 1, 500)]
    request, expected = bytearray(), []
    for case, (rows, N, B, Kp, K) in enumerate(shapes):
        for op in (0, 1, 2):
            dtype = dtypes[(case + op) % 5]
            stride = N + (case % 3) * 5
            a = np.ascontiguousarray(_values(rng, dtype, max(rows, 1), N, stride, (case + op) % 3))[:rows]
            flat = a.reshape(-1)[:((rows - 1) * stride + N) if rows else 0]
            request += np.array([op, dtype, rows, N, stride, K, Kp, B, 0], dtype=np.int64).tobytes()
            request += flat.tobytes()
            expected.append((op, rows, K, Kp, B, a.dtype) + _library_call(op, a if rows else np.zeros((1, stride), a.dtype)[:0], rows, N, stride, K, Kp, B))
    # the inner-product search of Section 7.3
    for (Q, N, D, K, Kp, B) in [(3, 256, 16, 20, 2, 32), (1, 64, 128, 64, 1, 64), (5, 96, 8, 7, 3, 4)]:
        q = rng.integers(-2, 3, (Q, D)).astype(np.float32)
        d = rng.integers(-2, 3, (N, D)).astype(np.float32)
        qb, db = (q.view(np.uint32) >> 16).astype(np.uint16), (d.view(np.uint32) >> 16).astype(np.uint16)
        request += np.array([3, oracle.BF16, Q, N, 0, K, Kp, B, D], dtype=np.int64).tobytes()
        request += qb.tobytes() + db.tobytes()
        ov, oi = oracle.mips_approx_topk(qb, db, K, Kp, B)
        expected.append((3, Q, K, Kp, B, np.dtype(np.float32), 0, ov, oi))
    # error paths: rejected before any access
    request += np.array([0, oracle.F32, 2, 8, 8, 3, 1, 3, 0], dtype=np.int64).tobytes() + np.zeros(16, np.float32).tobytes()
    expected.append((0, 2, 3, 1, 3, np.dtype(np.float32), -1, None, None))             # B does not divide N
    nan_row = np.array([1.0, np.nan, 2.0, 3.0], dtype=np.float32)
    request += np.array([1, oracle.F32, 1, 4, 4, 2, 0, 0, 0], dtype=np.int64).tobytes() + nan_row.tobytes()
    expected.append((1, 1, 2, 0, 0, np.dtype(np.float32), -2, None, None))             # NaN in the input

    p = subprocess.run([oracle_driver], input=bytes(request), capture_output=True, env=ENV, timeout=600)
    assert p.returncode == 0, p.stderr.decode()[-4000:]
    out, pos = p.stdout, 0
    for (op, rows, K, Kp, B, dt, rc, ov, oi) in expected:
        status = int(np.frombuffer(out, np.int64, 1, pos)[0]); pos += 8
        assert status == rc, (op, rows, K, Kp, B, status, rc)
        if rc != 0:
            continue
        n = rows * (Kp * B if op == 2 else K)
        got_v = np.frombuffer(out, dt, n, pos); pos += n * dt.itemsize
        got_i = np.frombuffer(out, np.int32, n, pos); pos += n * 4
        assert np.array_equal(got_i, oi.reshape(-1)), (op, rows, K, Kp, B)
        assert got_v.tobytes() == np.ascontiguousarray(ov).tobytes(), (op, rows, K, Kp, B)
    assert pos == len(out)


def test_sanitizer_build_does_catch_an_overrun(tmp_path):
    # the harness itself: a planted one-past-the-end read must make the child fail
    src = tmp_path / "overrun.c"
    src.write_text("#include <stdlib.h>\nint main(void){volatile int *a = malloc(16); int r = a[4]; free((void*)a); return r & 0;}\n")
    exe = str(tmp_path / "overrun")
    subprocess.run(["gcc"] + SAN + [str(src), "-o", exe], check=True)
    p = subprocess.run([exe], capture_output=True, env=ENV)
    assert p.returncode in (97, 98) and (b"heap-buffer-overflow" in p.stderr or b"runtime error" in p.stderr)


def test_host_arithmetic_is_clean_under_asan_and_ubsan(host_driver):
    from paper_2506_04165_amd import binding as atk
    cases = [(262144, 1024, 0.99, 4, 64), (14336, 287, 0.95, 8, 64), (1048576, 128, 0.999, 4, 64),
             (430080, 3360, 0.95, 4, 128), (4096, 32, 0.9999999, 4, 64), (60, 7, 0.5, 2, 1), (1, 1, 1.0, 1, 1),
             (2147418112, 1024, 0.9, 4, 64), (65536, 65536, 0.9, 4, 64), (1000003, 10, 0.9, 4, 1),
             (0, 1, 0.5, 4, 64), (100, 200, 0.5, 4, 64), (4096, 32, 1.5, 4, 64), (4096, 32, 0.9, 0, 64)]
    text = "".join("%d %d %r %d %d\n" % c for c in cases)
    p = subprocess.run([host_driver], input=text.encode(), capture_output=True, env=ENV, timeout=600)
    assert p.returncode == 0, p.stderr.decode()[-4000:]
    lines = p.stdout.decode().splitlines()
    assert len(lines) == len(cases)
    import ctypes
    for (N, K, target, maxkp, mult), line in zip(cases, lines):
        s1, kp, b, r, s2, kp2, b2, r2, e = line.split()
        ckp, cb, cr = ctypes.c_int(-1), ctypes.c_int(-1), ctypes.c_double(-1.0)
        st = atk.lib.atk_select_params(N, K, target, maxkp, mult, ctypes.byref(ckp), ctypes.byref(cb), ctypes.byref(cr))
        assert (int(s1), int(kp), int(b)) == (st, ckp.value, cb.value), (N, K, target)
        assert float(r) == cr.value
        ckp, cb, cr = ctypes.c_int(-1), ctypes.c_int(-1), ctypes.c_double(-1.0)
        st = atk.lib.atk_mips_select_params(N, K, target, ctypes.byref(ckp), ctypes.byref(cb), ctypes.byref(cr))
        assert (int(s2), int(kp2), int(b2)) == (st, ckp.value, cb.value), (N, K, target)
        assert float(r2) == cr.value
        if int(s1) == 0:
            assert float(e) == atk.expected_recall(N, int(b), K, int(kp))
