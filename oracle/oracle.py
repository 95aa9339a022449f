"""CPU oracle for the generalized two-stage approximate Top-K -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It shares nothing with the HIP library:
no kernels, headers, helpers, tables or constants.

Two parts:

* thin ``ctypes`` bindings to ``atk_oracle.c`` (the definition of the method,
  Section 6.1 Steps 1-4, written out with ``qsort``, and the same applied to the
  inner products of Section 7.3), taking and returning NumPy arrays;
* the theory of Section 6.2 / Theorem 1 in exact arithmetic: the closed-form
  expected recall, the K'=1 lower bound and bucket formula, a Monte-Carlo
  estimator of the same expectation, and the two recall measures used when
  comparing an approximate result with the exact one.

bf16 data travels as ``uint16`` arrays holding the raw bits.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "atk_oracle.c")
_LIB = os.path.join(_HERE, "libatk_oracle.so")

F32, BF16, F16, I32, U32 = 0, 1, 2, 3, 4


def build(force: bool = False) -> str:
    """Compile ``atk_oracle.c`` with gcc into ``oracle/libatk_oracle.so``."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.atk_oracle_stage1.argtypes = [vp, ci, i64, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_stage1.restype = ci
        lib.atk_oracle_approx_topk.argtypes = [vp, ci, i64, i64, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_approx_topk.restype = ci
        lib.atk_oracle_topk.argtypes = [vp, ci, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_topk.restype = ci
        lib.atk_oracle_approx_mink.argtypes = [vp, ci, i64, i64, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_approx_mink.restype = ci
        lib.atk_oracle_mink.argtypes = [vp, ci, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_mink.restype = ci
        lib.atk_oracle_stage1_min.argtypes = [vp, ci, i64, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_stage1_min.restype = ci
        lib.atk_oracle_num_threads.restype = ci
        lib.atk_oracle_mips_scores.argtypes = [vp, vp, ci, i64, i64, i64, vp]
        lib.atk_oracle_mips_scores.restype = ci
        lib.atk_oracle_mips_approx_topk.argtypes = [vp, vp, ci, i64, i64, i64, i64, i64, i64, vp, vp]
        lib.atk_oracle_mips_approx_topk.restype = ci
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the row loop of the C oracle will use."""
    return int(_load().atk_oracle_num_threads())


def _prep(values: np.ndarray):
    """float32, float16, int32 and uint32 arrays as they are; bf16 travels as uint16 bit patterns."""
    if values.ndim != 2:
        raise ValueError("values must be [rows, N]")
    codes = {np.dtype(np.float32): F32, np.dtype(np.uint16): BF16, np.dtype(np.float16): F16,
             np.dtype(np.int32): I32, np.dtype(np.uint32): U32}
    if values.dtype not in codes:
        raise TypeError("values must be float32, float16, int32, uint32, or uint16 holding bf16 bits")
    return np.ascontiguousarray(values), codes[values.dtype]


def _raise(rc: int, what: str):
    if rc == 0:
        return
    msg = {-1: "invalid arguments", -2: "NaN in input (precondition: no NaN)",
           -3: "out of memory"}.get(rc, f"error {rc}")
    raise ValueError(f"{what}: {msg}")


def approx_topk(values: np.ndarray, K: int, Kprime: int, B: int, smallest: bool = False):
    """Section 6.1 Steps 1-4.  Returns (vals[rows,K] in the input dtype, idx[rows,K] int32).
    smallest: the mirrored problem (the K smallest, smallest first, ties toward the lowest index)."""
    values, dtype = _prep(values)
    rows, N = values.shape
    out_vals = np.empty((rows, K), dtype=values.dtype)
    out_idx = np.empty((rows, K), dtype=np.int32)
    fn = _load().atk_oracle_approx_mink if smallest else _load().atk_oracle_approx_topk
    rc = fn(values.ctypes.data, dtype, rows, N, N, K, Kprime, B, out_vals.ctypes.data, out_idx.ctypes.data)
    _raise(rc, "oracle approx_topk")
    return out_vals, out_idx


def topk(values: np.ndarray, K: int, smallest: bool = False):
    """Exact Top-K (or min-K) under the same total order.  Returns (vals[rows,K], idx[rows,K])."""
    values, dtype = _prep(values)
    rows, N = values.shape
    out_vals = np.empty((rows, K), dtype=values.dtype)
    out_idx = np.empty((rows, K), dtype=np.int32)
    fn = _load().atk_oracle_mink if smallest else _load().atk_oracle_topk
    rc = fn(values.ctypes.data, dtype, rows, N, N, K, out_vals.ctypes.data, out_idx.ctypes.data)
    _raise(rc, "oracle topk")
    return out_vals, out_idx


def stage1(values: np.ndarray, Kprime: int, B: int, smallest: bool = False):
    """Steps 1-2 only: survivors as (vals[rows,K',B], idx[rows,K',B]), Section 6.3 layout."""
    values, dtype = _prep(values)
    rows, N = values.shape
    sv = np.empty((rows, Kprime, B), dtype=values.dtype)
    si = np.empty((rows, Kprime, B), dtype=np.int32)
    fn = _load().atk_oracle_stage1_min if smallest else _load().atk_oracle_stage1
    rc = fn(values.ctypes.data, dtype, rows, N, N, Kprime, B, sv.ctypes.data, si.ctypes.data)
    _raise(rc, "oracle stage1")
    return sv, si


def _prep_vectors(queries: np.ndarray, database: np.ndarray):
    if queries.ndim != 2 or database.ndim != 2 or queries.shape[1] != database.shape[1]:
        raise ValueError("queries must be [Q, D] and database [N, D]")
    if queries.dtype != database.dtype or queries.dtype not in (np.dtype(np.uint16), np.dtype(np.float16)):
        raise TypeError("vectors are float16 arrays, or bf16 bit patterns held in uint16 arrays")
    code = BF16 if queries.dtype == np.dtype(np.uint16) else F16
    return np.ascontiguousarray(queries), np.ascontiguousarray(database), code


def mips_scores(queries: np.ndarray, database: np.ndarray) -> np.ndarray:
    """Section 7.3: the [Q, N] inner products of bf16 vectors, each correctly rounded to float32."""
    queries, database, code = _prep_vectors(queries, database)
    Q, D = queries.shape
    N = database.shape[0]
    scores = np.empty((Q, N), dtype=np.float32)
    rc = _load().atk_oracle_mips_scores(queries.ctypes.data, database.ctypes.data, code, Q, N, D,
                                        scores.ctypes.data)
    _raise(rc, "oracle mips_scores")
    return scores


def mips_approx_topk(queries: np.ndarray, database: np.ndarray, K: int, Kprime: int, B: int):
    """Section 7.3: Steps 1-4 of Section 6.1 on every row of the score matrix, which is never
    stored as a whole.  Returns (scores[Q,K] float32, idx[Q,K] int32)."""
    queries, database, code = _prep_vectors(queries, database)
    Q, D = queries.shape
    N = database.shape[0]
    out_vals = np.empty((Q, K), dtype=np.float32)
    out_idx = np.empty((Q, K), dtype=np.int32)
    rc = _load().atk_oracle_mips_approx_topk(queries.ctypes.data, database.ctypes.data, code, Q, N, D,
                                             K, Kprime, B, out_vals.ctypes.data,
                                             out_idx.ctypes.data)
    _raise(rc, "oracle mips_approx_topk")
    return out_vals, out_idx


# --------------------------------------------------------------------------
# Theory (Section 6.2, Theorem 1 and its proof in the appendix)
# --------------------------------------------------------------------------

def expected_excess_per_bucket(N: int, B: int, K: int, Kprime: int) -> Fraction:
    """m_j = E[max(0, X - K')] for X ~ Hypergeometric(N, K, N/B), as an exact fraction.

    Proof of Theorem 1: sum over r = K'+1 .. min(K, N/B) of
    (r - K') * C(K, r) * C(N-K, N/B - r) / C(N, N/B).
    """
    if N % B:
        raise ValueError("B must divide N")
    n = N // B
    total = 0
    for r in range(Kprime + 1, min(K, n) + 1):
        if n - r > N - K:
            continue  # C(N-K, n-r) = 0
        total += (r - Kprime) * math.comb(K, r) * math.comb(N - K, n - r)
    return Fraction(total, math.comb(N, n))


def expected_recall(N: int, B: int, K: int, Kprime: int) -> float:
    """Theorem 1: E[recall] = 1 - (B/K) * m_j, evaluated in exact rational arithmetic."""
    m = expected_excess_per_bucket(N, B, K, Kprime)
    return float(1 - Fraction(B, K) * m)


def recall_lower_bound_k1(N: int, B: int, K: int) -> float:
    """K'=1 bound from the proof of Theorem 1: E[recall] >= 1 - (K/2)(1/B - 1/N)."""
    return 1.0 - (K / 2.0) * (1.0 / B - 1.0 / N)


def buckets_for_recall_k1(N: int, K: int, r: float) -> float:
    """Theorem 1: for K'=1, B = K / (2 (1 - r + K/(2N))) buckets suffice for recall r."""
    return K / (2.0 * (1.0 - r + K / (2.0 * N)))


def select_parameters(N: int, K: int, recall_target: float, allowed_kprime=(1, 2, 3, 4),
                      bucket_multiple: int = 128):
    """Parameter sweep of the appendix "Algorithm Parameter Selection", with the exact closed
    form in place of the Monte-Carlo estimate: over K' in `allowed_kprime` and every divisor B
    of N that is a multiple of `bucket_multiple`, with K' <= N/B and B*K' >= K, keep the
    configuration with the fewest stage-1 survivors B*K' whose expected recall reaches the
    target; on ties the smaller K'.  Plain exhaustive enumeration.  Returns (K', B) or None.
    """
    divisors = [d for d in range(1, N + 1) if N % d == 0] if N <= 4096 else sorted(
        {d for i in range(1, int(math.isqrt(N)) + 1) if N % i == 0 for d in (i, N // i)})
    best = None
    for kp in sorted(allowed_kprime):
        for B in divisors:
            if B % bucket_multiple or B * kp < K or kp > N // B or kp > K:
                continue
            if best is not None and B * kp >= best[0]:
                continue
            if expected_recall(N, B, K, kp) >= recall_target:
                best = (B * kp, kp, B)
    return None if best is None else (best[1], best[2])


def mips_select_parameters(N: int, K: int, recall_target: float):
    """Fusion-aware rule for the matmul-fused kernel (the paper's conclusion names fusion-aware
    selection as open work): every score costs about 5K'-2 list operations whatever B is
    (Section 6.3), so take the smallest K' <= 4 for which a legal B reaches the target by
    Theorem 1, then the smallest such B.  Legal: B divides N, B a multiple of 32,
    K <= B*K' <= 16384, K' <= N/B.  Plain enumeration, exact arithmetic.  Returns (K', B) or None.
    """
    for kp in range(1, min(4, K) + 1):
        for B in range(32, 16384 // kp + 1, 32):
            if N % B or B * kp < K or kp > N // B:
                continue
            if expected_recall(N, B, K, kp) >= recall_target:
                return kp, B
    return None


def expected_recall_mc(N: int, B: int, K: int, Kprime: int, num_trials: int,
                       rng: np.random.Generator):
    """Monte-Carlo estimate of the same expectation (Section 6.2; appendix on parameter selection).

    Draws the number of top-K elements landing in one bucket, X ~ Hypergeometric
    (K good, N-K bad, N/B draws); every bucket has this marginal, so the recall
    sample is 1 - B * max(X - K', 0) / K.  Returns (mean, standard error).
    """
    n = N // B
    x = rng.hypergeometric(K, N - K, n, size=num_trials)
    recall = 1.0 - B * np.maximum(x - Kprime, 0) / K
    return float(recall.mean()), float(recall.std(ddof=1) / math.sqrt(num_trials))


# --------------------------------------------------------------------------
# Recall of one result against the exact one (Section 3: |U ∩ V| / |U|)
# --------------------------------------------------------------------------

def index_recall(idx_approx: np.ndarray, idx_exact: np.ndarray) -> np.ndarray:
    """Per row: fraction of the exact Top-K positions that the approximate result holds."""
    out = np.empty(idx_exact.shape[0], dtype=np.float64)
    for r in range(idx_exact.shape[0]):
        out[r] = len(np.intersect1d(idx_approx[r], idx_exact[r])) / idx_exact.shape[1]
    return out


def value_recall(vals_approx_f32: np.ndarray, vals_exact_f32: np.ndarray) -> np.ndarray:
    """Per row: fraction of returned values that are >= the exact K-th value.

    Tie tolerant: when the K-th value is repeated, any holder of it counts.
    Both inputs are float32 views of the returned values.
    """
    kth = vals_exact_f32[:, -1:]
    return (vals_approx_f32 >= kth).mean(axis=1)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen raw bf16 bit patterns (uint16) to float32 (exact)."""
    return (bits.astype(np.uint32) << 16).view(np.float32)


# --------------------------------------------------------------------------
# Vector-throughput probe programs (appendix "Estimating peak VPU throughput")
# --------------------------------------------------------------------------

def valu_probe(kind: int, x: np.ndarray, y: np.ndarray, ops: int) -> np.ndarray:
    """What the two probe programs compute, in wrap-around 32-bit arithmetic.

    kind 0: `ops` steps of (x, y) -> (y, x + y), result y;  kind 1: x squared `ops` times.
    """
    a = x.astype(np.uint32).copy()
    if kind == 0:
        b = y.astype(np.uint32).copy()
        for _ in range(ops):
            a, b = b, a + b
        return b
    for _ in range(ops):
        a = a * a
    return a
