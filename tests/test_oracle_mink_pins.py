"""Pins for the mirrored problem in the CPU oracle (the K smallest, smallest first, ties toward
the lowest index): against a rank-count formulation written here with plain loops, NumPy's stable
argsort, the negation and complement symmetries that tie it to the Top-K oracle (which has pins
of its own), and the K'=K and B=1 special cases."""
import numpy as np
import pytest

from oracle import oracle


def before_min(va, ia, vb, ib):
    """The mirrored order: smaller value first, equal values -> lower index first."""
    return va < vb or (va == vb and ia < ib)


def brute_force_min(row, K, Kp, B):
    N = len(row)
    surv = []
    for n in range(N):
        c = sum(1 for m in range(n % B, N, B) if m != n and before_min(row[m], m, row[n], n))
        if c < Kp:
            surv.append(n)
    out = [None] * K
    for n in surv:
        c = sum(1 for m in surv if m != n and before_min(row[m], m, row[n], n))
        if c < K:
            assert out[c] is None
            out[c] = n
    return out


def legal_params(N):
    for B in [b for b in range(1, N + 1) if N % b == 0]:
        for Kp in range(1, N // B + 1):
            for K in range(Kp, min(N, B * Kp) + 1):
                yield B, Kp, K


@pytest.mark.parametrize("N,symbols", [(12, 3), (24, 3), (30, 50)])
def test_min_k_matches_rank_count_brute_force_all_legal_params(N, symbols):
    rng = np.random.default_rng(N * 7 + symbols)
    x = rng.integers(0, symbols, size=(2, N)).astype(np.float32)
    x[0, 1] = -0.0            # compares equal to the other zeros
    for B, Kp, K in legal_params(N):
        vals, idx = oracle.approx_topk(x, K, Kp, B, smallest=True)
        for r in range(x.shape[0]):
            want = brute_force_min(x[r], K, Kp, B)
            assert idx[r].tolist() == want, (N, B, Kp, K, r)
            assert np.array_equal(vals[r].view(np.uint32), x[r][want].view(np.uint32))


def test_exact_min_k_matches_numpy_stable_argsort():
    rng = np.random.default_rng(5)
    for dtype in (np.float32, np.int32, np.uint32):
        x = (rng.integers(-40, 40, (6, 5000)) if dtype != np.uint32 else rng.integers(0, 80, (6, 5000))).astype(dtype)
        for K in (1, 17, 300, 5000):
            vals, idx = oracle.topk(x, K, smallest=True)
            want = np.argsort(x, axis=1, kind="stable")[:, :K]
            assert np.array_equal(idx, want)
            assert np.array_equal(vals, np.take_along_axis(x, want, axis=1))


def test_min_k_is_top_k_of_the_negated_or_complemented_row():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((5, 4096)).astype(np.float32)
    x[1] = np.round(x[1] * 2) / 2
    for K, Kp, B in [(32, 4, 64), (100, 1, 256), (7, 7, 1), (64, 2, 128)]:
        v, i = oracle.approx_topk(x, K, Kp, B, smallest=True)
        v2, i2 = oracle.approx_topk(-x, K, Kp, B)
        assert np.array_equal(i, i2) and np.array_equal(v, -v2)
        v, i = oracle.stage1(x, Kp, B, smallest=True)
        v2, i2 = oracle.stage1(-x, Kp, B)
        assert np.array_equal(i, i2) and np.array_equal(v, -v2)
    y = rng.integers(-2**31, 2**31, (4, 2048), dtype=np.int64)
    for arr in (y.astype(np.int32), (y & 0xffffffff).astype(np.uint32)):
        v, i = oracle.approx_topk(arr, 50, 2, 64, smallest=True)
        v2, i2 = oracle.approx_topk(~arr, 50, 2, 64)        # the complement reverses the order of integers
        assert np.array_equal(i, i2) and np.array_equal(v, ~v2)
        v, i = oracle.topk(arr, 50, smallest=True)
        v2, i2 = oracle.topk(~arr, 50)
        assert np.array_equal(i, i2) and np.array_equal(v, ~v2)


@pytest.mark.parametrize("B", [1, 2, 64, 128])
def test_min_k_special_cases_are_exact(B):
    rng = np.random.default_rng(B)
    x = rng.standard_normal((3, 4096)).astype(np.float32)
    K = 32
    ev, ei = oracle.topk(x, K, smallest=True)
    v, i = oracle.approx_topk(x, K, K, B, smallest=True)      # K' = K
    assert np.array_equal(i, ei) and np.array_equal(v, ev)
    v, i = oracle.approx_topk(x, K, K, 1, smallest=True)      # one bucket
    assert np.array_equal(i, ei) and np.array_equal(v, ev)
    # plus infinity everywhere but a few places: the real +inf elements fill the rest, lowest index first
    y = np.full((1, 256), np.inf, dtype=np.float32)
    y[0, [9, 200]] = [2.0, 1.0]
    v, i = oracle.approx_topk(y, 5, 2, 16, smallest=True)
    assert i[0].tolist() == [200, 9, 0, 1, 2]
