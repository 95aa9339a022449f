"""Pins of the oracle's inner-product search (Section 7.3): what it computes is fixed by
things other than itself: a library matrix product, a database of scaled unit vectors that
turns the scores into a table known in closed form, and a brute-force count on tiny inputs."""
import numpy as np
import pytest

from oracle import oracle
from paper_2506_04165_amd import workloads


def bits(t):
    return workloads.to_numpy_bits(t)


def test_scores_match_library_matmul_in_float64():
    q, d = workloads.mips_vectors(7, 300, seed=3, dim=128)
    s = oracle.mips_scores(bits(q), bits(d))
    ref = q.double().numpy() @ d.double().numpy().T          # LAPACK/BLAS routine, own summation order
    assert s.shape == (7, 300) and s.dtype == np.float32
    # a float64 sum of 128 exact products is within 1e-15 of the truth; rounding either to
    # float32 gives the same number except when the truth sits within 1e-15 of a rounding boundary
    assert (s == ref.astype(np.float32)).mean() > 0.999
    assert np.abs(s.astype(np.float64) - ref).max() <= 2.0 ** -24 * np.abs(ref).max() * 1.01


def test_fp16_vectors_match_library_matmul_in_float64():
    import torch
    q, d = workloads.mips_vectors(5, 200, seed=7, dim=64, dtype=torch.float16)
    s = oracle.mips_scores(q.numpy(), d.numpy())
    ref = q.double().numpy() @ d.double().numpy().T
    assert (s == ref.astype(np.float32)).mean() > 0.999
    assert np.abs(s.astype(np.float64) - ref).max() <= 2.0 ** -24 * np.abs(ref).max() * 1.01
    qi, di = workloads.mips_vectors(5, 200, seed=8, dim=64, kind="integer", dtype=torch.float16)
    assert (oracle.mips_scores(qi.numpy(), di.numpy()) == qi.long().numpy() @ di.long().numpy().T).all()


def test_integer_vectors_give_exact_integer_scores():
    q, d = workloads.mips_vectors(5, 257, seed=4, dim=64, kind="integer")
    s = oracle.mips_scores(bits(q), bits(d))
    ref = q.long().numpy() @ d.long().numpy().T               # integer arithmetic
    assert (s == ref).all()


def test_scaled_unit_vector_database_reduces_to_a_known_table():
    # database[n] = c_n * e_(n mod D): score[r][n] = queries[r][n mod D] * c_n, one exact product.
    # Transposing an operand or indexing the wrong axis anywhere changes the table.
    D, N, Q = 16, 192, 4
    rng = np.random.default_rng(5)
    qf = rng.integers(-8, 9, (Q, D)).astype(np.float32)
    c = rng.integers(1, 6, N).astype(np.float32)
    dbf = np.zeros((N, D), np.float32)
    dbf[np.arange(N), np.arange(N) % D] = c
    to_bits = lambda x: (x.view(np.uint32) >> 16).astype(np.uint16)   # small integers are exact in bf16
    table = qf[:, np.arange(N) % D] * c[None, :]
    assert (oracle.mips_scores(to_bits(qf), to_bits(dbf)) == table).all()
    for K, Kp, B in [(8, 1, 16), (8, 2, 8), (12, 3, 4), (5, 5, 1)]:
        v, i = oracle.mips_approx_topk(to_bits(qf), to_bits(dbf), K, Kp, B)
        ev, ei = oracle.approx_topk(np.ascontiguousarray(table), K, Kp, B)   # pinned elsewhere
        assert (v == ev).all() and (i == ei).all()


@pytest.mark.parametrize("K,Kp,B", [(4, 1, 8), (6, 2, 4), (3, 3, 2)])
def test_tiny_case_by_rank_counting(K, Kp, B):
    q, d = workloads.mips_vectors(2, 24, seed=6, dim=8, kind="integer")
    qf, df = q.float().numpy(), d.float().numpy()
    v, i = oracle.mips_approx_topk(bits(q), bits(d), K, Kp, B)
    for r in range(2):
        score = [sum(float(qf[r, k]) * float(df[n, k]) for k in range(8)) for n in range(24)]
        ahead = lambda a, b: score[a] > score[b] or (score[a] == score[b] and a < b)
        surv = [n for n in range(24)
                if sum(ahead(m, n) for m in range(24) if m % B == n % B) < Kp]
        final = sorted((n for n in surv if sum(ahead(m, n) for m in surv) < K),
                       key=lambda n: sum(ahead(m, n) for m in surv))
        assert final == list(i[r])
        assert [score[n] for n in final] == list(v[r])


def test_bad_arguments():
    q, d = workloads.mips_vectors(2, 24, seed=6, dim=8)
    with pytest.raises(ValueError):
        oracle.mips_approx_topk(bits(q), bits(d), 4, 1, 7)      # B does not divide N
    with pytest.raises(ValueError):
        oracle.mips_scores(bits(q), bits(d)[:, :4])
