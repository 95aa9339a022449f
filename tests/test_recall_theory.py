"""Pins for the expected-recall theory (Section 6.2, Theorem 1) and the link to the oracle.

The closed form is checked against the values the paper prints (Table 1), the K'=1
identity and bound from the proof of Theorem 1, SciPy's hypergeometric distribution,
the Monte-Carlo estimator of the same expectation, and -- the link between theory and
the oracle's selection -- the oracle's empirical recall over 10^4 seeded random
permutations, which must agree with the closed form to 0.005 absolute.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_expected_recall.txt")


def table1_rows():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        kp, b, printed, pm, usable = line.split()
        rows.append((int(kp), int(b), float(printed), float(pm), int(usable)))
    return rows


def test_closed_form_reproduces_table1():
    # Table 1: K=1024 of N=262144; printed to three decimals
    n_checked = 0
    for kp, b, printed, _pm, usable in table1_rows():
        if not usable:
            continue
        got = oracle.expected_recall(262144, b, 1024, kp)
        assert abs(got - printed) <= 0.001, (kp, b, printed, got)
        n_checked += 1
    assert n_checked == 15


def test_table1_flagged_rows_stay_flagged():
    # the two rows excluded above really do disagree with Theorem 1 (so the exclusion is not
    # hiding an oracle error): (8, 512) printed 0.992 is the (8, 256) value
    assert abs(oracle.expected_recall(262144, 512, 1024, 8) - 0.99986) < 1e-5
    assert abs(oracle.expected_recall(262144, 256, 1024, 8) - 0.992) <= 0.001
    assert abs(oracle.expected_recall(262144, 65536, 1024, 1) - 0.99416) < 1e-5


@pytest.mark.parametrize("N,B,K", [(4096, 64, 32), (262144, 8192, 1024), (14336, 1024, 287),
                                   (1048576, 4096, 128), (60, 6, 7)])
def test_kprime1_identity_and_bound(N, B, K):
    # proof of Theorem 1: m_j = K/B - 1 + C(N-K, N/B) / C(N, N/B) for K'=1
    n = N // B
    m = oracle.expected_excess_per_bucket(N, B, K, 1)
    assert m == Fraction(K, B) - 1 + Fraction(math.comb(N - K, n), math.comb(N, n))
    r = oracle.expected_recall(N, B, K, 1)
    assert r >= oracle.recall_lower_bound_k1(N, B, K) - 1e-12
    # the bound is within a factor ~2 of tight in the high-recall regime, never vacuous here
    assert oracle.recall_lower_bound_k1(N, B, K) <= 1.0


# Hand-evaluated points of 1 - (K/2)(1/B - 1/N) (last line of the proof of Theorem 1), written as
# exact binary fractions so that a dropped 1/2, a flipped sign of 1/N or swapped B and N fails:
#   (4096, 64, 32):      1 - 16 (64/4096 - 1/4096)        = 1 - 1008/4096     = 0.75390625
#   (262144, 8192, 1024): 1 - 512 (32/262144 - 1/262144)  = 1 - 15872/262144  = 0.939453125
#   (1024, 4, 2):        1 - 1 (256/1024 - 1/1024)        = 1 - 255/1024      = 0.7509765625
#   (65536, 256, 256):   1 - 128 (256/65536 - 1/65536)    = 1 - 32640/65536   = 0.501953125
@pytest.mark.parametrize("N,B,K,want", [(4096, 64, 32, 0.75390625), (262144, 8192, 1024, 0.939453125),
                                        (1024, 4, 2, 0.7509765625), (65536, 256, 256, 0.501953125)])
def test_kprime1_bound_at_hand_evaluated_points(N, B, K, want):
    assert oracle.recall_lower_bound_k1(N, B, K) == pytest.approx(want, abs=1e-15)
    # and the bound really lies below the exact value there
    assert oracle.expected_recall(N, B, K, 1) >= want


# Hand-evaluated points of B = K / (2 (1 - r + K/(2N))) (Theorem 1):
#   N=4096, K=32, r=0.75390625:  1 - r = 1008/4096, K/2N = 16/4096, sum = 1024/4096 = 1/4, B = 32/(2/4)   = 64
#   N=1024, K=2,  r=0.7509765625: 255/1024 + 1/1024 = 1/4,                                 B = 2/(2/4)    = 4
#   N=262144, K=1024, r=0.939453125: 15872/262144 + 512/262144 = 1/16,                     B = 1024/(2/16) = 8192
#   N=1000, K=100, r=0.9:  0.1 + 0.05 = 0.15,                                              B = 100/0.3    = 333.333...
@pytest.mark.parametrize("N,K,r,want", [(4096, 32, 0.75390625, 64.0), (1024, 2, 0.7509765625, 4.0),
                                        (262144, 1024, 0.939453125, 8192.0), (1000, 100, 0.9, 1000.0 / 3.0)])
def test_bucket_formula_at_hand_evaluated_points(N, K, r, want):
    assert oracle.buckets_for_recall_k1(N, K, r) == pytest.approx(want, rel=1e-13)


@pytest.mark.parametrize("N,K,r", [(262144, 1024, 0.95), (262144, 1024, 0.99), (1048576, 128, 0.98),
                                   (14336, 287, 0.9), (60, 7, 0.5)])
def test_bucket_formula_inverts_the_bound(N, K, r):
    # plugging the formula's B (a real number) back into the bound returns the target exactly:
    # the two functions are inverse to each other in B <-> r
    b = oracle.buckets_for_recall_k1(N, K, r)
    assert 1.0 - (K / 2.0) * (1.0 / b - 1.0 / N) == pytest.approx(r, abs=1e-12)
    # through the other function too (it takes B as a number)
    assert oracle.recall_lower_bound_k1(N, b, K) == pytest.approx(r, abs=1e-12)
    # r = 1 asks for one bucket per element: B = N
    assert oracle.buckets_for_recall_k1(N, K, 1.0) == pytest.approx(N, rel=1e-13)


@pytest.mark.parametrize("N,K,target", [(262144, 1024, 0.95), (262144, 1024, 0.99),
                                        (1048576, 128, 0.98)])
def test_bucket_formula_meets_target(N, K, target):
    # Theorem 1: B = K / (2 (1 - r + K/2N)) suffices; round up to a divisor of N (powers of two)
    b_real = oracle.buckets_for_recall_k1(N, K, target)
    B = 1 << math.ceil(math.log2(b_real))
    assert oracle.expected_recall(N, B, K, 1) >= target
    # and it is at most half of the older K / (1 - r) rule
    assert b_real < 0.5 * K / (1 - target) + 1e-9


@pytest.mark.parametrize("N,B,K,Kp", [(4096, 64, 32, 1), (4096, 64, 32, 4), (14336, 128, 287, 4),
                                      (14336, 64, 287, 8), (256000, 512, 64, 2),
                                      (65536, 256, 256, 8), (24, 4, 7, 2)])
def test_closed_form_matches_scipy_hypergeom(N, B, K, Kp):
    # X ~ Hypergeometric(population N, K marked, N/B draws); E[max(0, X-K')] = sum_{r>K'} P(X >= r)
    n = N // B
    X = stats.hypergeom(N, K, n)
    excess = sum(X.sf(r - 1) for r in range(Kp + 1, min(K, n) + 1))
    want = 1.0 - B * excess / K
    assert oracle.expected_recall(N, B, K, Kp) == pytest.approx(want, abs=1e-9)


def test_edge_cases_of_closed_form():
    assert oracle.expected_recall(4096, 64, 32, 32) == 1.0          # K' = K
    assert oracle.expected_recall(4096, 4096, 32, 1) == 1.0         # one element per bucket
    assert oracle.expected_recall(4096, 1, 32, 1) == pytest.approx(1 / 32)   # one bucket keeps one
    # monotone in K' and in B
    r = [oracle.expected_recall(14336, 128, 287, kp) for kp in range(1, 9)]
    assert all(a < b for a, b in zip(r, r[1:]))
    r = [oracle.expected_recall(16384, b, 256, 2) for b in (128, 256, 512, 1024)]
    assert all(a < b for a, b in zip(r, r[1:]))


@pytest.mark.parametrize("N,B,K,Kp", [(262144, 2048, 1024, 2), (14336, 128, 287, 4),
                                      (430080, 3360, 3360, 2)])
def test_monte_carlo_estimator_agrees(N, B, K, Kp):
    rng = np.random.default_rng(1234)
    mean, se = oracle.expected_recall_mc(N, B, K, Kp, 262144, rng)
    assert abs(mean - oracle.expected_recall(N, B, K, Kp)) < max(4 * se, 1e-4)


# The reference values below were evaluated from Theorem 1 in exact rational arithmetic
# outside this repository (they are not produced by oracle.expected_recall).
CONFIG_RECALL = [
    (4096, 64, 32, 1, 0.794050), (4096, 64, 32, 2, 0.970808), (4096, 64, 32, 4, 0.999753),
    (14336, 1024, 287, 1, 0.880091), (14336, 128, 287, 4, 0.951360), (14336, 64, 287, 8, 0.986646),
    (256000, 512, 64, 2, 0.997673), (1048576, 4096, 128, 1, 0.984714),
    (65536, 256, 256, 1, 0.633559),
]


@pytest.mark.parametrize("N,B,K,Kp,want", CONFIG_RECALL)
def test_closed_form_at_benchmark_configs(N, B, K, Kp, want):
    assert oracle.expected_recall(N, B, K, Kp) == pytest.approx(want, abs=2e-6)


def _empirical_recall(N, K, params, trials, seed, batch=500):
    """Mean index-recall of the oracle's approximate result against its exact result over
    `trials` seeded random permutations of N distinct values (exact in fp32 below 2^24)."""
    rng = np.random.default_rng(seed)
    sums = {p: 0.0 for p in params}
    base = np.arange(N, dtype=np.float32)
    done = 0
    while done < trials:
        nb = min(batch, trials - done)
        x = rng.permuted(np.broadcast_to(base, (nb, N)), axis=1)
        _, ei = oracle.topk(x, K)
        for (B, Kp) in params:
            _, ai = oracle.approx_topk(x, K, Kp, B)
            # distinct values: recall = |exact ∩ approx| / K (Section 3)
            hit = np.zeros(nb)
            for r in range(nb):
                hit[r] = np.isin(ei[r], ai[r], assume_unique=True).sum()
            sums[(B, Kp)] += hit.sum() / K
        done += nb
    return {p: s / trials for p, s in sums.items()}


@pytest.mark.parametrize("N,K,params", [
    (4096, 32, ((64, 1), (64, 2), (64, 4), (16, 4))),
    (14336, 287, ((1024, 1), (128, 4), (64, 8))),
])
def test_empirical_recall_matches_closed_form_over_1e4_trials(N, K, params):
    got = _empirical_recall(N, K, params, trials=10_000, seed=2506)
    for (B, Kp), r in got.items():
        want = oracle.expected_recall(N, B, K, Kp)
        assert abs(r - want) <= 0.005, (N, K, B, Kp, r, want)
