"""Pins for the CPU oracle's result definition (Section 6.1, Steps 1-4).

The oracle is checked against things other than itself: a brute-force rank-count
formulation written here with plain loops, NumPy's stable argsort for the exact
Top-K, the K'=K and B=1 special cases (both must give the exact Top-K), the
collision identity of Section 6.2, and hand-made cases (the figure-caption example,
signed zeros, -inf rows, tie-dense rows, adversarial placement).
"""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2506_04165_amd import workloads


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def before(va, ia, vb, ib):
    """The total order: greater value first, equal values -> lower index first."""
    return va > vb or (va == vb and ia < ib)


def brute_force(row, K, Kp, B):
    """Second formulation, by counting ranks (no sorting anywhere).

    Element e survives stage 1 iff fewer than K' elements of its own bucket come
    before it; it is output iff fewer than K survivors come before it, and its
    output position is that count.
    """
    N = len(row)
    surv = []
    for n in range(N):
        c = 0
        for m in range(n % B, N, B):
            if m != n and before(row[m], m, row[n], n):
                c += 1
        if c < Kp:
            surv.append(n)
    out_idx = [None] * K
    for n in surv:
        c = sum(1 for m in surv if m != n and before(row[m], m, row[n], n))
        if c < K:
            assert out_idx[c] is None
            out_idx[c] = n
    return out_idx


def legal_params(N):
    for B in [b for b in range(1, N + 1) if N % b == 0]:
        for Kp in range(1, N // B + 1):
            for K in range(Kp, min(N, B * Kp) + 1):
                yield B, Kp, K


@pytest.mark.parametrize("N,symbols", [(12, 3), (24, 3), (30, 50)])
def test_matches_rank_count_brute_force_all_legal_params(N, symbols):
    rng = np.random.default_rng(100 + N)
    params = list(legal_params(N))
    if len(params) > 400:
        params = [params[i] for i in rng.choice(len(params), 400, replace=False)]
    for B, Kp, K in params:
        row = rng.integers(0, symbols, size=N).astype(np.float32) - 1.0
        vals, idx = oracle.approx_topk(row[None, :], K, Kp, B)
        want = brute_force(row, K, Kp, B)
        assert idx[0].tolist() == want, (N, B, Kp, K, row)
        assert np.array_equal(vals[0], row[want])


def test_exact_topk_matches_numpy_stable_argsort():
    rng = np.random.default_rng(7)
    for N, K, symbols in [(4096, 32, None), (1000, 1000, None), (512, 100, 5), (64, 1, 2)]:
        if symbols is None:
            x = rng.standard_normal((6, N)).astype(np.float32)
        else:
            x = rng.integers(0, symbols, size=(6, N)).astype(np.float32)
        vals, idx = oracle.topk(x, K)
        for r in range(x.shape[0]):
            want = np.argsort(-x[r], kind="stable")[:K]
            assert np.array_equal(idx[r], want)
            assert np.array_equal(vals[r], x[r][want])


@pytest.mark.parametrize("B", [1, 2, 64, 128, 4096 // 32])
def test_kprime_equals_k_is_exact(B):
    # 1 <= K' <= K (abstract); at K' = K every bucket keeps all it could contribute
    x = workloads.to_numpy_bits(workloads.make("c1_tiny", seed=3))
    K = 32
    av, ai = oracle.approx_topk(x, K, K, B)
    ev, ei = oracle.topk(x, K)
    assert np.array_equal(ai, ei) and np.array_equal(av, ev)


def test_single_bucket_is_exact_bf16():
    x = workloads.to_numpy_bits(workloads.gaussian(5, 2048, seed=11, dtype=torch.bfloat16))
    av, ai = oracle.approx_topk(x, 40, 40, 1)
    ev, ei = oracle.topk(x, 40)
    assert np.array_equal(ai, ei) and np.array_equal(av, ev)
    # bf16 ties: stable argsort of the widened values is the library cross-check
    w = oracle.bf16_bits_to_f32(x)
    for r in range(x.shape[0]):
        assert np.array_equal(ei[r], np.argsort(-w[r], kind="stable")[:40])


def check_invariants(x_f32, vals_f32, idx, K, Kp, B, exact_vals_f32):
    rows, N = x_f32.shape
    for r in range(rows):
        v, i = vals_f32[r], idx[r]
        assert np.all(v[:-1] >= v[1:])                       # non-increasing
        eq = v[:-1] == v[1:]
        assert np.all(i[:-1][eq] < i[1:][eq])                # ties: increasing index
        assert len(set(i.tolist())) == K and i.min() >= 0 and i.max() < N
        assert np.array_equal(x_f32[r][i], v)                # values are the elements at idx
        assert np.bincount(i % B, minlength=B).max() <= Kp   # at most K' per bucket
        assert np.all(v <= exact_vals_f32[r])                # never better than exact


@pytest.mark.parametrize("name,rows", [("c1_tiny", 4), ("c2_ffn", 3), ("c3_vocab", 2),
                                       ("c5_adversarial", 4)])
def test_structural_invariants_and_stage1_consistency(name, rows):
    w = workloads.WORKLOADS[name]
    x = workloads.to_numpy_bits(workloads.make(name, seed=5, rows=rows))
    xf = oracle.bf16_bits_to_f32(x) if x.dtype == np.uint16 else x
    ev, ei = oracle.topk(x, w.K)
    evf = oracle.bf16_bits_to_f32(ev) if ev.dtype == np.uint16 else ev
    for B, Kp in w.params:
        av, ai = oracle.approx_topk(x, w.K, Kp, B)
        avf = oracle.bf16_bits_to_f32(av) if av.dtype == np.uint16 else av
        check_invariants(xf, avf, ai, w.K, Kp, B, evf)
        # stage 1 alone: plane k of bucket b is that bucket's k-th greatest (library check)
        sv, si = oracle.stage1(x, Kp, B)
        for r in range(rows):
            for b in list(range(min(B, 3))) + [B - 1]:
                members = np.arange(b, w.N, B)
                order = members[np.argsort(-xf[r][members], kind="stable")[:Kp]]
                assert np.array_equal(si[r, :, b], order)
            # approx ∩ exact = the exact Top-K elements whose rank inside their bucket is < K'
            keep = set(si[r].ravel().tolist())
            want = [n for n in ei[r].tolist() if n in keep]
            got = [n for n in ai[r].tolist() if n in set(ei[r].tolist())]
            assert got == want


def test_recall_equals_collision_identity_for_distinct_values():
    # Section 6.2: recall = 1 - sum_b max(0, X_b - K') / K, exactly, when values are distinct
    rng = np.random.default_rng(21)
    N, K = 4096, 64
    x = np.stack([rng.permutation(N).astype(np.float32) for _ in range(16)])
    _, ei = oracle.topk(x, K)
    for B, Kp in [(64, 1), (64, 2), (128, 1), (16, 4), (256, 1)]:
        _, ai = oracle.approx_topk(x, K, Kp, B)
        got = oracle.index_recall(ai, ei)
        for r in range(x.shape[0]):
            xb = np.bincount(ei[r] % B, minlength=B)
            want = 1.0 - np.maximum(xb - Kp, 0).sum() / K
            assert got[r] == pytest.approx(want, abs=1e-12)


def test_figure_caption_example_two_of_three_collide():
    # Appendix figure of the original algorithm: 20 elements, 4 buckets (stride 4), K=3, K'=1;
    # two of the three greatest share a bucket, so one is lost: recall 2/3.  The caption prints
    # no values; these are made up to realise it.
    row = np.arange(20, dtype=np.float32) * 0.01
    row[5], row[13], row[2] = 9.0, 8.0, 7.0          # 5 and 13 are both in bucket 1
    row[7] = 3.0                                      # best of the rest, bucket 3
    _, ei = oracle.topk(row[None], 3)
    _, ai = oracle.approx_topk(row[None], 3, 1, 4)
    assert ei[0].tolist() == [5, 13, 2]
    assert ai[0].tolist() == [5, 2, 7]
    assert oracle.index_recall(ai, ei)[0] == pytest.approx(2 / 3)
    # with K'=2 the collision is absorbed
    _, ai2 = oracle.approx_topk(row[None], 3, 2, 4)
    assert ai2[0].tolist() == [5, 13, 2]


def test_strided_not_contiguous_buckets():
    # top-K in one contiguous index range (K <= B) is the benign case for stride-B buckets
    N, B, K = 1024, 64, 32
    row = np.zeros(N, dtype=np.float32)
    row[100:100 + K] = np.arange(K, 0, -1)
    _, ai = oracle.approx_topk(row[None], K, 1, B)
    assert ai[0].tolist() == list(range(100, 100 + K))
    # the same values in one stride-B class lose all but K' of them
    row2 = np.zeros(N, dtype=np.float32)
    pos = 5 + B * np.arange(N // B)
    row2[pos] = np.arange(N // B, 0, -1)
    _, ai2 = oracle.approx_topk(row2[None], K, 2, B)
    assert ai2[0][:2].tolist() == [5, 5 + B]
    assert set(ai2[0][2:].tolist()).isdisjoint(pos.tolist())


def test_signed_zero_and_minus_inf():
    # -0.0 == +0.0: the index decides, and the output carries the stored bits
    row = np.full(64, -1.0, dtype=np.float32)
    row[10] = -0.0
    row[3] = 0.0
    row[40] = -0.0
    vals, idx = oracle.topk(row[None], 3)
    assert idx[0].tolist() == [3, 10, 40]
    assert vals.view(np.uint32)[0].tolist() == [0x00000000, 0x80000000, 0x80000000]
    # a row that is mostly -inf: real -inf elements are legitimate outputs, lowest index first
    row = np.full(64, -np.inf, dtype=np.float32)
    row[[7, 50]] = [1.0, 2.0]
    vals, idx = oracle.approx_topk(row[None], 6, 2, 8)
    # bucket 2 keeps (50, 2), bucket 7 keeps (7, 15), every other bucket b keeps (b, b+8)
    assert idx[0].tolist() == [50, 7, 0, 1, 2, 3]
    assert np.isneginf(vals[0][2:]).all()
    # bf16 signed zeros
    rb = f32_to_bf16_bits(np.array([[-1, -0.0, 0.0, -2, 0.0, -0.0, -3, -4]], dtype=np.float32))
    vals, idx = oracle.approx_topk(rb, 4, 2, 2)
    assert idx[0].tolist() == [1, 2, 4, 5]
    assert vals[0].tolist() == [0x8000, 0x0000, 0x0000, 0x8000]


def test_nan_is_rejected():
    row = np.zeros((1, 16), dtype=np.float32)
    row[0, 5] = np.nan
    with pytest.raises(ValueError):
        oracle.topk(row, 2)
    with pytest.raises(ValueError):
        oracle.approx_topk(row, 2, 1, 4)


@pytest.mark.parametrize("bad", [dict(K=4, Kp=5, B=4), dict(K=9, Kp=2, B=4), dict(K=2, Kp=1, B=5),
                                 dict(K=4, Kp=0, B=4), dict(K=17, Kp=17, B=1),
                                 dict(K=8, Kp=5, B=4)])
def test_illegal_parameters_are_rejected(bad):
    row = np.zeros((1, 16), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.approx_topk(row, bad["K"], bad["Kp"], bad["B"])


def test_adversarial_placement_closed_form():
    # top-K spread evenly over c stride-B classes: recall = c * min(K', K/c) / K exactly
    w = workloads.WORKLOADS["c5_adversarial"]
    x = workloads.adversarial_sorted(3, w.N, seed=9, K=w.K, B=256).numpy()
    _, ei = oracle.topk(x, w.K)
    for Kp, want in [(1, 1 / 64), (8, 1 / 8), (32, 1 / 2)]:
        _, ai = oracle.approx_topk(x, w.K, Kp, 256)
        assert np.allclose(oracle.index_recall(ai, ei), want)


def test_heavy_tie_rows():
    # 16 distinct values: the greatest symbol occurs far more than K times, so the exact result
    # is its K lowest positions and the approximate one its lowest K among stage-1 survivors
    w = workloads.WORKLOADS["c5_adversarial"]
    x = workloads.heavy_ties(2, w.N, seed=4).numpy()
    ev, ei = oracle.topk(x, w.K)
    for r in range(2):
        top = x[r].max()
        assert np.array_equal(ei[r], np.flatnonzero(x[r] == top)[:w.K])
    for Kp in (1, 8, 32):
        av, ai = oracle.approx_topk(x, w.K, Kp, 256)
        assert np.all(oracle.value_recall(av, ev) == 1.0)
        for r in range(2):
            top = x[r].max()
            holders = np.flatnonzero(x[r] == top)
            # survivors holding `top`: the first K' holders of each bucket
            surv = sorted(n for b in range(256) for n in holders[holders % 256 == b][:Kp].tolist())
            if len(surv) >= w.K:
                assert ai[r].tolist() == surv[:w.K]


def test_c4_scores_shape_and_scale():
    x = workloads.make("c4_mips", seed=2, rows=2)
    assert x.shape == (2, 1048576) and x.dtype == torch.float32
    assert abs(float(x.std()) - 128 ** -0.5) < 0.01
