"""GPU parity of the matmul-fused entry point (Section 7.3) against the oracle.

Integer-valued vectors make every inner product exact in any format and order, so the two
sides must agree bit for bit (and such scores tie heavily, which exercises the index rule).
For Gaussian vectors the scores of the two sides differ by the rounding of a binary32
accumulation; there the comparison is: reported scores within the bound of the oracle's, and
every difference in the chosen sets explained by a score within that bound of a decision
threshold (a bucket's K'-th place or the K-th place overall)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2506_04165_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def atk():
    from paper_2506_04165_amd import binding
    return binding


def run_both(atk, Q, N, D, K, Kp, B, seed, kind, dtype=torch.bfloat16):
    q, d = workloads.mips_vectors(Q, N, seed=seed, dim=D, kind=kind, dtype=dtype)
    print(f"mips case Q={Q} N={N} D={D} K={K} K'={Kp} B={B} kind={kind} seed={seed}", flush=True)
    gv, gi = atk.mips_approx_topk(q.to(DEV), d.to(DEV), K, Kp, B)
    torch.cuda.synchronize()
    return q, d, gv.cpu().numpy(), gi.cpu().numpy()


@pytest.mark.parametrize("Q,N,D,K,Kp,B", [
    (128, 8192, 128, 64, 1, 64),        # one slab pair, K'=1
    (100, 8192, 128, 100, 2, 64),       # ragged query tile
    (130, 16384, 128, 128, 4, 128),     # two query tiles, the second nearly empty
    (33, 32768, 64, 96, 3, 32),         # K'=3 runs in lists of 4; one slab; D=64
    (64, 65536, 256, 256, 4, 256),      # D=256
    (8, 131072, 128, 300, 4, 128),      # few pairs: the walk is cut into segments
    (16, 4096, 128, 128, 4, 32),        # K = B*K': stage 2 is a pure sort
    (1, 2048, 64, 32, 1, 32),           # single query
    (5, 128, 64, 100, 4, 32),           # every bucket holds exactly K' vectors: all survive
    (3, 64, 64, 64, 1, 64),             # one vector per bucket, K = N: a sort of all scores
    (7, 4096, 128, 4, 4, 32),           # K' = K
])
def test_integer_vectors_bit_exact(atk, Q, N, D, K, Kp, B):
    q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=11, kind="integer")
    ov, oi = oracle.mips_approx_topk(workloads.to_numpy_bits(q), workloads.to_numpy_bits(d), K, Kp, B)
    assert (gi == oi).all()
    assert (gv.view(np.uint32) == ov.view(np.uint32)).all()


@pytest.mark.parametrize("Q,N,D,K,Kp,B", [(100, 8192, 128, 100, 2, 64), (33, 32768, 64, 96, 3, 32),
                                        (64, 65536, 256, 256, 4, 256), (130, 16384, 128, 128, 1, 128)])
def test_fp16_vectors(atk, Q, N, D, K, Kp, B):
    q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=21, kind="integer", dtype=torch.float16)
    ov, oi = oracle.mips_approx_topk(q.numpy(), d.numpy(), K, Kp, B)
    assert (gi == oi).all() and (gv.view(np.uint32) == ov.view(np.uint32)).all()
    q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=22, kind="unit", dtype=torch.float16)
    scores = oracle.mips_scores(q.numpy(), d.numpy())
    ov, oi = oracle.mips_approx_topk(q.numpy(), d.numpy(), K, Kp, B)
    tol = (D + 1) * 2.0 ** -24
    moved = sum(explain_differences(scores[r], gv[r], gi[r], ov[r], oi[r], K, Kp, B, tol) for r in range(Q))
    assert moved <= 0.01 * Q * K, moved


def test_segments_are_used_when_pairs_are_few(atk):
    st, text = atk.mips_describe_plan(8, 131072, 128, 300, 4, 128)
    assert st == 0 and "segments=16" in text, text
    st, text = atk.mips_describe_plan(1024, 1 << 20, 128, 1024, 4, 1024)
    assert st == 0 and "segments=2" in text and "grid=512" in text, text


def explain_differences(scores, gv, gi, ov, oi, K, Kp, B, tol):
    """Asserts the tolerance-aware validity of one row; returns how many places differ."""
    N = scores.shape[0]
    assert len(set(gi.tolist())) == K and gi.min() >= 0 and gi.max() < N
    assert np.bincount(gi % B, minlength=B).max() <= Kp
    assert np.abs(gv.astype(np.float64) - scores[gi].astype(np.float64)).max() <= tol
    assert (gv[:-1] > gv[1:]).all() or all(
        gv[j] > gv[j + 1] or (gv[j] == gv[j + 1] and gi[j] < gi[j + 1]) for j in range(K - 1))
    diff = set(gi.tolist()) ^ set(oi.tolist())
    if diff:
        kth = float(ov[-1])
        per_bucket = scores.reshape(N // B, B)
        for n in diff:
            col = np.sort(per_bucket[:, n % B])[::-1]
            near_bucket_edge = abs(float(scores[n]) - float(col[Kp - 1])) <= 2 * tol or (
                Kp < len(col) and abs(float(scores[n]) - float(col[Kp])) <= 2 * tol)
            near_k_edge = abs(float(scores[n]) - kth) <= 2 * tol
            assert near_bucket_edge or near_k_edge, (n, float(scores[n]), kth)
    return int((gi != oi).sum())


@pytest.mark.parametrize("Q,N,D,K,Kp,B", [
    (96, 65536, 128, 128, 4, 128),
    (160, 65536, 128, 256, 1, 1024),
    (40, 32768, 64, 64, 2, 256),
])
def test_gaussian_vectors_within_rounding(atk, Q, N, D, K, Kp, B):
    q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=12, kind="unit")
    qb, db = workloads.to_numpy_bits(q), workloads.to_numpy_bits(d)
    scores = oracle.mips_scores(qb, db)
    ov, oi = oracle.mips_approx_topk(qb, db, K, Kp, B)
    # binary32 accumulation of D products of unit-length vectors: |error| <= D * 2^-24 * sum|q_d x_d|
    # <= D * 2^-24 (Cauchy-Schwarz), plus the oracle's own final rounding (half an ulp of <= 1)
    tol = (D + 1) * 2.0 ** -24
    moved = sum(explain_differences(scores[r], gv[r], gi[r], ov[r], oi[r], K, Kp, B, tol) for r in range(Q))
    assert moved <= 0.01 * Q * K, moved
    # scores themselves: most are the correctly rounded value, all are within the bound
    assert (gv == np.take_along_axis(scores, gi.astype(np.int64), axis=1)).mean() > 0.5


def test_full_size_sampled_queries(atk):
    # the benchmark's shape (Section 7.3: 1024 queries, one million 128-d vectors, K=1024),
    # launch configuration as timed; the oracle checks a sample of the queries one by one
    Q, N, D, K, Kp, B = 1024, 1 << 20, 128, 1024, 4, 1024
    q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=13, kind="unit")
    qb, db = workloads.to_numpy_bits(q), workloads.to_numpy_bits(d)
    tol = (D + 1) * 2.0 ** -24
    for r in (0, 127, 128, 500, 1023):
        scores = oracle.mips_scores(qb[r:r + 1], db)[0]
        ov, oi = oracle.approx_topk(scores[None, :], K, Kp, B)
        explain_differences(scores, gv[r], gi[r], ov[0], oi[0], K, Kp, B, tol)
    # properties that hold at any size, all queries
    assert (np.diff(gv, axis=1) <= 0).all()
    assert (np.sort(gi, axis=1)[:, 1:] != np.sort(gi, axis=1)[:, :-1]).all()
    counts = np.stack([np.bincount(row % B, minlength=B) for row in gi[:64]])
    assert counts.max() <= Kp


def test_full_size_integer_sampled_bit_exact(atk):
    Q, N, D, K, Kp, B = 1024, 1 << 20, 128, 1024, 4, 1024
    q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=14, kind="integer")
    qb, db = workloads.to_numpy_bits(q), workloads.to_numpy_bits(d)
    for r in (3, 640, 1023):
        ov, oi = oracle.mips_approx_topk(qb[r:r + 1], db, K, Kp, B)
        assert (gi[r] == oi[0]).all() and (gv[r] == ov[0]).all()


def test_seeded_random_shapes_integer_vectors(atk):
    # shapes the list above does not name: any B that is a multiple of 32, every K', every
    # supported D and both vector types, ragged query tiles, short and long walks
    rng = np.random.default_rng(77)
    for case in range(24):
        D = int(rng.choice([64, 128, 256]))
        B = 32 * int(rng.integers(1, 40))
        steps = int(rng.integers(1, max(1, min(400, 200000 // B)) + 1))
        N = B * steps
        Kp = int(rng.integers(1, min(4, steps) + 1))
        K = int(rng.integers(Kp, min(B * Kp, N, 2048) + 1))
        Q = int(rng.integers(1, 300))
        dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float16
        q, d, gv, gi = run_both(atk, Q, N, D, K, Kp, B, seed=1000 + case, kind="integer", dtype=dtype)
        qh = workloads.to_numpy_bits(q) if dtype == torch.bfloat16 else q.numpy()
        dh = workloads.to_numpy_bits(d) if dtype == torch.bfloat16 else d.numpy()
        ov, oi = oracle.mips_approx_topk(qh, dh, K, Kp, B)
        assert (gi == oi).all() and (gv.view(np.uint32) == ov.view(np.uint32)).all(), case


def test_recall_front_end(atk):
    q, d = workloads.mips_vectors(40, 65536, seed=31, dim=128, kind="integer")
    gv, gi, kp, b = atk.mips_approx_topk_recall(q.to(DEV), d.to(DEV), 256, 0.97)
    torch.cuda.synchronize()
    assert (kp, b) == oracle.mips_select_parameters(65536, 256, 0.97)
    ov, oi = oracle.mips_approx_topk(workloads.to_numpy_bits(q), workloads.to_numpy_bits(d), 256, kp, b)
    assert (gi.cpu().numpy() == oi).all() and (gv.cpu().numpy() == ov).all()


def test_errors(atk):
    q, d = workloads.mips_vectors(4, 4096, seed=1, dim=128)
    q, d = q.to(DEV), d.to(DEV)
    with pytest.raises(atk.AtkError):
        atk.mips_approx_topk(q, d, 64, 1, 48)            # B not a multiple of 32
    with pytest.raises(atk.AtkError):
        atk.mips_approx_topk(q, d, 64, 8, 64)            # K' beyond the fused lists
    with pytest.raises(ValueError):
        atk.mips_approx_topk(q.cpu(), d, 64, 1, 64)
    with pytest.raises(ValueError):
        atk.mips_approx_topk(q, d[:, :64], 64, 1, 64)
