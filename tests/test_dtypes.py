"""fp16, int32 and uint32 inputs (the compute-type promotion of Section 6.3's listing).

CPU part: the oracle's handling of the new element types is pinned against NumPy's own
conversions and sorts.  GPU part: the HIP path against the oracle, bit for bit, over every
launch route (fused, shared buckets, slab, split, chunked, unfused, exact, batched lists, stage 1 only)."""
import numpy as np
import pytest
import torch

from oracle import oracle

DEV = "cuda:0"
I32_MIN, I32_MAX = -2 ** 31, 2 ** 31 - 1


# ---------------------------------------------------------------------------------------------
# seeded inputs
# ---------------------------------------------------------------------------------------------
def int_rows(rows, N, seed, kind, unsigned=False):
    rng = np.random.default_rng(seed)
    if kind == "full":          # the whole 32-bit range, extremes planted
        x = rng.integers(0, 2 ** 32, (rows, N), dtype=np.uint64).astype(np.uint32)
        for r in range(rows):
            pos = rng.choice(N, 6, replace=False)
            x[r, pos[:2]] = 0
            x[r, pos[2:4]] = 0xFFFFFFFF
            x[r, pos[4]] = 0x80000000
            x[r, pos[5]] = 0x7FFFFFFF
    elif kind == "ties":        # few distinct values around the sign change
        x = rng.integers(-3, 4, (rows, N)).astype(np.int32).view(np.uint32)
    elif kind == "floor":       # nearly everything is the least value: it must fill the lists
        x = np.full((rows, N), 0x80000000 if not unsigned else 0, dtype=np.uint32)
        for r in range(rows):
            pos = rng.choice(N, 5, replace=False)
            x[r, pos] = x[r, pos] + rng.integers(1, 100, 5).astype(np.uint32)
    else:
        raise ValueError(kind)
    return x if unsigned else x.view(np.int32)


def half_rows(rows, N, seed, kind):
    rng = np.random.default_rng(seed)
    if kind == "patterns":      # uniform over the non-NaN bit patterns: subnormals, infinities, zeros
        mag = rng.integers(0, 0x7C01, (rows, N)).astype(np.uint16)
        sign = (rng.integers(0, 2, (rows, N)) << 15).astype(np.uint16)
        return (mag | sign).view(np.float16)
    return rng.standard_normal((rows, N)).astype(np.float16)


# ---------------------------------------------------------------------------------------------
# oracle pins (CPU)
# ---------------------------------------------------------------------------------------------
def test_oracle_half_widening_matches_numpy_on_every_pattern():
    pats = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    pats = pats[(pats & 0x7FFF) <= 0x7C00]                       # NaN excluded
    x = pats.view(np.float16)[None, :]
    v, i = oracle.topk(x, x.shape[1])
    ref = np.argsort(-x[0].astype(np.float32), kind="stable")    # NumPy's conversion and sort
    assert (i[0] == ref).all()
    assert (v[0].view(np.uint16) == pats[ref]).all()


@pytest.mark.parametrize("unsigned", [False, True])
@pytest.mark.parametrize("kind", ["full", "ties", "floor"])
def test_oracle_integer_topk_matches_numpy(kind, unsigned):
    x = int_rows(3, 4096, seed=21, kind=kind, unsigned=unsigned)
    v, i = oracle.topk(x, 100)
    for r in range(3):
        ref = np.argsort(-x[r].astype(np.int64), kind="stable")[:100]
        assert (i[r] == ref).all() and (v[r] == x[r][ref]).all()


def test_oracle_integer_approx_agrees_with_its_float_path_on_small_values():
    # values below 2^24 are exact in float32: the two element types must select the same elements
    rng = np.random.default_rng(22)
    x = rng.integers(-1000, 1000, (4, 2048)).astype(np.int32)
    for K, Kp, B in [(32, 1, 64), (48, 3, 16), (17, 17, 1)]:
        vi, ii = oracle.approx_topk(x, K, Kp, B)
        vf, jf = oracle.approx_topk(x.astype(np.float32), K, Kp, B)
        assert (ii == jf).all() and (vi == vf.astype(np.int32)).all()


def test_oracle_extremes_order():
    x = np.array([[0, -1, I32_MIN, I32_MAX, I32_MIN, 5]], dtype=np.int32)
    v, i = oracle.topk(x, 6)
    assert list(i[0]) == [3, 5, 0, 1, 2, 4]
    v, i = oracle.topk(x.view(np.uint32), 6)                     # same words, unsigned order
    assert list(i[0]) == [1, 2, 4, 3, 5, 0]


# ---------------------------------------------------------------------------------------------
# GPU parity
# ---------------------------------------------------------------------------------------------
@pytest.fixture(scope="module")
def atk():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04165_amd import binding
    return binding


def to_device(x: np.ndarray) -> torch.Tensor:
    if x.dtype == np.uint32:
        return torch.from_numpy(x.view(np.int32)).to(DEV).view(torch.uint32)
    return torch.from_numpy(x).to(DEV)


def words(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    return t.view(torch.int16).numpy() if t.element_size() == 2 else t.view(torch.int32).numpy()


def host_words(x: np.ndarray) -> np.ndarray:
    return x.view(np.int16) if x.dtype.itemsize == 2 else x.view(np.int32)


def check(atk, x, K, Kp, B, route=None):
    print(f"dtype case {x.dtype} {x.shape} K={K} K'={Kp} B={B}", flush=True)
    xd = to_device(x)
    if route is not None:
        st, plan = atk.describe_plan(xd.dtype, x.shape[0], x.shape[1], K, Kp, B)
        assert st == 0 and plan.startswith(route), plan
    gv, gi = atk.approx_topk(xd, K, Kp, B)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(x, K, Kp, B)
    assert np.array_equal(gi.cpu().numpy(), oi)
    assert np.array_equal(words(gv), host_words(ov))


ROUTES = [
    # rows, N, K, K', B, route
    (37, 4096, 32, 4, 64, "fused"),
    (16, 14336, 287, 4, 128, "fused"),
    (16, 14336, 287, 1, 1024, "fused"),
    (9, 8192, 40, 6, 16, "fused"),             # several lanes share a bucket
    (5, 4100, 10, 3, 4, "fused"),              # B = 4, N not a multiple of anything large
    (3, 3600, 64, 3, 900, "fused"),            # B not a power of two
    (8, 262144, 1024, 4, 1024, "slab"),
    (8, 262144, 1024, 4, 1024, "split"),
    (4, 131072, 128, 16, 2048, "chunked"),     # survivors beyond LDS: every chunk's K greatest through memory
    (4, 131072, 128, 16, 2048, "unfused"),     # ... or all survivors
    (6, 65536, 256, 32, 256, "fused"),        # long lists: sorted batches (16-bit rows: packed lists, few-row route)
    (5, 8192, 40, 40, 8, "exact"),             # K' = K beyond the register lists
]


@pytest.mark.gpu
@pytest.mark.parametrize("rows,N,K,Kp,B,route", ROUTES)
@pytest.mark.parametrize("unsigned", [False, True])
def test_integer_rows_every_route(atk, rows, N, K, Kp, B, route, unsigned, knobs):
    if route == "split":     # the default for so few rows is the slab route
        knobs.set("slab", 0)
    if route == "chunked":
        knobs.set("chunked", 1)
    for kind in ("full", "ties", "floor"):
        check(atk, int_rows(rows, N, seed=31, kind=kind, unsigned=unsigned), K, Kp, B, route)


@pytest.mark.gpu
@pytest.mark.parametrize("rows,N,K,Kp,B,route", ROUTES)
def test_half_rows_every_route(atk, rows, N, K, Kp, B, route, knobs):
    if route == "split":     # rows this short are not split by themselves: ask for it
        knobs.set("slab", 0)
        knobs.set("segments", 4)
    if route == "chunked":
        knobs.set("chunked", 1)
    if (Kp, B) == (32, 256):
        # 16-bit rows keep packed keys in long lists as well (instead of sorted batches), which
        # opens the few-row route to them; the sorted batches with the packed keys switched off
        for kind in ("patterns", "gauss"):
            check(atk, half_rows(rows, N, seed=32, kind=kind), K, Kp, B, "slab lists32")
        knobs.set("packed", 0)
        route = "fused batched"
    for kind in ("patterns", "gauss"):
        check(atk, half_rows(rows, N, seed=32, kind=kind), K, Kp, B, route)


@pytest.mark.gpu
@pytest.mark.parametrize("make", [lambda: int_rows(7, 50000, 33, "full"),
                                  lambda: int_rows(7, 50000, 33, "ties", unsigned=True),
                                  lambda: half_rows(7, 50000, 33, "patterns")])
def test_exact_topk_and_stage1(atk, make):
    x = make()
    xd = to_device(x)
    for K in (1, 77, 2048):
        gv, gi = atk.topk(xd, K)
        torch.cuda.synchronize()
        ov, oi = oracle.topk(x, K)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(words(gv), host_words(ov))
    sv, si = atk.approx_topk_stage1(xd, 3, 400)
    torch.cuda.synchronize()
    ov, oi = oracle.stage1(x, 3, 400)
    assert np.array_equal(si.cpu().numpy(), oi) and np.array_equal(words(sv), host_words(ov))


@pytest.mark.gpu
def test_unaligned_integer_rows(atk):
    # odd row stride and an offset base: single-element loads
    base = int_rows(6, 4099, 34, "full")
    xd = to_device(base)[:, 3:]                                  # 4096 columns, stride 4099
    x = np.ascontiguousarray(base[:, 3:])
    gv, gi = atk.approx_topk(xd, 64, 2, 128)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(x, 64, 2, 128)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(words(gv), host_words(ov))


@pytest.mark.gpu
def test_recall_front_end_accepts_the_new_types(atk):
    x = int_rows(4, 65536, 35, "full")
    gv, gi, kp, b = atk.approx_topk_recall(to_device(x), 128, 0.95)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(x, 128, kp, b)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gv.cpu().numpy(), ov)
