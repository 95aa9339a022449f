"""GPU parity of the mirrored problem (min-K: the K smallest, smallest first, ties toward the
lowest index) against the CPU oracle's own definition of it, bit for bit, on every route and
element type; and the symmetry that ties it to Top-K (min-K of x = Top-K of -x, or of ~x)."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2506_04165_amd import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def atk():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04165_amd import binding
    return binding


def raw(t):
    t = t.detach().cpu().contiguous()
    return (t.view(torch.int16).numpy().view(np.uint16) if t.element_size() == 2
            else t.view(torch.int32).numpy().view(np.uint32))


def oracle_raw(a):
    return a.view(np.uint16) if a.dtype.itemsize == 2 else a.view(np.uint32)


def check(atk, x, K, Kp, B, route=None):
    rows, N = x.shape
    if route is not None:
        st, text = atk.describe_plan(x.dtype, rows, N, K, Kp, B)
        assert st == atk.OK and text.startswith(route), text
    print(f"min-K: {x.dtype} rows={rows} N={N} K={K} K'={Kp} B={B} route={route}", flush=True)
    xh = workloads.to_numpy_bits(x)
    xd = x.view(torch.int32).to(DEV).view(torch.uint32) if x.dtype == torch.uint32 else x.to(DEV)
    gv, gi = atk.approx_topk(xd, K, Kp, B, smallest=True)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(xh, K, Kp, B, smallest=True)
    assert np.array_equal(gi.cpu().numpy(), oi), "approximate min-K indices differ"
    assert np.array_equal(raw(gv), oracle_raw(ov)), "approximate min-K values differ"
    ev, ei = atk.topk(xd, K, smallest=True)
    torch.cuda.synchronize()
    ov, oi = oracle.topk(xh, K, smallest=True)
    assert np.array_equal(ei.cpu().numpy(), oi) and np.array_equal(raw(ev), oracle_raw(ov)), "exact min-K differs"


def ints(rows, N, seed, lo=-50, hi=50, unsigned=False):
    x = np.random.default_rng(seed).integers(lo, hi, (rows, N)).astype(np.uint32).view(np.int32)
    t = torch.from_numpy(x)
    return t.view(torch.uint32) if unsigned else t


def test_min_k_on_the_benchmark_shapes_reduced(atk):
    for name, rows in [("c1_tiny", 4), ("c2_ffn", 40), ("c3_vocab", 3), ("c4_mips", 2), ("c5_adversarial", 6)]:
        w = workloads.WORKLOADS[name]
        x = workloads.make(name, seed=7, rows=rows)
        for B, Kp in w.params:
            check(atk, x, w.K, Kp, B)


@pytest.mark.parametrize("route", ["fused", "slab", "split", "unfused", "chunked", "exact"])
def test_min_k_on_every_route_and_element_type(atk, knobs, route):
    shape = {"fused": (37, 8192, 100, 4, 64), "slab": (8, 262144, 1024, 4, 1024), "split": (8, 262144, 1024, 4, 1024),
             "unfused": (4, 131072, 300, 16, 2048), "chunked": (4, 131072, 300, 16, 2048), "exact": (5, 8192, 40, 40, 8)}[route]
    if route == "split":
        knobs.set("slab", 0)
    if route == "chunked":
        knobs.set("chunked", 1)
    rows, N, K, Kp, B = shape
    check(atk, workloads.gaussian(rows, N, seed=1), K, Kp, B, route)
    check(atk, workloads.heavy_ties(rows, N, seed=2, symbols=3), K, Kp, B, route)
    if route == "split":      # half the bytes: rows of 16-bit elements are not split by themselves
        knobs.set("segments", 4)
    check(atk, workloads.gaussian(rows, N, seed=3, dtype=torch.bfloat16), K, Kp, B, route)
    check(atk, workloads.gaussian(rows, N, seed=4).to(torch.float16), K, Kp, B, route)
    if route == "split":
        knobs.set("segments", -1)
    check(atk, ints(rows, N, 5), K, Kp, B, route)
    check(atk, ints(rows, N, 6, -(1 << 31), 1 << 31, unsigned=True), K, Kp, B, route)


def test_min_k_list_representations_zeros_and_infinities(atk):
    # packed 16-bit keys, several rows per wavefront, sorted batches, lanes sharing buckets
    check(atk, workloads.gaussian(1030, 2048, seed=8, dtype=torch.bfloat16), 287, 4, 128)
    check(atk, workloads.gaussian(1030, 2048, seed=9, dtype=torch.bfloat16), 300, 8, 64)
    check(atk, workloads.gaussian(129, 65536, seed=10), 256, 32, 256)
    check(atk, workloads.gaussian(9, 8192, seed=11), 40, 6, 16)
    check(atk, ints(65, 6000, 12), 77, 3, 125)
    # zeros of both signs (equal in the order; stored bits returned), +inf rows (real +inf elements are
    # legitimate outputs), -inf (the smallest there is)
    x = torch.full((3, 4096), float("inf"))
    x[0, [7, 50, 4000]] = torch.tensor([1.0, -2.0, 3.0])
    x[1, 100] = float("-inf")
    x[2, :] = 1.0
    x[2, [10, 40, 77]] = -0.0
    x[2, [3, 50]] = 0.0
    for K, Kp, B in [(64, 2, 64), (64, 1, 64), (16, 16, 1), (300, 8, 64), (40, 4, 16)]:
        check(atk, x, K, Kp, B)
    check(atk, x.to(torch.bfloat16), 64, 2, 64)


def test_min_k_is_top_k_of_the_reversed_values(atk):
    x = workloads.gaussian(50, 16384, seed=13).to(DEV)
    v, i = atk.approx_topk(x, 128, 4, 1024, smallest=True)
    v2, i2 = atk.approx_topk(-x, 128, 4, 1024)
    torch.cuda.synchronize()
    assert torch.equal(i, i2) and torch.equal(v, -v2)
    y = ints(20, 16384, 14, -(1 << 31), 1 << 31).to(DEV)
    v, i = atk.topk(y, 500, smallest=True)
    v2, i2 = atk.topk(~y, 500)
    torch.cuda.synchronize()
    assert torch.equal(i, i2) and torch.equal(v, ~v2)


def test_min_k_for_a_recall_target(atk):
    # atk_approx_mink_recall: the library's (K', B) for the target, the K smallest; the same bits
    # as the oracle's mirrored problem at those parameters; the exact fallback as well
    for dtype, rows, N, K, target in [(torch.float32, 6, 65536, 256, 0.95), (torch.bfloat16, 9, 14336, 287, 0.99),
                                      (torch.int32, 4, 262144, 100, 0.9), (torch.float32, 5, 30000, 50, 0.9)]:
        x = ints(rows, N, seed=K) if dtype == torch.int32 else workloads.gaussian(rows, N, seed=K, dtype=dtype)
        v, i, kp, B = atk.approx_topk_recall(x.to(DEV), K, target, smallest=True)
        torch.cuda.synchronize()
        assert (kp, B) == atk.recall_params(dtype, rows, N, K, target)[:2]
        xh = workloads.to_numpy_bits(x)
        ov, oi = (oracle.topk(xh, K, smallest=True) if (kp, B) == (K, 1)
                  else oracle.approx_topk(xh, K, kp, B, smallest=True))
        assert np.array_equal(i.cpu().numpy(), oi), (dtype, N, K, kp, B)
        assert np.array_equal(raw(v), oracle_raw(ov)), (dtype, N, K, kp, B)
