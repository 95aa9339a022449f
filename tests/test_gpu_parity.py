"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, bit for bit.

Bar: integer/index work and fp compare-and-select only, so every output must be identical:
same int32 indices, same stored value bits, same order (ties toward the lowest index).
"""
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


def bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.view(torch.int32).numpy().view(np.uint32)


def host_bits(x: np.ndarray) -> np.ndarray:
    return x if x.dtype == np.uint16 else x.view(np.uint32)


def check_approx(atk, x: torch.Tensor, K, Kp, B, rows_to_check=None):
    """x: host tensor.  Runs the HIP path on all rows, the oracle on `rows_to_check` (all if None)."""
    xd = x.to(DEV)
    gv, gi = atk.approx_topk(xd, K, Kp, B)
    torch.cuda.synchronize()
    sel = np.arange(x.shape[0]) if rows_to_check is None else np.asarray(rows_to_check)
    xh = workloads.to_numpy_bits(x)[sel]
    ov, oi = oracle.approx_topk(xh, K, Kp, B)
    gi_h = gi.cpu().numpy()[sel]
    gv_h = bits(gv)[sel]
    assert np.array_equal(gi_h, oi), f"indices differ (K={K}, K'={Kp}, B={B})"
    assert np.array_equal(gv_h, host_bits(ov)), f"values differ (K={K}, K'={Kp}, B={B})"
    return gv, gi


def check_exact(atk, x: torch.Tensor, K, rows_to_check=None):
    xd = x.to(DEV)
    gv, gi = atk.topk(xd, K)
    torch.cuda.synchronize()
    sel = np.arange(x.shape[0]) if rows_to_check is None else np.asarray(rows_to_check)
    ov, oi = oracle.topk(workloads.to_numpy_bits(x)[sel], K)
    assert np.array_equal(gi.cpu().numpy()[sel], oi), f"exact indices differ (K={K})"
    assert np.array_equal(bits(gv)[sel], host_bits(ov)), f"exact values differ (K={K})"
    return gv, gi


def check_stage1(atk, x: torch.Tensor, Kp, B):
    sv, si = atk.approx_topk_stage1(x.to(DEV), Kp, B)
    torch.cuda.synchronize()
    ov, oi = oracle.stage1(workloads.to_numpy_bits(x), Kp, B)
    assert np.array_equal(si.cpu().numpy(), oi), f"stage-1 indices differ (K'={Kp}, B={B})"
    assert np.array_equal(bits(sv), host_bits(ov)), f"stage-1 values differ (K'={Kp}, B={B})"


# ---------------------------------------------------------------------------------------
# the five workloads at sizes the oracle finishes in seconds (several tiles + ragged tails)
# ---------------------------------------------------------------------------------------

def test_c1_tiny_all_params(atk):
    w = workloads.WORKLOADS["c1_tiny"]
    x = workloads.make("c1_tiny", seed=1)
    ev, ei = check_exact(atk, x, w.K)
    for B, Kp in w.params:
        gv, gi = check_approx(atk, x, w.K, Kp, B)
        check_stage1(atk, x, Kp, B)
        if Kp == w.K:   # K' = K and B = 1 must both give the exact Top-K
            assert torch.equal(gi, ei) and torch.equal(gv, ev)


@pytest.mark.parametrize("rows", [1, 37])
def test_c2_ffn_reduced_rows(atk, rows):
    w = workloads.WORKLOADS["c2_ffn"]
    x = workloads.make("c2_ffn", seed=2, rows=rows)
    for B, Kp in w.params:
        check_approx(atk, x, w.K, Kp, B)
    check_stage1(atk, x, 4, 128)
    check_exact(atk, x, w.K)


def test_c3_vocab_reduced_rows(atk):
    w = workloads.WORKLOADS["c3_vocab"]
    x = workloads.make("c3_vocab", seed=3, rows=5)
    for B, Kp in w.params:
        check_approx(atk, x, w.K, Kp, B)
    check_exact(atk, x, w.K)


def test_c4_mips_reduced_rows(atk):
    w = workloads.WORKLOADS["c4_mips"]
    x = workloads.make("c4_mips", seed=4, rows=3)
    for B, Kp in w.params:
        check_approx(atk, x, w.K, Kp, B)
    check_stage1(atk, x, 1, 4096)
    check_exact(atk, x, w.K)


def test_c5_adversarial_reduced_rows(atk):
    w = workloads.WORKLOADS["c5_adversarial"]
    x = workloads.make("c5_adversarial", seed=5, rows=6)   # 3 sorted-adversarial + 3 heavy-tie rows
    for B, Kp in w.params:
        check_approx(atk, x, w.K, Kp, B)
    check_stage1(atk, x, 8, 256)
    check_exact(atk, x, w.K)


# ---------------------------------------------------------------------------------------
# edge cases of the method and of the launch geometry
# ---------------------------------------------------------------------------------------

@pytest.mark.parametrize("B,Kp,K", [
    (1, 16, 16), (2, 8, 16), (4, 3, 12), (8, 2, 9), (16, 1, 16), (32, 4, 100),   # several lanes per bucket
    (64, 1, 64), (64, 5, 200), (64, 7, 33), (128, 12, 500), (256, 20, 1000),     # list length > K'
    (512, 2, 1024), (2048, 1, 77), (4096, 2, 2), (8192, 1, 2048),                # many buckets
])
def test_parameter_sweep_fp32(atk, B, Kp, K):
    x = workloads.gaussian(5, 16384, seed=100 + B + Kp)
    check_approx(atk, x, K, Kp, B)
    check_stage1(atk, x, Kp, B)


@pytest.mark.parametrize("B,Kp,K", [(1, 8, 8), (8, 4, 20), (64, 8, 287), (128, 4, 287),
                                    (256, 3, 700), (1024, 1, 287), (2048, 2, 64), (7168, 1, 287)])
def test_parameter_sweep_bf16(atk, B, Kp, K):
    x = workloads.gaussian(9, 14336, seed=200 + B + Kp, dtype=torch.bfloat16)
    check_approx(atk, x, K, Kp, B)
    check_stage1(atk, x, Kp, B)


@pytest.mark.parametrize("N,B,Kp,K", [(1344, 448, 2, 600), (900, 3, 30, 40), (900, 100, 9, 900),
                                      (210, 7, 30, 210), (1000, 125, 1, 100), (96, 96, 1, 50),
                                      (6, 3, 2, 5), (1, 1, 1, 1), (64, 64, 1, 64)])
def test_bucket_counts_that_are_not_powers_of_two_and_tiny_rows(atk, N, B, Kp, K):
    x = workloads.gaussian(3, N, seed=300 + N + B)
    check_approx(atk, x, K, Kp, B)
    check_stage1(atk, x, Kp, B)
    xb = workloads.gaussian(3, N, seed=301 + N + B, dtype=torch.bfloat16)
    check_approx(atk, xb, K, Kp, B)


@pytest.mark.parametrize("N,B,Kp,K", [(65536, 256, 4, 300), (65536, 1024, 1, 1000), (65536, 64, 16, 1024),
                                      (65536, 512, 2, 512), (131072, 256, 4, 300), (32768, 128, 6, 700),
                                      (1 << 21, 64, 8, 300), (1 << 23, 128, 3, 200), (1 << 23, 64, 4, 100)])
def test_bf16_packed_key_limits(atk, N, B, Kp, K):
    # rows of up to 65536 bf16 elements run on packed 32-bit keys (positions 0..65535 must all
    # be representable); longer rows keep packed keys of value and step in their lists and build
    # the general keys from them (lists of up to 8 entries, up to 65535 steps: the very last step
    # must be representable too), beyond that the general lists; ties are dense in bf16
    st, text = atk.describe_plan(torch.bfloat16, 5, N, K, Kp, B)
    assert st == atk.OK and (" packed" in text) == (N <= 65536), text
    assert (" lists32" in text) == (N > 65536 and Kp <= 8 and N // B <= 65535), text
    x = workloads.gaussian(5, N, seed=500 + B + Kp, dtype=torch.bfloat16)
    x[0, N - 1] = 100.0        # the very last position must be able to win
    x[1, :] = 1.5              # one value everywhere: the index alone decides
    check_approx(atk, x, K, Kp, B)
    z = workloads.heavy_ties(3, N, seed=501, symbols=5).to(torch.bfloat16)
    check_approx(atk, z, K, Kp, B)


@pytest.mark.parametrize("B,Kp,K", [(128, 4, 287), (64, 8, 300), (256, 2, 100), (64, 3, 64), (512, 2, 1000)])
def test_many_short_bf16_rows_several_rows_per_wavefront(atk, B, Kp, K):
    # >= 1024 short bf16 rows: groups of fewer than 64 lanes own a row, a wavefront holds several
    # rows; 1030 rows leave the last workgroup partly empty
    x = workloads.gaussian(1030, 2048, seed=600 + B, dtype=torch.bfloat16)
    x[5, :] = -2.0          # a constant row: index order only
    x[1029, 2047] = 50.0
    check_approx(atk, x, K, Kp, B)


def test_kprime_equals_k_and_single_bucket_are_exact(atk):
    x = workloads.gaussian(4, 8192, seed=7)
    for K, Kp, B in [(32, 32, 64), (32, 32, 1), (20, 20, 256), (100, 100, 64), (100, 100, 1),
                     (50, 50, 128)]:
        gv, gi = check_approx(atk, x, K, Kp, B)
        ev, ei = check_exact(atk, x, K)
        assert torch.equal(gi, ei) and torch.equal(gv, ev)


def test_signed_zeros_minus_inf_and_ties(atk):
    # signed zeros: equal in the order, stored bits returned
    x = torch.full((2, 256), -1.0)
    x[0, [10, 40, 77]] = -0.0
    x[0, [3, 50]] = 0.0
    x[1, 5] = -0.0
    for K, Kp, B in [(5, 5, 1), (5, 2, 16), (5, 1, 64), (4, 4, 256 // 4)]:
        check_approx(atk, x, K, Kp, B)
    check_exact(atk, x, 6)
    check_stage1(atk, x, 2, 16)
    xb = x.to(torch.bfloat16)
    check_approx(atk, xb, 5, 2, 16)
    check_exact(atk, xb, 6)
    # rows that are almost entirely -inf: real -inf elements are legitimate outputs
    y = torch.full((3, 4096), float("-inf"))
    y[0, [7, 50, 4000]] = torch.tensor([1.0, 2.0, 3.0])
    y[1, 100] = float("inf")
    for K, Kp, B in [(64, 2, 64), (64, 1, 64), (16, 16, 1), (300, 8, 64), (40, 4, 16)]:
        check_approx(atk, y, K, Kp, B)
        check_stage1(atk, y, Kp, B)
    check_exact(atk, y, 64)
    # heavy ties: 2, 3 and 16 distinct values
    for symbols in (1, 2, 3, 16):
        z = workloads.heavy_ties(4, 8192, seed=symbols, symbols=symbols)
        for K, Kp, B in [(256, 1, 256), (256, 8, 256), (256, 32, 64), (100, 4, 32), (50, 50, 1)]:
            check_approx(atk, z, K, Kp, B)
        check_exact(atk, z, 256)
        check_exact(atk, z.to(torch.bfloat16), 2048)


def test_row_stride_and_views(atk):
    big = workloads.gaussian(6, 4096 + 64, seed=11).to(DEV)
    view = big[:, 32:32 + 4096]            # row stride 4160, base offset 128 bytes
    gv, gi = atk.approx_topk(view, 32, 4, 64)
    ev, ei = atk.topk(view, 32)
    torch.cuda.synchronize()
    xh = view.cpu().contiguous().numpy()
    ov, oi = oracle.approx_topk(xh, 32, 4, 64)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gv.cpu().numpy(), ov)
    ov, oi = oracle.topk(xh, 32)
    assert np.array_equal(ei.cpu().numpy(), oi) and np.array_equal(ev.cpu().numpy(), ov)
    # an odd element offset forces the single-element-load variants
    view2 = big[:, 1:1 + 4096]
    gv, gi = atk.approx_topk(view2, 100, 2, 2048)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(view2.cpu().contiguous().numpy(), 100, 2, 2048)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(gv.cpu().numpy(), ov)


def test_zero_rows(atk):
    x = torch.empty((0, 1024), device=DEV)
    v, i = atk.approx_topk(x, 8, 1, 64)
    assert v.shape == (0, 8) and i.shape == (0, 8)
    v, i = atk.topk(x, 8)
    assert v.shape == (0, 8)


def test_largest_fused_candidate_set(atk, knobs):
    # B*K' = 16384 candidates per row: the most the fused kernel keeps in LDS (128 KB of keys).
    # With so few rows the default route is the slab one (same candidates, in the finishing
    # launch's LDS): first that, then the single fused launch
    N, B, Kp, K = 32768, 2048, 8, 2000
    st, text = atk.describe_plan(torch.float32, 3, N, K, Kp, B)
    assert st == atk.OK and text.startswith("slab") and "cand=16384" in text, text
    check_approx(atk, workloads.gaussian(3, N, seed=17), K, Kp, B)
    knobs.set("slab", 0)
    st, text = atk.describe_plan(torch.float32, 3, N, K, Kp, B)
    assert st == atk.OK and text.startswith("fused") and "cand=16384" in text, text
    check_approx(atk, workloads.gaussian(3, N, seed=17), K, Kp, B)
    check_approx(atk, workloads.heavy_ties(3, N, seed=18, symbols=7), K, Kp, B)
    check_approx(atk, workloads.gaussian(3, N, seed=19, dtype=torch.bfloat16), K, Kp, B)


@pytest.mark.parametrize("route", ["chunked", "unfused"])
def test_survivors_beyond_lds_go_through_the_workspace(atk, knobs, route):
    # B*K' = 32768 survivors per row do not fit the fused kernel's LDS: two launches + workspace.
    # By default all survivors are passed on ("unfused"); with option "chunked" every workgroup
    # takes a chunk of the buckets, runs stage 2 on the chunk's own survivors and passes on its K
    # greatest.
    if route == "chunked":
        knobs.set("chunked", 1)
    N, B, Kp, K = 131072, 2048, 16, 300
    st, text = atk.describe_plan(torch.float32, 4, N, K, Kp, B)
    assert st == atk.OK and text.startswith(route), text
    x = workloads.gaussian(4, N, seed=12)
    check_approx(atk, x, K, Kp, B)
    x = workloads.heavy_ties(3, N, seed=13, symbols=4)
    check_approx(atk, x, K, Kp, B)
    xb = workloads.gaussian(4, N, seed=14, dtype=torch.bfloat16)
    check_approx(atk, xb, K, Kp, B)
    # enough rows that the chip is full without cutting rows any finer than LDS asks for
    st, text = atk.describe_plan(torch.float32, 600, N, K, Kp, B)
    assert st == atk.OK and text.startswith(route) and ("x2 " if route == "chunked" else "x1 ") in text, text
    check_approx(atk, workloads.gaussian(600, N, seed=15), K, Kp, B, rows_to_check=[0, 1, 299, 598, 599])
    # K close to what a chunk holds, ties across chunks
    z = workloads.heavy_ties(3, N, seed=16, symbols=2)
    check_approx(atk, z, 2048, Kp, B)


@pytest.mark.parametrize("rows,N,K,Kp,B,dtype", [
    (8, 262144, 1024, 1, 65536, torch.float32),      # Table 1's K'=1 rows with the most buckets
    (8, 262144, 1024, 1, 32768, torch.float32),
    (8, 262144, 1024, 2, 16384, torch.bfloat16),
    (2, 1 << 20, 5000, 4, 32768, torch.float32),     # K beyond 2048
    (3, 150000, 100, 1, 50000, torch.float32),       # bucket count that is no power of two: ragged last chunk
    (3, 150000, 8192, 3, 50000, torch.int32),
    (1, 1 << 21, 8192, 1, 1 << 20, torch.float32),   # a million buckets
    (70, 1 << 18, 2000, 8, 4096, torch.uint32),
])
def test_large_bucket_counts_unfused_in_bucket_chunks(atk, rows, N, K, Kp, B, dtype):
    st, text = atk.describe_plan(dtype, rows, N, K, Kp, B)
    assert st == atk.OK and text.startswith("unfused"), text
    if dtype in (torch.int32, torch.uint32):
        g = torch.Generator().manual_seed(B)
        x = torch.randint(-4000, 4000, (rows, N), generator=g, dtype=torch.int64)
        x = (x & 0xffffffff).to(torch.uint32) if dtype == torch.uint32 else x.to(torch.int32)
    else:
        x = workloads.gaussian(rows, N, seed=B % 1000, dtype=dtype)
    check_approx(atk, x, K, Kp, B)
    check_stage1(atk, x, Kp, B)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_elements_set_aside_and_inserted_later(atk, knobs, dtype):
    # value+step lists may keep an element that beats a list's least entry aside and insert it
    # when another element of the same list turns up in any lane of the wavefront, or at the end
    # (option "defer": 2 wherever the lists allow it, 0 never).  Same bits as the oracle on
    # random order, ascending order (every element beats its list: the kernel goes back to
    # inserting at once, batch by batch), descending order (nothing ever beats a full list),
    # dense ties, infinities, and one value everywhere; every list length; rows of a few steps
    # up to a thousand
    for rows, N, B, K in [(5, 65536, 256, 200), (6, 1 << 18, 1024, 128), (5, 9 * 640, 640, 64), (7, 40 * 96, 96, 50)]:
        base = torch.randn(rows, N, generator=torch.Generator().manual_seed(N + B))
        x = base.clone()
        x[1] = torch.sort(base[1]).values
        x[2] = torch.sort(base[2], descending=True).values
        x[3] = torch.round(base[3] * 2) / 2
        x[4] = 1.5
        if rows > 5:
            x[5, ::7] = float("inf")
            x[5, 3::11] = float("-inf")
        x = x.to(dtype)
        for Kp in (2, 3, 4, 6, 8):
            if Kp * B < K or Kp > N // B:
                continue
            for defer in (2, 0):
                knobs.set("defer", defer)
                # (16-bit rows: the packed-key lists have no such form; they are switched off)
                knobs.set("packed", 0)
                print(f"defer={defer} {dtype} rows={rows} N={N} B={B} K'={Kp}", flush=True)
                check_approx(atk, x, K, Kp, B)
                check_stage1(atk, x, Kp, B)
            knobs.set("defer", -1)
    # the split route (segments of a row) and the mirrored problem
    knobs.set("defer", 2)
    y = workloads.gaussian(3, 1 << 20, seed=77)
    y[1] = torch.sort(y[1]).values
    check_approx(atk, y, 128, 4, 512)
    gv, gi = atk.approx_topk(y.to(DEV), 128, 4, 512, smallest=True)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(workloads.to_numpy_bits(y), 128, 4, 512, smallest=True)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv), host_bits(ov))


def test_ranking_finish_signed_zeros_and_row_strides(atk):
    # rows whose greatest values are zeros of both signs (equal in the order: the lowest index
    # first, each reported with its own sign, which the second launch reads back from the row),
    # as views with a row stride and a base that is not 16-byte aligned; few-row and unfused routes
    for rows, N, K, Kp, B, route in [(5, 262144, 1024, 4, 1024, "slab"), (6, 1 << 19, 1024, 4, 8192, "unfused")]:
        g = torch.Generator().manual_seed(N + B)
        z = -torch.abs(torch.round(torch.randn(rows, N, generator=g) * 0.7))       # zeros are -0.0
        flip = (z == 0) & (torch.rand(rows, N, generator=g) < 0.5)
        z[flip] = 0.0                                                              # ... half of them +0.0
        z[rows - 1, ::5] = float("-inf")
        big = torch.full((rows, N + 72), 7.0)
        for off in (0, 4, 3):
            big[:, off:off + N] = z
            view = big.to(DEV)[:, off:off + N]
            st, text = atk.describe_plan(torch.float32, rows, N, K, Kp, B)
            assert st == atk.OK and text.startswith(route) and "rank_finish" in text, text
            gv, gi = atk.approx_topk(view, K, Kp, B)
            torch.cuda.synchronize()
            ov, oi = oracle.approx_topk(workloads.to_numpy_bits(z), K, Kp, B)
            assert np.array_equal(gi.cpu().numpy(), oi), (route, off)
            assert np.array_equal(bits(gv), host_bits(ov)), (route, off)
            assert (bits(gv) == 0x80000000).any() and (bits(gv) == 0).any()


def test_unfused_route_with_the_ranking_finish(atk, knobs):
    # survivors beyond LDS whose lanes hold 8 or 16 list entries: every wavefront's survivors
    # leave as one sorted run of 512 or 1024 keys and the second launch places every key by
    # counting the keys above it (many workgroups per row); without the option the survivors
    # leave as values and positions and the exact kernel selects among them
    cases = [(workloads.gaussian(6, 1 << 20, seed=51), 1024, 4, 8192),
             (workloads.gaussian(5, 262144, seed=52, dtype=torch.bfloat16), 1024, 2, 16384),
             (workloads.gaussian(4, 131072, seed=53), 128, 16, 2048),
             (workloads.gaussian(3, 3 << 17, seed=54), 500, 3, 8192),            # three entries per list: padded runs
             (workloads.heavy_ties(7, 65536, seed=55, symbols=5), 2000, 4, 8192),
             (workloads.gaussian(70, 65536, seed=57), 64, 4, 8192)]
    g = torch.Generator().manual_seed(58)
    cases.append((torch.randint(-3000, 3000, (5, 262144), generator=g, dtype=torch.int32), 1024, 4, 8192))
    # the greatest values all in buckets that one wavefront owns: its run holds the whole result
    w = workloads.gaussian(4, 1 << 20, seed=59)
    n = torch.arange(1 << 20)
    for r, b0 in enumerate((0, 128, 8192 - 128, 4096)):
        w[r, (n % 8192 >= b0) & (n % 8192 < b0 + 128)] += 100.0
    cases.append((w, 1024, 4, 8192))
    for x, K, Kp, B in cases:
        st, text = atk.describe_plan(x.dtype, x.shape[0], x.shape[1], K, Kp, B)
        assert st == atk.OK and text.startswith("unfused") and "rank_finish" in text, text
        check_approx(atk, x, K, Kp, B)
        knobs.set("rank_finish", 0)
        st, text = atk.describe_plan(x.dtype, x.shape[0], x.shape[1], K, Kp, B)
        assert st == atk.OK and text.startswith("unfused") and "rank_finish" not in text, text
        check_approx(atk, x, K, Kp, B)
        knobs.set("rank_finish", -1)
    # K so large that the heads of the runs would not fit LDS: the exact kernel selects
    for x, K, Kp, B in [(workloads.heavy_ties(7, 65536, seed=55, symbols=5), 3360, 4, 8192),
                        (workloads.gaussian(2, 1 << 20, seed=56), 8192, 8, 4096)]:
        st, text = atk.describe_plan(x.dtype, x.shape[0], x.shape[1], K, Kp, B)
        assert st == atk.OK and text.startswith("unfused") and "rank_finish" not in text, text
        check_approx(atk, x, K, Kp, B)
    # the K smallest
    x = cases[0][0].to(DEV)
    gv, gi = atk.approx_topk(x, 1024, 4, 8192, smallest=True)
    torch.cuda.synchronize()
    ov, oi = oracle.approx_topk(workloads.to_numpy_bits(cases[0][0]), 1024, 4, 8192, smallest=True)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(bits(gv), host_bits(ov))


def test_forced_unfused_route_matches_on_every_list_representation(atk, knobs):
    # the survivors of any call can be sent through the workspace: lanes sharing buckets, packed
    # and batched lists, integers -- same bits as the oracle
    knobs.set("unfused", 1)
    for x, K, Kp, B in [(workloads.gaussian(37, 8192, seed=33), 40, 4, 16),
                        (workloads.gaussian(300, 16384, seed=31), 128, 4, 1024),
                        (workloads.gaussian(1031, 2048, seed=34, dtype=torch.bfloat16), 287, 4, 128),
                        (workloads.gaussian(129, 65536, seed=35), 256, 32, 256),
                        (workloads.heavy_ties(8, 262144, seed=16, symbols=3), 1024, 4, 1024),
                        (workloads.gaussian(5, 900, seed=36), 40, 30, 3)]:
        st, text = atk.describe_plan(x.dtype, x.shape[0], x.shape[1], K, Kp, B)
        assert st == atk.OK and text.startswith("unfused"), text
        check_approx(atk, x, K, Kp, B)


@pytest.mark.parametrize("N,K", [(5000, 2049), (20000, 4096), (100000, 8192), (8192, 8192), (300000, 5000)])
def test_exact_topk_large_k(atk, N, K):
    check_exact(atk, workloads.gaussian(3, N, seed=N % 89), K)
    check_exact(atk, workloads.heavy_ties(2, N, seed=N % 83, symbols=3).to(torch.bfloat16), K)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.int32])
def test_exact_one_pass_with_rising_threshold_and_its_fallback(atk, knobs, dtype):
    # the exact kernel tries long rows in one pass (keys above a rising threshold collected in LDS,
    # compacted when half full) and falls back to two passes when the buffer overflows; option
    # "onepass" = 2 asks for the attempt on short rows as well.  Random order (the attempt
    # succeeds), ascending order (every element beats the threshold: overflow, fallback),
    # descending order (nothing passes after the first round), dense ties, one value everywhere.
    knobs.set("onepass", 2)
    rng = np.random.default_rng(11)
    for N, K in [(8192, 1), (8192, 1024), (20000, 64), (65536 + 17, 300), (300000, 1000), (1 << 20, 128),
                 (131072 + 8, 1024)]:
        base = torch.randn(5, N, generator=torch.Generator().manual_seed(N + K))
        rows = [base[0], torch.sort(base[1]).values, torch.sort(base[2], descending=True).values,
                torch.round(base[3] * 2) / 2, torch.full((N,), 1.5)]
        x = torch.stack(rows)
        if dtype == torch.int32:
            x = (x * 1000).to(torch.int32)
        else:
            x = x.to(dtype)
        print(f"one pass: {dtype} N={N} K={K}", flush=True)
        check_exact(atk, x, K)
    # survivor mode (the unfused route's second launch reads values and positions from the workspace)
    knobs.set("unfused", 1)
    for rows, N, K, Kp, B in [(6, 65536, 500, 4, 4096), (3, 1 << 18, 1024, 2, 16384), (4, 32768, 100, 1, 8192)]:
        x = workloads.gaussian(rows, N, seed=K)
        x[1] = torch.sort(x[1]).values
        x = x.to(dtype) if dtype != torch.int32 else (x * 1000).to(torch.int32)
        assert atk.describe_plan(x.dtype, rows, N, K, Kp, B)[1].startswith("unfused")
        check_approx(atk, x, K, Kp, B)


def test_long_rows_sharing_a_wavefront(atk):
    # three buckets and rows of 3 * 2^24 elements: the rows a workgroup may address from its first
    # row by 32-bit offsets do not fill a wavefront.  Expected output from planted values (the
    # oracle is not run on rows this long): a background of negative values and, per row, distinct
    # positive values at seeded positions; per bucket the K' greatest planted values survive.
    rows, B, Kp, K = 9, 3, 2, 5
    N = 3 * 2 ** 24
    x = torch.empty((rows, N), dtype=torch.float32, device=DEV)
    n = torch.arange(N, device=DEV, dtype=torch.int64)
    for r in range(rows):
        x[r] = -1.0 - ((n + r) % 977).to(torch.float32) * 1e-3
    del n
    rng = np.random.default_rng(9)
    expected = []
    for r in range(rows):
        pos = np.unique(np.concatenate([[0, 1, 2, N - 1, N - 2, N - 3], rng.integers(0, N, 30)]))
        vals = (1.0 + rng.permutation(len(pos)) * 0.25 + r).astype(np.float32)
        x[r, torch.from_numpy(pos).to(DEV)] = torch.from_numpy(vals).to(DEV)
        surv = []
        for b in range(B):
            inb = sorted(((v, p_) for p_, v in zip(pos.tolist(), vals.tolist()) if p_ % B == b), key=lambda t: -t[0])
            surv += inb[:Kp]
        expected.append(sorted(surv, key=lambda t: -t[0])[:K])
    st, text = atk.describe_plan(torch.float32, rows, N, K, Kp, B)
    print(text, flush=True)
    assert st == atk.OK and "rows_per_wg=8 " in text and "lanes_per_row=8 " in text, text
    gv, gi = atk.approx_topk(x, K, Kp, B)
    torch.cuda.synchronize()
    for r in range(rows):
        assert gi[r].cpu().tolist() == [p_ for _, p_ in expected[r]], r
        assert gv[r].cpu().tolist() == [v for v, _ in expected[r]], r


def test_slab_path_very_few_rows(atk, knobs):
    # the shape of the paper's Table 1 and its neighbours: every workgroup takes 32 buckets of a
    # row over all steps, several lanes per bucket; stage 2 runs in a second launch
    for dtype in (torch.float32, torch.bfloat16, torch.int32):
        for rows, N in [(8, 262144), (1, 65536), (3, 1048576)]:
            if dtype == torch.int32:
                g = torch.Generator().manual_seed(18)
                x = torch.randint(-1000, 1000, (rows, N), generator=g, dtype=torch.int32)   # dense ties
            else:
                x = workloads.gaussian(rows, N, seed=17, dtype=dtype)
            for B, Kp in [(1024, 4), (4096, 2), (8192, 1), (1024, 6), (1024, 16), (16384, 1)]:
                st, text = atk.describe_plan(dtype, rows, N, 1024, Kp, B)
                assert st == atk.OK
                # chosen while the launch stays within 2048 workgroups (slabs of 32 buckets; short
                # lists are given wider slabs), rows of 16-bit elements: from 128 KB on
                # and buckets of at least eight elements (two lanes per bucket, four steps each)
                slab = N // B >= 8 and (rows * (B // 32) <= 2048 or
                                        (Kp == 1 and rows * (B // 128) <= 1024 and N * x.element_size() >= 131072))
                assert text.startswith("slab") == slab, text
                # stage 2 spread over several workgroups per row (every key placed by its rank
                # among the sorted runs the slabs leave) up to 8192 keys per row and lists of 8
                assert ("rank_finish" in text) == (slab and Kp <= 8), text
                if "rank_finish" not in text and not text.startswith("slab"):
                    continue            # (checked by the tests of those routes)
                check_approx(atk, x, 1024, Kp, B)
                if "rank_finish" in text:
                    # ... and in one workgroup per row
                    knobs.set("rank_finish", 0)
                    st, text = atk.describe_plan(dtype, rows, N, 1024, Kp, B)
                    assert text.startswith("slab") == (rows * (B // 32) <= 2048 and N // B >= 8), text
                    assert "rank_finish" not in text, text
                    check_approx(atk, x, 1024, Kp, B)
                    knobs.set("rank_finish", -1)
    z = workloads.heavy_ties(8, 262144, seed=16, symbols=3)
    check_approx(atk, z, 1024, 4, 1024)
    # K from one key to every survivor
    zd = z.to(DEV)
    y = workloads.gaussian(8, 262144, seed=21)
    for K in (4, 33, 2048, 4096):
        check_approx(atk, y, K, 4, 1024)
    check_approx(atk, y, 1, 1, 8192)
    # the greatest values all in the buckets of one slab (and of two): that slab's sorted run
    # holds the whole result, far beyond the head of the run that the placing launch fetches first
    for B, Kp, width in [(1024, 4, 32), (4096, 2, 128), (8192, 1, 128), (8192, 2, 128)]:
        w = workloads.gaussian(4, 262144, seed=22)
        n = torch.arange(262144)
        for r, b0 in enumerate((0, width, B - width, 5 * width)):
            inside = (n % B >= b0) & (n % B < b0 + width)
            if r == 3:
                inside |= (n % B >= B - 2 * width) & (n % B < B - width)
            w[r, inside] += 100.0
        check_approx(atk, w, 1024, Kp, B)
        check_approx(atk, w, 200, Kp, B)
    # asked for where the planner would not choose it: few buckets, bucket counts that are only
    # a multiple of 32, rows that one lane per bucket would cover in a handful of steps
    knobs.set("slab", 2)
    for rows, N, B, Kp, K in [(5, 16384, 64, 4, 200), (2, 96 * 64, 96, 3, 100), (9, 32768, 512, 2, 64),
                              (4, 8192, 256, 8, 256), (3, 160 * 24, 160, 2, 300)]:
        st, text = atk.describe_plan(torch.float32, rows, N, K, Kp, B)
        assert st == atk.OK and text.startswith("slab"), text
        check_approx(atk, workloads.gaussian(rows, N, seed=19), K, Kp, B)
        check_approx(atk, workloads.heavy_ties(rows, N, seed=20, symbols=5), K, Kp, B)
    knobs.set("slab", -1)
    # a workspace that is too small: the call falls back to a route that needs none
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    v1, i1 = atk.approx_topk(zd, 1024, 4, 1024)
    out = (torch.empty_like(v1), torch.empty_like(i1))
    st = atk.lib.atk_approx_topk(zd.data_ptr(), 0, 8, 262144, 262144, 1024, 4, 1024,
                                 out[0].data_ptr(), out[1].data_ptr(), small.data_ptr(), 1024, None)
    torch.cuda.synchronize()
    assert st == atk.OK and torch.equal(out[1], i1) and torch.equal(out[0], v1)


def test_split_path_few_long_rows(atk, knobs):
    # the same shape with rows cut into segments along their length (the route for rows that
    # are few but not very few)
    knobs.set("slab", 0)
    for dtype in (torch.float32, torch.bfloat16):
        x = workloads.gaussian(8, 262144, seed=15, dtype=dtype)
        if dtype == torch.bfloat16:     # half the bytes: the planner would not split by itself
            knobs.set("segments", 8)
        for B, Kp in [(1024, 4), (8192, 1), (512, 6), (2048, 2), (256, 16)]:
            st, text = atk.describe_plan(dtype, 8, 262144, 1024, Kp, B)
            assert st == atk.OK
            if (B, Kp) == (1024, 4):
                assert text.startswith("split"), text
            check_approx(atk, x, 1024, Kp, B)
    knobs.set("segments", -1)
    # ties across segment boundaries, and a workspace that is too small (falls back to one launch)
    z = workloads.heavy_ties(8, 262144, seed=16, symbols=3)
    check_approx(atk, z, 1024, 4, 1024)
    zd = z.to(DEV)
    small = torch.empty(1024, dtype=torch.uint8, device=DEV)
    v1, i1 = atk.approx_topk(zd, 1024, 4, 1024)
    out = (torch.empty_like(v1), torch.empty_like(i1))
    st = atk.lib.atk_approx_topk(zd.data_ptr(), 0, 8, 262144, 262144, 1024, 4, 1024,
                                 out[0].data_ptr(), out[1].data_ptr(), small.data_ptr(), 1024, None)
    torch.cuda.synchronize()
    assert st == atk.OK and torch.equal(out[1], i1) and torch.equal(out[0], v1)


@pytest.mark.parametrize("rows,N,B,Kp,K", [(300001, 32, 4, 2, 7), (1000003, 8, 8, 1, 3), (65537, 1, 1, 1, 1)])
def test_very_many_tiny_rows(atk, rows, N, B, Kp, K):
    # the other extreme: rows far shorter than a wavefront, in a number that is not a multiple of
    # anything (many rows per workgroup, a ragged last workgroup)
    x = workloads.gaussian(rows, N, seed=21)
    check_approx(atk, x, K, Kp, B)
    check_exact(atk, x, K)
    check_approx(atk, workloads.gaussian(rows, N, seed=22, dtype=torch.bfloat16), K, Kp, B)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_longest_row(atk, dtype):
    # one row of the greatest supported length, 2^31 - 65536 elements.  The oracle is not run
    # on 8 GB: the row is a background of negative values with 300 distinct positive values
    # planted at seeded positions (first and last elements, bucket edges, the far end), so the
    # expected output follows from the planted set alone: per bucket its K' greatest planted
    # values survive, the K greatest survivors come out in order; the exact Top-K returns the K
    # greatest planted values.
    N, B, Kp, K = 2 ** 31 - 65536, 8192, 1, 64
    x = torch.empty(N, dtype=dtype, device=DEV)
    chunk = 1 << 26
    for start in range(0, N, chunk):
        n = torch.arange(start, min(N, start + chunk), device=DEV, dtype=torch.int64)
        x[start:start + n.numel()] = (-1.0 - (n % 977).to(torch.float32) * 1e-3).to(dtype)
        del n
    rng = np.random.default_rng(5)
    pos = np.unique(np.concatenate([[0, 1, B - 1, B, N - 1, N - B, N - B - 1, 2 ** 30, 2 ** 30 - 1],
                                    rng.integers(0, N, 291), rng.integers(N - 100000, N, 20)]))
    order = rng.permutation(len(pos))
    if dtype == torch.float32:
        vals = (1.0 + order * 0.01).astype(np.float32)
    else:       # distinct bf16 values: consecutive bit patterns from 1.0 up
        vals = ((0x3F80 + order).astype(np.uint32) << 16).view(np.float32)
    x[torch.from_numpy(pos).to(DEV)] = torch.from_numpy(vals).to(DEV).to(dtype)
    # expected survivors: the greatest planted value of every bucket that holds one
    best = {}
    for p_, v in zip(pos.tolist(), vals.tolist()):
        b = p_ % B
        if b not in best or v > best[b][0]:
            best[b] = (v, p_)
    surv = sorted(best.values(), key=lambda t: -t[0])[:K]
    xd = x.view(1, N)
    print("longest row: approximate", flush=True)
    gv, gi = atk.approx_topk(xd, K, Kp, B)
    torch.cuda.synchronize()
    assert gi.cpu().numpy()[0].tolist() == [p_ for _, p_ in surv]
    assert gv.float().cpu().numpy()[0].tolist() == [v for v, _ in surv]
    print("longest row: exact", flush=True)
    ev, ei = atk.topk(xd, K)
    torch.cuda.synchronize()
    top = sorted(zip(vals.tolist(), pos.tolist()), key=lambda t: -t[0])[:K]
    assert ei.cpu().numpy()[0].tolist() == [p_ for _, p_ in top]
    assert ev.float().cpu().numpy()[0].tolist() == [v for v, _ in top]


def test_exact_topk_sizes(atk):
    for N, K in [(1, 1), (63, 63), (64, 1), (1000, 1000), (5000, 2048), (100000, 7), (300000, 1500)]:
        x = workloads.gaussian(3, N, seed=400 + N % 97)
        check_exact(atk, x, K)
    # all-equal row: every digit of the value is shared, the index digits decide
    x = torch.zeros(2, 70000)
    check_exact(atk, x, 100)
    x = workloads.heavy_ties(2, 200000, seed=8, symbols=2).to(torch.bfloat16)
    check_exact(atk, x, 2000)


def test_results_do_not_depend_on_launch_geometry(atk, knobs):
    # the same problem under different lanes-per-row choices must give identical bits
    x = workloads.gaussian(7, 32768, seed=21).to(DEV)
    ref = None
    for lanes in (64, 128, 256, 512, 1024):
        knobs.set("lanes_per_row", lanes)
        for (K, Kp, B) in [(64, 2, 512), (64, 4, 16)]:
            v, i = atk.approx_topk(x, K, Kp, B)
            torch.cuda.synchronize()
            key = (K, Kp, B)
            if ref is None:
                ref = {}
            if key not in ref:
                ref[key] = (v.clone(), i.clone())
            else:
                assert torch.equal(ref[key][1], i) and torch.equal(ref[key][0], v), (lanes, key)
    knobs.set("lanes_per_row", -1)


def test_results_do_not_depend_on_the_list_representation(atk, knobs):
    # packed 32-bit keys vs value+step lists vs several rows per wavefront (bf16), and sorted
    # batches vs position-by-position updates (fp32, K'=16): identical bits
    xb = workloads.gaussian(1100, 4096, seed=22, dtype=torch.bfloat16).to(DEV)
    for (K, Kp, B) in [(200, 4, 128), (300, 8, 64), (64, 1, 1024)]:
        base = atk.approx_topk(xb, K, Kp, B)
        for env in ({"packed": 0}, {"subwave": 0}, {"lanes_per_row": 128}):
            for k, v in env.items():
                knobs.set(k, v)
            other = atk.approx_topk(xb, K, Kp, B)
            torch.cuda.synchronize()
            for k in env:
                knobs.set(k, -1)
            assert torch.equal(base[1], other[1]) and torch.equal(base[0], other[0]), (K, Kp, B, env)
    xf = workloads.gaussian(64, 32768, seed=23).to(DEV)
    base = atk.approx_topk(xf, 500, 16, 128)
    knobs.set("batch_min_kp", 64)
    other = atk.approx_topk(xf, 500, 16, 128)
    torch.cuda.synchronize()
    knobs.set("batch_min_kp", -1)
    assert torch.equal(base[1], other[1]) and torch.equal(base[0], other[0])


# ---------------------------------------------------------------------------------------
# full benchmark sizes, in the launch configuration bench.py times: every row of every setting
# against the oracle, bit for bit; structural properties as a second line of defence
# ---------------------------------------------------------------------------------------

def check_properties(xd, gv, gi, K, Kp, B):
    rows, N = xd.shape
    gi64 = gi.long()
    assert int(gi64.min()) >= 0 and int(gi64.max()) < N
    gathered = torch.gather(xd, 1, gi64)
    assert torch.equal(gathered.view(torch.int16 if xd.dtype == torch.bfloat16 else torch.int32),
                       gv.view(torch.int16 if xd.dtype == torch.bfloat16 else torch.int32))
    vf = gv.float()
    assert bool((vf[:, :-1] >= vf[:, 1:]).all())
    tie = vf[:, :-1] == vf[:, 1:]
    assert bool((gi64[:, :-1][tie] < gi64[:, 1:][tie]).all())
    # distinct indices; at most K' per bucket
    srt = torch.sort(gi64, dim=1).values
    assert bool((srt[:, 1:] != srt[:, :-1]).all())
    counts = torch.zeros(rows, B, dtype=torch.int32, device=xd.device)
    counts.scatter_add_(1, gi64 % B, torch.ones_like(gi64, dtype=torch.int32))
    assert int(counts.max()) <= Kp


@pytest.mark.parametrize("name", ["c2_ffn", "c3_vocab", "c4_mips", "c5_adversarial"])
def test_full_size_every_row_against_the_oracle(atk, name):
    w = workloads.WORKLOADS[name]
    xd = workloads.make(name, seed=1, device=DEV)
    assert xd.shape == (w.rows, w.N)
    xh = workloads.to_numpy_bits(xd)
    for B, Kp in w.params:
        print(f"{name}: B={B} K'={Kp}", flush=True)
        # the plan bench.py times (same rows, same arguments, no workspace offered or needed)
        assert atk.describe_plan(w.dtype, w.rows, w.N, w.K, Kp, B)[1].startswith("fused")
        gv, gi = atk.approx_topk(xd, w.K, Kp, B)
        torch.cuda.synchronize()
        check_properties(xd, gv, gi, w.K, Kp, B)
        ov, oi = oracle.approx_topk(xh, w.K, Kp, B)
        gi_h, gv_h = gi.cpu().numpy(), bits(gv)
        bad = np.flatnonzero((gi_h != oi).any(axis=1) | (gv_h != host_bits(ov)).any(axis=1))
        assert bad.size == 0, (name, B, Kp, "rows that differ:", bad[:10].tolist(), "of", bad.size)
    print(f"{name}: exact", flush=True)
    gv, gi = atk.topk(xd, w.K)
    torch.cuda.synchronize()
    check_properties(xd, gv, gi, w.K, w.K, 1)
    ov, oi = oracle.topk(xh, w.K)
    gi_h, gv_h = gi.cpu().numpy(), bits(gv)
    bad = np.flatnonzero((gi_h != oi).any(axis=1) | (gv_h != host_bits(ov)).any(axis=1))
    assert bad.size == 0, (name, "exact: rows that differ:", bad[:10].tolist(), "of", bad.size)
    # the radix-selection kernel by itself (no workspace), and the mirrored problem: approximate at
    # the first setting, exact
    print(f"{name}: exact without a workspace, min-K", flush=True)
    rv, ri = atk.topk(xd, w.K, workspace=False)
    torch.cuda.synchronize()
    assert torch.equal(ri, gi) and np.array_equal(bits(rv), gv_h)
    B, Kp = w.params[0]
    for call, ref in ((lambda: atk.approx_topk(xd, w.K, Kp, B, smallest=True),
                       lambda: oracle.approx_topk(xh, w.K, Kp, B, smallest=True)),
                      (lambda: atk.topk(xd, w.K, smallest=True), lambda: oracle.topk(xh, w.K, smallest=True))):
        mv, mi = call()
        torch.cuda.synchronize()
        ov, oi = ref()
        bad = np.flatnonzero((mi.cpu().numpy() != oi).any(axis=1) | (bits(mv) != host_bits(ov)).any(axis=1))
        assert bad.size == 0, (name, "min-K: rows that differ:", bad[:10].tolist(), "of", bad.size)


def test_hip_graph_capture_and_replay(atk, knobs):
    # The library enqueues on the caller's stream, allocates nothing and never synchronises, so a
    # call can be captured into a HIP graph.  Every replay (with eager work and synchronisation
    # in between, and new contents in the captured input buffer) must equal the eager result.
    cases = [
        ("fused", lambda x, out, ws: atk.approx_topk(x, 128, 4, 1024, out=out, workspace=ws), (256, 65536)),
        ("slab", lambda x, out, ws: atk.approx_topk(x, 1024, 4, 1024, out=out, workspace=ws), (8, 262144)),
        ("split", lambda x, out, ws: atk.approx_topk(x, 1024, 4, 1024, out=out, workspace=ws), (8, 262144)),
        # exact Top-K: two-stage kernels, certificate kernel, radix kernel over the flagged rows
        ("certified", lambda x, out, ws: atk.topk(x, 128, out=out, workspace=ws), (40, 65536)),
    ]
    for name, call, (rows, N) in cases:
        K = 128 if name in ("fused", "certified") else 1024
        if name == "split":
            knobs.set("slab", 0)
        if name == "certified":
            assert atk.describe_topk_plan(torch.float32, rows, N, K)[1].startswith(name)
        else:
            assert atk.describe_plan(torch.float32, rows, N, K, 4, 1024)[1].startswith(name)
        static_in = workloads.gaussian(rows, N, seed=70).to(DEV)
        ws = torch.empty(64 << 20, dtype=torch.uint8, device=DEV)
        out = (torch.empty((rows, K), device=DEV), torch.empty((rows, K), dtype=torch.int32, device=DEV))
        ref = (torch.empty_like(out[0]), torch.empty_like(out[1]))
        call(static_in, out, ws)                       # eager once before capturing
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        with torch.cuda.graph(graph, stream=side):
            call(static_in, out, ws)
        for replay in range(4):
            fresh = workloads.gaussian(rows, N, seed=71 + replay).to(DEV)
            static_in.copy_(fresh)
            out[0].zero_(); out[1].zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            call(fresh, ref, ws)                       # eager, same input
            torch.cuda.synchronize()
            assert torch.equal(out[1], ref[1]) and torch.equal(out[0], ref[0]), (name, replay)
        # and one replay against the oracle
        if name == "certified":
            ov, oi = oracle.topk(static_in.cpu().numpy()[:2], K)
        else:
            ov, oi = oracle.approx_topk(static_in.cpu().numpy()[:2], K, 4, 1024)
        assert np.array_equal(out[1].cpu().numpy()[:2], oi)


def test_random_bit_patterns_through_every_stage2(atk):
    # values drawn uniformly from the non-NaN binary32 patterns: both signs, infinities,
    # subnormals, the whole exponent range -- the band of keys stage 2 sees is as wide as it gets
    rng = np.random.default_rng(77)
    def patterns(rows, N):
        mag = rng.integers(0, 0x7F800001, (rows, N), dtype=np.int64).astype(np.uint32)
        sign = (rng.integers(0, 2, (rows, N), dtype=np.int64) << 31).astype(np.uint32)
        return torch.from_numpy((mag | sign).view(np.float32))
    x = patterns(8, 262144)
    check_approx(atk, x, 1024, 4, 1024)          # slab route, finish kernel
    check_approx(atk, x, 1024, 2, 4096)          # fused, one row per workgroup
    check_exact(atk, x, 2048)
    y = patterns(64, 16384)
    for B, Kp, K in [(64, 8, 300), (256, 4, 1000), (1024, 1, 512), (16, 2, 20)]:
        check_approx(atk, y, K, Kp, B)
    # a narrow band that straddles a power of two (patterns differ in a high bit, values barely)
    z = (2.0 + (torch.from_numpy(rng.integers(-2000, 2000, (8, 262144))).float() * 2.0 ** -22)).contiguous()
    check_approx(atk, z, 1024, 4, 1024)
    check_exact(atk, z, 1500)


@pytest.mark.parametrize("seed,cases,max_n,min_ran", [(2024, 90, 150000, 70), (2025, 30, 1500000, 20)])
def test_seeded_random_shapes_all_element_types(atk, seed, cases, max_n, min_ran):
    # shapes no hand-written case lists: bucket counts of every kind (tiny, powers of two,
    # multiples of 32, arbitrary), list lengths up to 32, every element type, inputs with dense
    # ties or in descending order; approximate and exact kernels against the oracle, bit for bit.
    # The second setting draws long rows (largest workgroups, few-row routes).
    rng = np.random.default_rng(seed)
    dtypes = [torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.uint32]

    def raw(t):
        t = t.detach().cpu().contiguous()
        return (t.view(torch.int16).numpy().view(np.uint16) if t.element_size() == 2
                else t.view(torch.int32).numpy().view(np.uint32))

    def oracle_raw(a):
        return a.view(np.uint16) if a.dtype.itemsize == 2 else a.view(np.uint32)

    ran = 0
    for case in range(cases):
        dt = dtypes[int(rng.integers(5))]
        kind = int(rng.integers(4))
        B = (int(rng.integers(1, 65)) if kind == 0 else int(2 ** rng.integers(0, 13)) if kind == 1
             else int(rng.integers(1, 40)) * 32 if kind == 2 else int(rng.integers(65, 5000)))
        steps = int(rng.integers(1, max(1, min(300 if max_n <= 150000 else 3000, max_n // B)) + 1))
        N = B * steps
        Kp = int(rng.integers(1, min(steps, 32) + 1))
        if rng.random() < 0.5:
            Kp = min(Kp, 4)
        K = int(rng.integers(Kp, min(B * Kp, N, 2048) + 1))
        rows = int(rng.integers(1, 40 if N < 300000 else 6))
        style = int(rng.integers(3))
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        if dt in (torch.int32, torch.uint32):
            lo, hi = (-(1 << 31), 1 << 31) if style == 0 else (-50, 50)
            x = torch.randint(lo, hi, (rows, N), generator=g, dtype=torch.int64)
            x = (x & 0xffffffff).to(torch.uint32) if dt == torch.uint32 else x.to(torch.int32)
        else:
            x = torch.randn(rows, N, generator=g)
            if style == 1:
                x = torch.round(x * 4) / 4
            elif style == 2:
                x = torch.sort(x, dim=1, descending=True).values
            x = x.to(dt)
        status, _ = atk.describe_plan(dt, rows, N, K, Kp, B)
        if status == atk.UNSUPPORTED:      # more than 16384 list entries per row: documented limit
            assert B * Kp > 8192
            continue
        print(f"case {case}: {dt} rows={rows} N={N} B={B} K'={Kp} K={K} style={style}", flush=True)
        xh, xd = workloads.to_numpy_bits(x), x.to(DEV)
        gv, gi = atk.approx_topk(xd, K, Kp, B)
        torch.cuda.synchronize()
        ov, oi = oracle.approx_topk(xh, K, Kp, B)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(raw(gv), oracle_raw(ov)), case
        ev, ei = atk.topk(xd, K)
        torch.cuda.synchronize()
        ov, oi = oracle.topk(xh, K)
        assert np.array_equal(ei.cpu().numpy(), oi) and np.array_equal(raw(ev), oracle_raw(ov)), case
        ran += 1
    assert ran >= min_ran


@pytest.mark.parametrize("seed,cases,finish_options", [(3101, 50, False), (4202, 50, True)])
def test_seeded_random_shapes_many_buckets_large_k_and_options(atk, knobs, seed, cases, finish_options):
    # what the sweep above does not reach: bucket counts up to 2^18 (survivors through the
    # workspace, rows cut along the bucket axis), K up to 8192, random developer options (chunked,
    # unfused, one-pass exact, slab; finish_options: also the ranking finish switched off, slab
    # widths, lanes per bucket and workgroup counts other than the planner's), and the entry that
    # allocates nothing; approximate and exact kernels against the oracle, bit for bit
    rng = np.random.default_rng(seed)
    dtypes = [torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.uint32]

    def raw(t):
        t = t.detach().cpu().contiguous()
        return (t.view(torch.int16).numpy().view(np.uint16) if t.element_size() == 2
                else t.view(torch.int32).numpy().view(np.uint32))

    def oracle_raw(a):
        return a.view(np.uint16) if a.dtype.itemsize == 2 else a.view(np.uint32)

    for case in range(cases):
        dt = dtypes[int(rng.integers(5))]
        kind = int(rng.integers(3))
        B = (int(2 ** rng.integers(10, 19)) if kind == 0 else int(rng.integers(1, 300)) * int(2 ** rng.integers(5, 11))
             if kind == 1 else int(rng.integers(2000, 60000)))
        steps = int(rng.integers(1, max(2, min(64, 2000000 // B)) + 1))
        N = B * steps
        Kp = int(rng.integers(1, min(steps, 32) + 1))
        if rng.random() < 0.6:
            Kp = min(Kp, 4)
        K = int(rng.integers(Kp, min(B * Kp, N, 8192) + 1))
        if rng.random() < 0.5:
            K = min(K, 1024)
        rows = int(rng.integers(1, 12 if N < 500000 else 4))
        style = int(rng.integers(3))
        opts = {}
        if rng.random() < 0.3:
            opts["chunked"] = 1
        if rng.random() < 0.3:
            opts["unfused"] = 1
        if rng.random() < 0.4:
            opts["onepass"] = 2
        if rng.random() < 0.2:
            opts["slab"] = int(rng.integers(0, 3))
        if finish_options:
            if rng.random() < 0.5:
                opts["slab"] = 2
            if rng.random() < 0.25:
                opts["rank_finish"] = 0
            if rng.random() < 0.3:
                opts["slab_width"] = int(2 ** rng.integers(5, 9))
            if rng.random() < 0.3:
                opts["slab_owners"] = int(2 ** rng.integers(1, 5))
            if rng.random() < 0.3:
                opts["rank_wgs"] = int(2 ** rng.integers(4, 13))
            if rng.random() < 0.5:
                opts["defer"] = int(rng.choice([0, 2]))
        for k, v in opts.items():
            knobs.set(k, v)
        g = torch.Generator().manual_seed(int(rng.integers(1 << 30)))
        if dt in (torch.int32, torch.uint32):
            lo, hi = (-(1 << 31), 1 << 31) if style == 0 else (-50, 50)
            x = torch.randint(lo, hi, (rows, N), generator=g, dtype=torch.int64)
            x = (x & 0xffffffff).to(torch.uint32) if dt == torch.uint32 else x.to(torch.int32)
        else:
            x = torch.randn(rows, N, generator=g)
            if style == 1:
                x = torch.round(x * 4) / 4
            elif style == 2:
                x = torch.sort(x, dim=1, descending=bool(rng.integers(2))).values
            x = x.to(dt)
        status, plan = atk.describe_plan(dt, rows, N, K, Kp, B)
        assert status == atk.OK, plan
        print(f"case {case}: {dt} rows={rows} N={N} B={B} K'={Kp} K={K} style={style} {opts} "
              f"{plan.split(' KP=')[0]}{' ranked' if 'rank_finish' in plan else ''}", flush=True)
        xh, xd = workloads.to_numpy_bits(x), x.to(DEV)
        gv, gi = atk.approx_topk(xd, K, Kp, B)
        torch.cuda.synchronize()
        ov, oi = oracle.approx_topk(xh, K, Kp, B)
        assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(raw(gv), oracle_raw(ov)), case
        out = (torch.zeros_like(gv), torch.zeros_like(gi))
        rc = atk.lib.atk_approx_topk_noalloc(xd.data_ptr(), atk._CODES[dt], rows, N, N, K, Kp, B,
                                             out[0].data_ptr(), out[1].data_ptr(), None)
        torch.cuda.synchronize()
        assert rc == atk.WORKSPACE_TOO_SMALL or (rc == atk.OK and torch.equal(out[1], gi)), (case, rc)
        ev, ei = atk.topk(xd, K)
        torch.cuda.synchronize()
        ov, oi = oracle.topk(xh, K)
        assert np.array_equal(ei.cpu().numpy(), oi) and np.array_equal(raw(ev), oracle_raw(ov)), case
        for k in opts:
            knobs.set(k, -1)
