"""Exact Top-K through the two-stage kernels plus the exactness certificate (the route atk_topk
takes on rows that are long against K when it is handed a workspace): bit for bit the oracle's
exact Top-K, on rows that certify at once, rows that need buckets repaired, and rows the
certificate kernel gives up on (which the radix-selection kernel then does)."""
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


def check(atk, x, K, smallest=False, expect="certified"):
    rows, N = x.shape
    st, text = atk.describe_topk_plan(x.dtype, rows, N, K)
    assert st == atk.OK and text.startswith(expect), text
    print(f"exact via {text.split(' (')[0]}: {x.dtype} rows={rows} N={N} K={K} smallest={smallest}", flush=True)
    xd = x.view(torch.int32).to(DEV).view(torch.uint32) if x.dtype == torch.uint32 else x.to(DEV)
    gv, gi = atk.topk(xd, K, smallest=smallest)                      # workspace allocated by the binding
    rv, ri = atk.topk(xd, K, smallest=smallest, workspace=False)     # the radix-selection kernel alone
    torch.cuda.synchronize()
    ov, oi = oracle.topk(workloads.to_numpy_bits(x), K, smallest=smallest)
    assert np.array_equal(gi.cpu().numpy(), oi), "indices differ from the oracle"
    assert np.array_equal(raw(gv), oracle_raw(ov)), "values differ from the oracle"
    assert torch.equal(gi, ri) and np.array_equal(raw(gv), raw(rv))


def packed_into_buckets(rows, N, K, B, buckets, seed, extra=0):
    """N(0,1) rows whose K + extra greatest values all sit at positions p with p mod B in the first
    `buckets` residues of a seeded offset: those buckets hold far more than K' of the Top-K."""
    g = np.random.default_rng(seed)
    x = g.standard_normal((rows, N)).astype(np.float32)
    per = -(-(K + extra) // buckets)
    assert per <= N // B
    for r in range(rows):
        b0 = int(g.integers(0, B - buckets))
        pos = (b0 + np.arange(buckets)[None, :] + B * g.choice(N // B, per, replace=False)[:, None]).ravel()[:K + extra]
        x[r, pos] = 10.0 + g.random(len(pos)).astype(np.float32)
    return torch.from_numpy(x)


def test_rows_in_random_order_certify_or_repair_single_buckets(atk):
    check(atk, workloads.gaussian(300, 65536, seed=1), 64)
    check(atk, workloads.gaussian(70, 262144, seed=2), 128)
    check(atk, workloads.gaussian(33, 65536, seed=3), 256)            # about one bucket per row in doubt
    check(atk, workloads.gaussian(16, 4096, seed=4), 32)
    check(atk, workloads.gaussian(7, 50000, seed=5), 77)              # B = 400: no power of two divides N far enough
    check(atk, workloads.vocab_logits(64, 256000, seed=6), 64)
    check(atk, workloads.gaussian(6, 262144, seed=7), 1024)           # few rows: stage 1 through the workspace
    check(atk, workloads.gaussian(300, 65536, seed=8), 64, smallest=True)


def test_every_element_type(atk):
    check(atk, workloads.gaussian(130, 65536, seed=11, dtype=torch.bfloat16), 100)
    check(atk, workloads.gaussian(130, 65536, seed=12).to(torch.float16), 100, smallest=True)
    g = np.random.default_rng(13)
    i32 = torch.from_numpy(g.integers(-2 ** 31, 2 ** 31, (50, 65536)).astype(np.int32))
    check(atk, i32, 128)
    check(atk, i32.view(torch.uint32), 128, smallest=True)
    check(atk, torch.from_numpy(g.integers(-40, 40, (50, 65536)).astype(np.int32)), 200)   # heavy ties


def test_top_k_packed_into_few_buckets_is_repaired(atk):
    # 64 greatest in 2 buckets (32 each), in 4, in 16: two, four, sixteen buckets read again
    check(atk, packed_into_buckets(40, 65536, 64, 256, 2, seed=21), 64)
    check(atk, packed_into_buckets(40, 65536, 64, 256, 4, seed=22), 64)
    check(atk, packed_into_buckets(40, 65536, 64, 256, 16, seed=23), 64)
    # the benchmark's adversarial rows (ascending, Top-K in four adjacent buckets) and its tie rows
    check(atk, workloads.make("c5_adversarial", seed=24, rows=64), 256)
    check(atk, workloads.make("c5_adversarial", seed=25, rows=64), 256, smallest=True)
    # ascending and descending rows
    asc = torch.sort(workloads.gaussian(5, 131072, seed=26), dim=1).values
    check(atk, asc, 128)
    check(atk, asc.flip(1).contiguous(), 128)
    check(atk, asc, 128, smallest=True)


def test_rows_the_certificate_kernel_gives_up_on_go_to_the_radix_kernel(atk):
    # one bucket holds more qualifying elements than the repair buffer takes (1024 keys at K = 128):
    # K + 1000 planted values in one bucket of 1024 elements
    check(atk, packed_into_buckets(6, 1 << 20, 128, 1024, 1, seed=31, extra=890), 128)
    # massive ties: every value equal, and rows of two symbols
    check(atk, torch.ones(5, 65536), 64)
    check(atk, workloads.heavy_ties(20, 65536, seed=32, symbols=2), 256)
    check(atk, workloads.heavy_ties(20, 65536, seed=33, symbols=2), 256, smallest=True)
    # zeros of both signs among the greatest
    z = -torch.rand(9, 65536, generator=torch.Generator().manual_seed(34))
    z[:, ::3] = 0.0
    z[:, 1::3] = -0.0
    check(atk, z, 100)
    # mixed: some rows certify, some are repaired, some are given up on, in one call
    x = workloads.gaussian(12, 1 << 20, seed=35)
    x[3:6] = packed_into_buckets(3, 1 << 20, 128, 1024, 2, seed=36)
    x[8:10] = packed_into_buckets(2, 1 << 20, 128, 1024, 1, seed=37, extra=890)
    x[11] = 1.0
    check(atk, x, 128)


def test_switched_off_and_without_workspace(atk, knobs):
    x = workloads.gaussian(50, 65536, seed=41)
    knobs.set("certified", 0)
    check(atk, x, 64, expect="radix")


def test_poisoned_workspace_and_guard_bands(atk):
    from test_gpu_guard import Guarded, POISONS
    x = packed_into_buckets(30, 65536, 64, 256, 4, seed=51)
    x[10:20] = workloads.gaussian(10, 65536, seed=52)
    x[25:] = 2.0
    rows, N, K = 30, 65536, 64
    ov, oi = oracle.topk(x.numpy(), K)
    need = atk.workspace_bytes(atk.OP_TOPK, x.dtype, rows, N, K, 0, 0)
    assert 0 < need < atk.SIZE_MAX
    xd = x.to(DEV)
    for poison in POISONS:
        gv, gi = Guarded(rows * K * 4, fill=0x3C), Guarded(rows * K * 4, fill=0x3C)
        ws = Guarded(need, fill=poison)
        print(f"guarded certified exact: poison={poison:#x}", flush=True)
        rc = atk.lib.atk_topk(xd.data_ptr(), atk.F32, rows, N, N, K, gv.ptr, gi.ptr, ws.ptr, ws.nbytes, None)
        torch.cuda.synchronize()
        assert rc == atk.OK and gv.intact() and gi.intact() and ws.intact()
        assert np.array_equal(gi.view(torch.int32, (rows, K)).cpu().numpy(), oi)
        assert np.array_equal(raw(gv.view(torch.float32, (rows, K))), ov.view(np.uint32))


def test_short_rows_kept_in_registers(atk, knobs):
    """Rows of at most 256 x 8 vectors of 16 bytes: the radix-selection kernel loads them once and runs
    every pass from registers; with the option off the same kernel streams them from memory."""
    g = np.random.default_rng(61)
    cases = [
        (workloads.gaussian(300, 14336, seed=62, dtype=torch.bfloat16), 287),
        (workloads.gaussian(300, 14336, seed=63, dtype=torch.bfloat16).to(torch.float16), 100),
        (workloads.gaussian(100, 8192, seed=64), 2048),                 # K large against the row
        (workloads.gaussian(100, 8192, seed=65), 1),
        (workloads.gaussian(50, 4100, seed=66), 33),                    # a ragged last vector round
        (workloads.heavy_ties(60, 8192, seed=67, symbols=2), 500),      # further digits, down to the index
        (torch.ones(9, 16384, dtype=torch.bfloat16), 300),
        (torch.from_numpy(g.integers(-2 ** 31, 2 ** 31, (40, 8192)).astype(np.int32)), 77),
        (torch.from_numpy(g.integers(-3, 3, (40, 8192)).astype(np.int32)).view(torch.uint32), 700),
        (workloads.gaussian(20, 1024, seed=68), 1024),                  # K = N
    ]
    for x, K in cases:
        for smallest in (False, True):
            xd = x.view(torch.int32).to(DEV).view(torch.uint32) if x.dtype == torch.uint32 else x.to(DEV)
            ov, oi = oracle.topk(workloads.to_numpy_bits(x), K, smallest=smallest)
            for regs in (1, 0):
                knobs.set("reg_rows", regs)
                print(f"short rows: {x.dtype} {tuple(x.shape)} K={K} smallest={smallest} reg_rows={regs}", flush=True)
                gv, gi = atk.topk(xd, K, smallest=smallest, workspace=False)
                torch.cuda.synchronize()
                assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(raw(gv), oracle_raw(ov))
    # an unaligned view (odd row stride): single-element loads, rows never go into registers
    base = workloads.gaussian(6, 8195, seed=69)
    xd = base.to(DEV)[:, 3:]
    gv, gi = atk.topk(xd, 64, workspace=False)
    torch.cuda.synchronize()
    ov, oi = oracle.topk(np.ascontiguousarray(base[:, 3:].numpy()), 64)
    assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(raw(gv), oracle_raw(ov))


def _random_rows(rng, rows, N, dt, style, K):
    if dt in (torch.int32, torch.uint32):
        lo, hi = (-(1 << 31), (1 << 31)) if style % 2 == 0 else (-50, 50)
        x = rng.integers(lo, hi, (rows, N)).astype(np.uint32).view(np.int32)
        if style == 2:
            x = np.sort(x, axis=1)
        t = torch.from_numpy(x)
        return t.view(torch.uint32) if dt == torch.uint32 else t
    x = rng.standard_normal((rows, N)).astype(np.float32)
    if style == 1:                                     # heavy ties
        x = np.round(x * 4) / 4
    elif style == 2:                                   # sorted, either way
        x = np.sort(x, axis=1)[:, ::-1 if rng.integers(2) else 1].copy()
    elif style == 3:                                   # extremes packed into a few residues of a random modulus
        m = int(2 ** rng.integers(6, 12))
        nb = int(rng.integers(1, 5))
        cnt = min(N // m, (K + int(rng.integers(0, 900))) // nb + 1)
        for r in range(rows):
            if N // m == 0:
                break
            b0 = int(rng.integers(0, m - nb))
            pos = (b0 + np.arange(nb)[None, :] + m * rng.choice(N // m, cnt, replace=False)[:, None]).ravel()
            pos = pos[pos < N]
            x[r, pos] = (10.0 + rng.random(len(pos))) * (1 if rng.integers(2) else -1)
    return torch.from_numpy(x).to(dt)


@pytest.mark.parametrize("seed,cases", [(4101, 60)])
def test_seeded_random_shapes_exact_and_min_k(atk, knobs, seed, cases):
    """Random row lengths (powers of two, odd multiples, arbitrary, short), K, element types, value
    patterns and developer options through atk_topk / atk_mink, against the oracle bit for bit."""
    rng = np.random.default_rng(seed)
    dts = [torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.uint32]
    for c in range(cases):
        dt = dts[int(rng.integers(5))]
        kind = int(rng.integers(4))
        if kind == 0:
            N = int(2 ** rng.integers(10, 21))
        elif kind == 1:
            N = int(rng.integers(1, 64)) * int(2 ** rng.integers(6, 15))
        elif kind == 2:
            N = int(rng.integers(1000, 300000))
        else:
            N = int(rng.integers(1, 9)) * 2048
        K = int(rng.integers(1, min(N, 1100) + 1))
        if rng.random() < 0.5:
            K = min(K, int(rng.integers(1, 300)))
        rows = int(rng.integers(1, 40 if N < 100000 else 6))
        style = int(rng.integers(4))
        smallest = bool(rng.integers(2))
        opts = {}
        if rng.random() < 0.2:
            opts["certified"] = 0
        if rng.random() < 0.3:
            opts["reg_rows"] = 0
        if rng.random() < 0.3:
            opts["onepass"] = 2
        for k, v in opts.items():
            knobs.set(k, v)
        plan = atk.describe_topk_plan(dt, rows, N, K)[1]
        print(f"case {c}: {dt} rows={rows} N={N} K={K} style={style} smallest={smallest} opts={opts} {plan[:28]}", flush=True)
        x = _random_rows(rng, rows, N, dt, style, K)
        xd = x.view(torch.int32).to(DEV).view(torch.uint32) if dt == torch.uint32 else x.to(DEV)
        ev, ei = atk.topk(xd, K, smallest=smallest)
        torch.cuda.synchronize()
        ov, oi = oracle.topk(workloads.to_numpy_bits(x), K, smallest=smallest)
        assert np.array_equal(ei.cpu().numpy(), oi) and np.array_equal(raw(ev), oracle_raw(ov)), f"case {c}"
        for k in opts:
            knobs.set(k, -1)


def test_many_short_rows_certified_by_single_wavefronts(atk):
    """4096 rows and more with at most 1024 buckets: every wavefront of the certificate kernel takes
    rows by itself and hands the workgroup what it cannot settle (a ragged last workgroup, rows with
    elements to merge in, rows with many buckets in doubt, rows given up on)."""
    rows = 4100 + 3
    x = workloads.gaussian(rows, 4096, seed=71)
    x[100:140] = packed_into_buckets(40, 4096, 64, 64, 2, seed=72)        # 32 per bucket: merged by the workgroup
    x[1000:1010] = packed_into_buckets(10, 4096, 64, 64, 16, seed=73)     # sixteen buckets in doubt
    x[2000:2004] = 1.0                                                     # ties
    x[4099:] = packed_into_buckets(4, 4096, 64, 64, 1, seed=74)           # the ragged tail
    check(atk, x, 64)
    check(atk, x, 64, smallest=True)
    check(atk, x.to(torch.bfloat16), 64)
    # the FFN shape at reduced row count: K' = 8 on the packed-key kernels
    y = workloads.gaussian(4200, 14336, seed=75, dtype=torch.bfloat16)
    assert "K'=8" in atk.describe_topk_plan(y.dtype, 4200, 14336, 287)[1]
    check(atk, y, 287)
    check(atk, y.to(torch.float16), 287, smallest=True)


def test_strided_and_unaligned_rows_through_the_exact_route(atk):
    """Views with a row stride beyond N and a base that is not 16-byte aligned: the two-stage
    kernels take their single-element loads, the certificate kernel and the radix kernel read the
    same rows through the same stride."""
    for dt in (torch.float32, torch.bfloat16):
        base = workloads.gaussian(37, 65536 + 5, seed=81, dtype=dt)
        base[5:9, 3:65539] = packed_into_buckets(4, 65536, 64, 256, 2, seed=82).to(dt)      # rows that need a repair
        base[20, 3:65539] = 1.0                                                         # ties
        xd = base.to(DEV)[:, 3:65539]
        assert xd.stride(0) == 65541 and xd.data_ptr() % 16 != 0
        assert atk.describe_topk_plan(dt, 37, 65536, 64)[1].startswith("certified")
        x = base[:, 3:65539].contiguous()
        for smallest in (False, True):
            gv, gi = atk.topk(xd, 64, smallest=smallest)
            torch.cuda.synchronize()
            ov, oi = oracle.topk(workloads.to_numpy_bits(x), 64, smallest=smallest)
            assert np.array_equal(gi.cpu().numpy(), oi) and np.array_equal(raw(gv), oracle_raw(ov)), (dt, smallest)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.int32, torch.uint32])
def test_very_small_k_through_lists_of_k_entries(atk, knobs, dtype):
    # K below 8: the two-stage kernels with K' = K keep the whole Top-K by construction, so they are
    # the exact route (few long rows: the routes that cut rows; many short ones: several rows per
    # workgroup; bucket counts that are no power of two); lists of 5 to 7 entries only when the
    # rows are few.  Dense ties, both zeros, infinities, the K smallest, no workspace, option off.
    for rows, N, Ks in [(3, 1 << 20, (1, 2, 4, 7)), (50, 65536, (1, 3, 4, 6)), (3000, 4096, (1, 2, 4)),
                        (700, 30000, (1, 4)), (9, 15015 * 16, (2, 5))]:
        g = torch.Generator().manual_seed(N + rows)
        if dtype in (torch.int32, torch.uint32):
            x = torch.randint(-40, 40, (rows, N), generator=g, dtype=torch.int64)
            x = (x & 0xffffffff).to(torch.uint32) if dtype == torch.uint32 else x.to(torch.int32)
        else:
            x = torch.round(torch.randn(rows, N, generator=g) * 3) / 3
            x[0, 5::7] = 0.0
            x[0, 6::7] = -0.0
            x[rows - 1, ::1001] = float("inf")
            x[rows - 1, 1::1003] = float("-inf")
            x = x.to(dtype)
        for K in Ks:
            check(atk, x, K, expect="two-stage")
            check(atk, x, K, smallest=True, expect="two-stage")
    # rows too short for it, and lists of more than four entries with many rows: the radix kernel
    x = workloads.gaussian(400, 480, seed=5).to(dtype) if dtype not in (torch.int32, torch.uint32) else \
        torch.randint(0, 1000, (400, 480), dtype=torch.int32).to(dtype)
    check(atk, x, 1, expect="radix")
    # short rows that 64 buckets divide: several rows per workgroup
    y = workloads.gaussian(5000, 512, seed=8).to(dtype) if dtype not in (torch.int32, torch.uint32) else \
        torch.randint(0, 50, (5000, 512), dtype=torch.int32).to(dtype)
    for K in (1, 4):
        check(atk, y, K, expect="two-stage B=64")
    check(atk, y[:, :128].contiguous(), 2, smallest=True, expect="two-stage B=64")
    if dtype == torch.float32:
        check(atk, workloads.gaussian(300, 65536, seed=6), 7, expect="radix")
        knobs.set("certified", 0)
        check(atk, workloads.gaussian(5, 1 << 18, seed=7), 2, expect="radix")
