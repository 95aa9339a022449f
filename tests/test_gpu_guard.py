"""Guard bands and poisoned workspaces: no route writes outside its outputs or depends on what
its workspace held before the call.

Every output and the workspace are carved out of larger allocations whose margins hold a canary
pattern; the workspace interior is pre-filled with a poison pattern (all ones, then a pattern
that reads as plausible large keys, then zeros).  After the call, through the C ABI with raw
pointers, the canaries must be intact, the results must equal the oracle's bit for bit, and they
must be the same for every poison pattern.
"""

import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2506_04165_amd import workloads

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
MARGIN = 4096            # bytes of canary on each side (a multiple of every alignment asked for)
CANARY = 0xA5
POISONS = [0xFF, 0x7E, 0x00]


@pytest.fixture(scope="module")
def atk():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2506_04165_amd import binding
    return binding


class Guarded:
    """`nbytes` of device memory between two canary margins."""

    def __init__(self, nbytes: int, fill: int = 0):
        self.nbytes = int(nbytes)
        self.raw = torch.full((self.nbytes + 2 * MARGIN,), CANARY, dtype=torch.uint8, device=DEV)
        self.inner = self.raw[MARGIN:MARGIN + self.nbytes]
        self.inner.fill_(fill)
        assert self.inner.data_ptr() % 256 == 0

    @property
    def ptr(self):
        return self.inner.data_ptr() if self.nbytes else None

    def intact(self) -> bool:
        lo, hi = self.raw[:MARGIN], self.raw[MARGIN + self.nbytes:]
        return bool((lo == CANARY).all()) and bool((hi == CANARY).all())

    def view(self, dtype, shape):
        return self.inner.view(dtype).view(shape)


def raw_bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    return (t.view(torch.int16).numpy().view(np.uint16) if t.element_size() == 2
            else t.view(torch.int32).numpy().view(np.uint32))


def oracle_bits(a: np.ndarray) -> np.ndarray:
    return a.view(np.uint16) if a.dtype.itemsize == 2 else a.view(np.uint32)


def run_guarded_approx(atk, x: torch.Tensor, K, Kp, B, route, extra_ws=0):
    """x on the host.  Calls atk_approx_topk with guarded outputs and a guarded, poisoned
    workspace of exactly the size the library asks for (+extra_ws), once per poison pattern."""
    rows, N = x.shape
    code = atk._CODES[x.dtype]
    st, text = atk.describe_plan(x.dtype, rows, N, K, Kp, B)
    assert st == atk.OK and text.startswith(route), (route, text)
    need = atk.workspace_bytes(atk.OP_APPROX_TOPK, x.dtype, rows, N, K, Kp, B)
    assert need != atk.SIZE_MAX
    xin = Guarded(x.numel() * x.element_size())
    xin.inner.copy_(x.contiguous().view(torch.uint8).view(-1))
    ov, oi = oracle.approx_topk(workloads.to_numpy_bits(x), K, Kp, B)
    es = x.element_size()
    for poison in POISONS:
        gv, gi = Guarded(rows * K * es, fill=0x3C), Guarded(rows * K * 4, fill=0x3C)
        ws = Guarded(need + extra_ws, fill=poison)
        print(f"guarded {route}: rows={rows} N={N} K={K} K'={Kp} B={B} ws={need} poison={poison:#x}", flush=True)
        rc = atk.lib.atk_approx_topk(xin.ptr, code, rows, N, N, K, Kp, B, gv.ptr, gi.ptr,
                                     ws.ptr, ws.nbytes, None)
        torch.cuda.synchronize()
        assert rc == atk.OK, atk.status_string(rc)
        assert gv.intact() and gi.intact() and ws.intact() and xin.intact(), (route, poison)
        assert np.array_equal(gi.view(torch.int32, (rows, K)).cpu().numpy(), oi), (route, poison)
        assert np.array_equal(raw_bits(gv.view(x.dtype, (rows, K))), oracle_bits(ov)), (route, poison)
    # the input was not written either
    assert torch.equal(xin.inner.cpu(), x.contiguous().view(torch.uint8).view(-1))


def test_fused_route_guard_bands(atk):
    # one row per workgroup, several rows per workgroup with a ragged last one, lanes sharing buckets
    run_guarded_approx(atk, workloads.gaussian(300, 16384, seed=31), 128, 4, 1024, "fused")
    run_guarded_approx(atk, workloads.gaussian(301, 4096, seed=32), 100, 2, 512, "fused")
    run_guarded_approx(atk, workloads.gaussian(37, 8192, seed=33), 40, 4, 16, "fused")
    run_guarded_approx(atk, workloads.gaussian(1031, 2048, seed=34, dtype=torch.bfloat16), 287, 4, 128, "fused packed")
    run_guarded_approx(atk, workloads.gaussian(260, 65536, seed=35), 256, 32, 256, "fused")
    # (half as many rows leave CUs idle: every row is cut in two)
    run_guarded_approx(atk, workloads.gaussian(129, 65536, seed=35), 256, 32, 256, "split batched")
    g = torch.Generator().manual_seed(36)
    run_guarded_approx(atk, torch.randint(-99, 99, (65, 6000), generator=g, dtype=torch.int32), 77, 3, 125, "fused")


def test_slab_and_split_routes_guard_bands_and_poisoned_workspace(atk, knobs):
    x = workloads.gaussian(8, 262144, seed=37)
    run_guarded_approx(atk, x, 1024, 4, 1024, "slab")
    run_guarded_approx(atk, x, 1024, 2, 4096, "slab")
    run_guarded_approx(atk, workloads.gaussian(3, 65536, seed=38, dtype=torch.bfloat16), 500, 6, 1024, "slab")
    knobs.set("slab", 0)
    run_guarded_approx(atk, x, 1024, 4, 1024, "split")
    # a segment count that leaves the last segment short, and segments shorter than K' steps
    knobs.set("segments", 7)
    run_guarded_approx(atk, workloads.gaussian(5, 40 * 512, seed=39), 600, 8, 512, "split")
    knobs.set("segments", 20)
    run_guarded_approx(atk, workloads.heavy_ties(2, 40 * 256, seed=40, symbols=3), 256, 4, 256, "split")


@pytest.mark.parametrize("route", ["chunked", "unfused"])
def test_workspace_routes_for_survivors_beyond_lds_guard_bands_and_poison(atk, knobs, route):
    if route == "chunked":
        knobs.set("chunked", 1)
    run_guarded_approx(atk, workloads.gaussian(4, 131072, seed=41), 300, 16, 2048, route)
    # zeros of both signs among the survivors (their stored bits come from the row)
    z = workloads.heavy_ties(3, 131072, seed=42, symbols=3)
    z[z == z.max()] = 0.0
    z[:, ::7] = -0.0
    run_guarded_approx(atk, z, 2048, 16, 2048, route)
    g = torch.Generator().manual_seed(43)
    run_guarded_approx(atk, torch.randint(-3, 3, (3, 98304), generator=g, dtype=torch.int32), 1000, 12, 2048, route)
    # a bucket count that chunks do not divide evenly: all survivors through the workspace either way
    run_guarded_approx(atk, workloads.gaussian(3, 150000, seed=44), 100, 1, 50000, "unfused")


def test_exact_and_stage1_guard_bands(atk):
    for x, K in [(workloads.gaussian(33, 50000, seed=44), 2048), (workloads.gaussian(70, 1000, seed=45, dtype=torch.bfloat16), 999),
                 (workloads.heavy_ties(5, 70001, seed=46, symbols=2), 100)]:
        rows, N = x.shape
        es = x.element_size()
        gv, gi = Guarded(rows * K * es, fill=0x3C), Guarded(rows * K * 4, fill=0x3C)
        xd = x.to(DEV)
        rc = atk.lib.atk_topk(xd.data_ptr(), atk._CODES[x.dtype], rows, N, N, K, gv.ptr, gi.ptr, None, 0, None)
        torch.cuda.synchronize()
        assert rc == atk.OK and gv.intact() and gi.intact()
        ov, oi = oracle.topk(workloads.to_numpy_bits(x), K)
        assert np.array_equal(gi.view(torch.int32, (rows, K)).cpu().numpy(), oi)
        assert np.array_equal(raw_bits(gv.view(x.dtype, (rows, K))), oracle_bits(ov))
    for x, Kp, B in [(workloads.gaussian(9, 16384, seed=47), 4, 1024), (workloads.gaussian(9, 16384, seed=48), 3, 16),
                     (workloads.gaussian(5, 14336, seed=49, dtype=torch.bfloat16), 8, 64)]:
        rows, N = x.shape
        es = x.element_size()
        sv, si = Guarded(rows * Kp * B * es, fill=0x3C), Guarded(rows * Kp * B * 4, fill=0x3C)
        xd = x.to(DEV)
        rc = atk.lib.atk_approx_topk_stage1(xd.data_ptr(), atk._CODES[x.dtype], rows, N, N, Kp, B, sv.ptr, si.ptr, None)
        torch.cuda.synchronize()
        assert rc == atk.OK and sv.intact() and si.intact()
        ov, oi = oracle.stage1(workloads.to_numpy_bits(x), Kp, B)
        assert np.array_equal(si.view(torch.int32, (rows, Kp, B)).cpu().numpy(), oi)
        assert np.array_equal(raw_bits(sv.view(x.dtype, (rows, Kp, B))), oracle_bits(ov))


def test_fused_inner_product_entry_guard_bands_and_poisoned_workspace(atk):
    # integer-valued vectors: scores are exact whatever the summation order, so the comparison
    # with the oracle is bit for bit; 100 queries leave the last query tile ragged
    for (Q, N, D, K, Kp, B) in [(100, 16384, 128, 200, 2, 256), (33, 8192, 64, 64, 4, 64), (130, 32768, 256, 500, 1, 1024)]:
        q, d = workloads.mips_vectors(Q, N, seed=50 + Kp, dim=D, kind="integer")
        ov, oi = oracle.mips_approx_topk(workloads.to_numpy_bits(q), workloads.to_numpy_bits(d), K, Kp, B)
        need = atk.mips_workspace_bytes(Q, N, D, K, Kp, B)
        assert need != atk.SIZE_MAX and need > 0
        qd, dd = q.to(DEV), d.to(DEV)
        for poison in POISONS:
            gv, gi = Guarded(Q * K * 4, fill=0x3C), Guarded(Q * K * 4, fill=0x3C)
            ws = Guarded(need, fill=poison)
            print(f"guarded mips: Q={Q} N={N} D={D} K={K} K'={Kp} B={B} poison={poison:#x}", flush=True)
            rc = atk.lib.atk_mips_approx_topk(qd.data_ptr(), dd.data_ptr(), atk.BF16, Q, N, D, K, Kp, B,
                                              gv.ptr, gi.ptr, ws.ptr, ws.nbytes, None)
            torch.cuda.synchronize()
            assert rc == atk.OK, atk.status_string(rc)
            assert gv.intact() and gi.intact() and ws.intact()
            assert np.array_equal(gi.view(torch.int32, (Q, K)).cpu().numpy(), oi)
            assert np.array_equal(raw_bits(gv.view(torch.float32, (Q, K))), ov.view(np.uint32))
