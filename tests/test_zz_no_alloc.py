"""The entry point that allocates nothing (atk_approx_topk_noalloc) against atk_approx_topk,
through the C ABI: same bits, on two calls in a row of which the second has the smaller input,
for every route that uses the library's scratch array in place of a workspace."""
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


def both(atk, x, K, Kp, B, route):
    """Runs the problem through both entry points with raw pointers; returns the no-alloc result."""
    rows, N = x.shape
    code = atk._CODES[x.dtype]
    st, text = atk.describe_plan(x.dtype, rows, N, K, Kp, B)
    assert st == atk.OK and (route is None or text.startswith(route)), (route, text)
    xd = x.to(DEV)
    need = atk.workspace_bytes(atk.OP_APPROX_TOPK, x.dtype, rows, N, K, Kp, B)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device=DEV)
    ref_v = torch.empty((rows, K), dtype=x.dtype, device=DEV)
    ref_i = torch.empty((rows, K), dtype=torch.int32, device=DEV)
    got_v, got_i = torch.zeros_like(ref_v), torch.zeros_like(ref_i)
    print(f"no-alloc {route}: rows={rows} N={N} K={K} K'={Kp} B={B} dtype={x.dtype}", flush=True)
    rc = atk.lib.atk_approx_topk(xd.data_ptr(), code, rows, N, N, K, Kp, B, ref_v.data_ptr(), ref_i.data_ptr(),
                                 ws.data_ptr(), need, None)
    assert rc == atk.OK, atk.status_string(rc)
    rc = atk.lib.atk_approx_topk_noalloc(xd.data_ptr(), code, rows, N, N, K, Kp, B, got_v.data_ptr(),
                                         got_i.data_ptr(), None)
    assert rc == atk.OK, atk.status_string(rc)
    torch.cuda.synchronize()
    assert torch.equal(got_i, ref_i), route
    nbits = torch.int16 if x.element_size() == 2 else torch.int32
    assert torch.equal(got_v.view(nbits), ref_v.view(nbits)), route
    return got_v, got_i


@pytest.mark.parametrize("route,first,second", [
    # (rows, N, K, K', B): the second call is the smaller problem and finds the first one's keys in the array
    ("slab", (8, 262144, 1024, 4, 1024), (3, 65536, 500, 2, 1024)),
    ("split", (8, 262144, 1024, 4, 1024), (6, 262144, 300, 4, 512)),
    ("chunked", (6, 131072, 300, 16, 2048), (2, 65536, 2000, 1, 32768)),
    ("unfused", (6, 131072, 300, 16, 2048), (2, 65536, 2000, 1, 32768)),
    ("fused", (300, 16384, 128, 4, 1024), (7, 4096, 32, 4, 64)),
])
def test_no_alloc_entry_matches_the_workspace_entry_on_two_calls_in_a_row(atk, knobs, route, first, second):
    if route == "split":
        knobs.set("slab", 0)
    if route == "chunked":
        knobs.set("chunked", 1)
    for call, (rows, N, K, Kp, B) in enumerate((first, second)):
        x = workloads.gaussian(rows, N, seed=90 + call)
        gv, gi = both(atk, x, K, Kp, B, route)
        if call == 1:       # and once against the oracle
            ov, oi = oracle.approx_topk(workloads.to_numpy_bits(x), K, Kp, B)
            assert np.array_equal(gi.cpu().numpy(), oi)
            assert np.array_equal(gv.cpu().numpy().view(np.uint32), ov.view(np.uint32))
    # 16-bit elements and heavy ties through the same array, smaller again
    z = workloads.heavy_ties(2, 65536, seed=93, symbols=3).to(torch.bfloat16)
    both(atk, z, 256, 4, 1024, None)


def test_no_alloc_entry_refuses_what_the_array_cannot_hold(atk):
    # 50000 buckets (chunks cannot divide them evenly, so all survivors go through the array):
    # 40 rows x 50000 survivors x 8 bytes = 16.0 MB fit, 45 rows do not
    x = workloads.gaussian(45, 150000, seed=94).to(DEV)
    out_v = torch.empty((45, 100), device=DEV)
    out_i = torch.empty((45, 100), dtype=torch.int32, device=DEV)
    rc = atk.lib.atk_approx_topk_noalloc(x.data_ptr(), 0, 45, 150000, 150000, 100, 1, 50000, out_v.data_ptr(),
                                         out_i.data_ptr(), None)
    assert rc == atk.WORKSPACE_TOO_SMALL
    gv, gi = atk.approx_topk_noalloc(x[:40], 100, 1, 50000, (out_v[:40], out_i[:40]))
    rv, ri = atk.approx_topk(x[:40], 100, 1, 50000)
    torch.cuda.synchronize()
    assert torch.equal(gi, ri) and torch.equal(gv, rv)
