"""CPU-only checks of the C-ABI boundary: the library loads, exports what include/atk.h
declares, rejects bad arguments on the host (no GPU needed: validation happens before any
launch), and its host-side helpers agree with the oracle's theory."""
import ctypes
import os
import re

import pytest
import torch

from oracle import oracle
from paper_2506_04165_amd import binding as atk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x100000  # a non-null, 16-byte aligned "device pointer"; never dereferenced on error paths


def declared_functions():
    text = open(os.path.join(ROOT, "include", "atk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(atk_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 9
    for n in names:
        assert hasattr(atk.lib, n), n
    assert sorted(atk.EXPORTS) == names


def test_status_strings_and_version():
    assert atk.status_string(0) == "ATK_OK"
    assert atk.status_string(1) == "ATK_INVALID_ARG"
    assert atk.status_string(2) == "ATK_UNSUPPORTED"
    assert atk.status_string(3) == "ATK_WORKSPACE_TOO_SMALL"
    assert atk.status_string(4) == "ATK_HIP_ERROR"
    assert atk.status_string(99) == "ATK_UNKNOWN_STATUS"
    assert re.match(r"\d+\.\d+\.\d+", atk.version())


def call_approx(values=FAKE, dtype=0, rows=4, N=4096, stride=None, K=32, Kp=4, B=64,
                out_vals=FAKE, out_idx=FAKE, ws=None, ws_bytes=0):
    stride = N if stride is None else stride
    return atk.lib.atk_approx_topk(values, dtype, rows, N, stride, K, Kp, B, out_vals, out_idx,
                                   ws, ws_bytes, None)


@pytest.mark.parametrize("kw", [
    dict(values=None), dict(out_vals=None), dict(out_idx=None),
    dict(rows=-1), dict(N=0), dict(N=2**31), dict(N=2**31 - 65536 + 64), dict(stride=100),
    dict(B=0), dict(B=63),                 # B must divide N
    dict(Kp=0), dict(Kp=33),               # 1 <= K' <= K
    dict(B=1024, Kp=5, K=32),              # K' > N/B
    dict(K=300),                           # K > B*K'
    dict(K=0),
    dict(values=FAKE + 2),                 # misaligned for fp32
    dict(out_idx=FAKE + 2),
])
def test_invalid_arguments(kw):
    assert call_approx(**kw) == atk.INVALID_ARG


def test_longest_row_is_accepted():
    # 2^31 - 65536 elements (ATK_MAX_N); rows=0 validates and launches nothing
    assert call_approx(rows=0, N=2**31 - 65536, K=32, Kp=4, B=64, values=None, out_vals=None,
                       out_idx=None) == atk.OK
    st, text = atk.describe_plan(torch.float32, 1, 2**31 - 65536, 64, 1, 8192)
    assert st == atk.OK, text


def test_unsupported_arguments():
    assert call_approx(dtype=7) == atk.UNSUPPORTED
    # K' beyond the register lists (and not the K'=K case)
    assert call_approx(N=65536, K=128, Kp=40, B=64) == atk.UNSUPPORTED
    # more survivors than LDS holds go through the workspace; K beyond the exact kernel's range
    assert call_approx(N=262144, K=1024, Kp=1, B=65536) == atk.WORKSPACE_TOO_SMALL
    assert call_approx(N=262144, K=9000, Kp=1, B=65536) == atk.UNSUPPORTED
    assert call_approx(N=2 ** 26, K=100, Kp=1, B=2 ** 25) == atk.UNSUPPORTED      # B > 2^24


def test_large_bucket_counts_run_in_bucket_chunks(knobs):
    # Table 1's K'=1 rows with 32768 and 65536 buckets of 262144 elements, and neighbours: rows
    # are cut along the bucket axis; a chunk's workgroup passes on all its survivors ("unfused")
    # or, with option "chunked" and chunks that divide the buckets evenly, its K greatest
    cases = [(8, 262144, 1024, 1, 65536), (8, 262144, 1024, 1, 32768), (64, 1 << 20, 1024, 4, 16384),
             (2, 1 << 20, 5000, 4, 32768), (3, 3 * 50000, 100, 1, 50000), (1, 1 << 21, 8192, 1, 1 << 20)]
    for chunked in (0, 1):
        knobs.set("chunked", chunked)
        for rows, N, K, Kp, B in cases:
            st, text = atk.describe_plan(torch.float32, rows, N, K, Kp, B)
            route = "chunked" if (chunked and B % 1024 == 0) else "unfused"
            assert st == atk.OK and text.startswith(route), (rows, N, K, Kp, B, text)
            gy = int(re.search(r"grid=\d+x(\d+)", text).group(1))
            lanes = int(re.search(r"lanes_per_row=(\d+)", text).group(1))
            V, R = int(re.search(r" V=(\d+)", text).group(1)), int(re.search(r" R=(\d+)", text).group(1))
            assert gy == -(-B // (lanes * V * R)) and gy > 1, text
            need = atk.workspace_bytes(atk.OP_APPROX_TOPK, torch.float32, rows, N, K, Kp, B)
            assert need == (rows * B * Kp * 8 if route == "unfused" else rows * gy * K * 8)
            if route == "chunked":      # a chunk's survivors fit LDS and are a few times K
                assert 2 * K <= lanes * V * R * Kp <= 16384
    # stage 1 alone with as many buckets
    assert atk.lib.atk_approx_topk_stage1(None, 0, 0, 1 << 21, 1 << 21, 2, 1 << 20, None, None, None) == atk.OK


def test_rows_sharing_a_wavefront_stay_within_32_bit_offsets():
    # few buckets that are not a power of two and very long rows: the rows of a workgroup are
    # addressed by 32-bit byte offsets from its first row, so only so many may share it; the lanes
    # of a wavefront that this leaves without a row idle rather than wrap around
    for dtype, es in ((torch.float32, 4), (torch.bfloat16, 2)):
        for rows, N, B in [(16, 3 * 2 ** 25, 3), (5, 3 * 2 ** 25, 3), (40, 5 * 2 ** 24, 5), (7, 2 ** 30 + 2 ** 29, 3)]:
            st, text = atk.describe_plan(dtype, rows, N, 2, 2, B)
            assert st == atk.OK, text
            rpw = int(re.search(r"rows_per_wg=(\d+)", text).group(1))
            lanes = int(re.search(r"lanes_per_row=(\d+)", text).group(1))
            assert (rpw == 1 or rpw * N * es < 2 ** 31) and rpw * lanes >= 64, text


def test_rows_zero_is_ok_without_gpu():
    assert call_approx(rows=0, values=None, out_vals=None, out_idx=None) == atk.OK
    assert atk.lib.atk_topk(None, 0, 0, 128, 128, 4, None, None, None, 0, None) == atk.OK
    assert atk.lib.atk_approx_topk_stage1(None, 0, 0, 128, 128, 2, 8, None, None, None) == atk.OK


def test_topk_and_stage1_validation():
    assert atk.lib.atk_topk(FAKE, 0, 2, 128, 128, 0, FAKE, FAKE, None, 0, None) == atk.INVALID_ARG
    assert atk.lib.atk_topk(FAKE, 0, 2, 128, 128, 129, FAKE, FAKE, None, 0, None) == atk.INVALID_ARG
    assert atk.lib.atk_topk(FAKE, 0, 2, 16384, 16384, 8193, FAKE, FAKE, None, 0, None) == atk.UNSUPPORTED
    assert atk.lib.atk_topk(None, 0, 2, 128, 128, 4, FAKE, FAKE, None, 0, None) == atk.INVALID_ARG
    st1 = atk.lib.atk_approx_topk_stage1
    assert st1(FAKE, 0, 2, 128, 128, 3, 64, FAKE, FAKE, None) == atk.INVALID_ARG   # K' > N/B
    assert st1(FAKE, 0, 2, 128, 128, 1, 5, FAKE, FAKE, None) == atk.INVALID_ARG    # B does not divide N
    assert st1(FAKE, 0, 2, 128, 128, 1, 8, None, FAKE, None) == atk.INVALID_ARG


def test_workspace_query_and_too_small():
    f32 = torch.float32
    # fused cases need no workspace
    assert atk.workspace_bytes(atk.OP_APPROX_TOPK, f32, 256, 1048576, 128, 4, 1024) == 0
    # the exact entry: the flag words of the certified route where it applies, else nothing
    assert atk.workspace_bytes(atk.OP_TOPK, f32, 4, 4096, 32, 0, 0) == 512
    assert atk.describe_topk_plan(f32, 4, 4096, 32)[1].startswith("certified B=64 K'=4")
    assert atk.workspace_bytes(atk.OP_TOPK, f32, 16384, 14336, 287, 0, 0) == 0               # short rows
    assert atk.describe_topk_plan(f32, 16384, 14336, 287) == (atk.OK, "radix threads=256")
    # ... unless of 16-bit elements: the packed-key kernels, K' = 8
    assert atk.workspace_bytes(atk.OP_TOPK, torch.bfloat16, 16384, 14336, 287, 0, 0) == 2 * 16384 * 4
    assert atk.describe_topk_plan(torch.bfloat16, 16384, 14336, 287)[1].startswith("certified B=128 K'=8")
    # K' = K beyond the list lengths is the exact Top-K: the same workspace
    assert atk.workspace_bytes(atk.OP_APPROX_TOPK, f32, 4, 65536, 64, 64, 8) == \
        atk.workspace_bytes(atk.OP_TOPK, f32, 4, 65536, 64, 0, 0) > 0
    # K < 8: the two-stage kernels with K' = K, exact by construction; the workspace is what that call
    # takes (few rows: the slab route); rows too short for it stay with the radix kernel
    assert atk.describe_topk_plan(f32, 4, 65536, 4)[1].startswith("two-stage B=1024 K'=K=4")
    assert atk.workspace_bytes(atk.OP_TOPK, f32, 4, 65536, 4, 0, 0) == \
        atk.workspace_bytes(atk.OP_APPROX_TOPK, f32, 4, 65536, 4, 4, 1024) > 0
    assert atk.describe_topk_plan(f32, 100000, 512, 1)[1].startswith("two-stage B=64 K'=K=1")   # short rows: 64 buckets
    assert atk.describe_topk_plan(f32, 100000, 480, 1) == (atk.OK, "radix threads=64")           # ... when they divide
    assert atk.describe_topk_plan(f32, 300, 65536, 7) == (atk.OK, "radix threads=1024")       # many rows: lists of up to 4
    assert atk.describe_topk_plan(f32, 30, 65536, 7)[1].startswith("two-stage B=512 K'=K=7")
    assert atk.describe_topk_plan(f32, 2000, 30000, 1)[1].startswith("two-stage B=1875 K'=K=1")   # no power of two fits
    assert atk.workspace_bytes(atk.OP_TOPK, f32, 4, 1 << 20, 2048, 0, 0) == 0                # K > 1024
    # survivors beyond LDS go through memory: rows * B*K' * (4 + 4) bytes
    need = atk.workspace_bytes(atk.OP_APPROX_TOPK, f32, 8, 131072, 128, 16, 2048)
    assert need == 8 * 2048 * 16 * 8
    assert call_approx(rows=8, N=131072, K=128, Kp=16, B=2048, ws=None, ws_bytes=0) == atk.WORKSPACE_TOO_SMALL
    assert call_approx(rows=8, N=131072, K=128, Kp=16, B=2048, ws=FAKE, ws_bytes=need - 1) == atk.WORKSPACE_TOO_SMALL
    # illegal arguments
    assert atk.workspace_bytes(atk.OP_APPROX_TOPK, f32, 4, 4096, 32, 4, 63) == atk.SIZE_MAX
    assert atk.workspace_bytes(99, f32, 4, 4096, 32, 4, 64) == atk.SIZE_MAX


def test_plans_for_benchmark_configs_are_fused_single_launch():
    from paper_2506_04165_amd.workloads import WORKLOADS
    for w in WORKLOADS.values():
        for B, Kp in w.params:
            st, text = atk.describe_plan(w.dtype, w.rows, w.N, w.K, Kp, B)
            assert st == atk.OK, (w.name, B, Kp)
            assert text.startswith("fused"), (w.name, B, Kp, text)
            assert "workspace=0" in text


def test_few_long_rows_are_spread_over_workgroups(knobs):
    # 8 rows of 262144 (the shape of the paper's Table 1) cannot fill 256 CUs one row per
    # workgroup.  Such rows are given out in slabs of 32 buckets; the plan asks for a workspace
    # for the B*K' keys of every row
    st, text = atk.describe_plan(torch.float32, 8, 262144, 1024, 4, 1024)
    assert st == atk.OK and text.startswith("slab"), text
    need = atk.workspace_bytes(atk.OP_APPROX_TOPK, torch.float32, 8, 262144, 1024, 4, 1024)
    assert re.search(r"grid=8x(\d+)", text).group(1) == "32" and need == 8 * 4 * 1024 * 8
    # with that route switched off, rows are cut into segments along their length instead
    knobs.set("slab", 0)
    st, text = atk.describe_plan(torch.float32, 8, 262144, 1024, 4, 1024)
    assert st == atk.OK and text.startswith("split"), text
    need = atk.workspace_bytes(atk.OP_APPROX_TOPK, torch.float32, 8, 262144, 1024, 4, 1024)
    nseg = int(re.search(r"grid=\d+x(\d+)", text).group(1))
    assert nseg > 1 and need == 8 * nseg * 4 * 1024 * 8
    knobs.set("slab", -1)
    # many rows, short rows, few buckets or very long bucket walks go other ways
    for rows, N, B in [(256, 262144, 1024), (8, 16384, 1024), (8, 262144, 64), (8, 1048576, 512)]:
        st, text = atk.describe_plan(torch.float32, rows, N, 64, 4, B)
        assert st == atk.OK and not text.startswith("slab"), text
    # both are optimisations: without a workspace the call is still legal (validation only
    # here: rows=0 launches nothing)
    assert call_approx(rows=0, N=262144, K=1024, Kp=4, B=1024, values=None, out_vals=None,
                       out_idx=None) == atk.OK


@pytest.mark.parametrize("N,B,K,Kp", [(4096, 64, 32, 1), (4096, 64, 32, 4), (14336, 128, 287, 4),
                                      (262144, 1024, 1024, 4), (1048576, 4096, 128, 1),
                                      (65536, 256, 256, 8), (256000, 512, 64, 2), (4096, 64, 32, 32)])
def test_expected_recall_matches_exact_rational_evaluation(N, B, K, Kp):
    # the library's log-gamma evaluation of Theorem 1 against the oracle's exact fractions
    assert atk.expected_recall(N, B, K, Kp) == pytest.approx(oracle.expected_recall(N, B, K, Kp), abs=1e-9)


def test_expected_recall_rejects_bad_arguments():
    assert atk.expected_recall(4096, 63, 32, 1) < 0
    assert atk.expected_recall(0, 1, 1, 1) < 0
    assert atk.expected_recall(4096, 64, 5000, 1) < 0


def test_binding_refuses_cpu_tensors():
    x = torch.zeros(2, 128)
    with pytest.raises(ValueError):
        atk.approx_topk(x, 4, 1, 8)
    with pytest.raises(ValueError):
        atk.topk(x, 4)


def test_mips_validation_and_plan():
    m = atk.lib.atk_mips_approx_topk
    BF = 1
    ok = dict(Q=4, N=4096, D=128, K=64, Kp=2, B=64)
    def call(queries=FAKE, database=FAKE, dtype=BF, out_vals=FAKE, out_idx=FAKE, ws=FAKE, ws_bytes=1 << 30, **kw):
        a = dict(ok); a.update(kw)
        return m(queries, database, dtype, a["Q"], a["N"], a["D"], a["K"], a["Kp"], a["B"],
                 out_vals, out_idx, ws, ws_bytes, None)
    assert call(Q=0, queries=None, database=None, out_vals=None, out_idx=None, ws=None, ws_bytes=0) == atk.OK
    assert call(queries=None) == atk.INVALID_ARG
    assert call(database=FAKE + 2) == atk.INVALID_ARG
    assert call(N=4095) == atk.INVALID_ARG           # B does not divide N
    assert call(K=200) == atk.INVALID_ARG            # K > B*K'
    assert call(Kp=0) == atk.INVALID_ARG
    assert call(D=0) == atk.INVALID_ARG
    assert call(dtype=0) == atk.UNSUPPORTED          # fp32 vectors
    assert call(D=96) == atk.UNSUPPORTED
    assert call(B=16, K=16) == atk.UNSUPPORTED       # B not a multiple of 32
    assert call(Kp=5, K=64) == atk.UNSUPPORTED
    assert call(N=1 << 20, B=8192, Kp=4, K=64) == atk.UNSUPPORTED   # B*K' beyond stage 2's LDS
    need = atk.mips_workspace_bytes(4, 4096, 128, 64, 2, 64)
    assert need == 4 * 1 * 2 * 64 * 8
    assert call(ws=None, ws_bytes=0) == atk.WORKSPACE_TOO_SMALL
    assert call(ws_bytes=need - 1) == atk.WORKSPACE_TOO_SMALL
    assert atk.mips_workspace_bytes(4, 4096, 96, 64, 2, 64) == atk.SIZE_MAX
    assert atk.lib.atk_mips_workspace_bytes(2, 4, 4096, 128, 64, 2, 64) == need       # fp16 vectors
    assert atk.lib.atk_mips_workspace_bytes(3, 4, 4096, 128, 64, 2, 64) == atk.SIZE_MAX   # integers
    st, text = atk.mips_describe_plan(1024, 1 << 20, 128, 1024, 4, 1024)
    assert st == atk.OK and text.startswith("mfma32x32x16") and "workspace=67108864" in text


def test_no_alloc_entry_validates_like_the_workspace_entry():
    f = atk.lib.atk_approx_topk_noalloc
    assert f(None, 0, 4, 4096, 4096, 32, 4, 64, FAKE, FAKE, None) == atk.INVALID_ARG
    assert f(FAKE, 0, 4, 4096, 4096, 32, 4, 63, FAKE, FAKE, None) == atk.INVALID_ARG
    assert f(FAKE, 7, 4, 4096, 4096, 32, 4, 64, FAKE, FAKE, None) == atk.UNSUPPORTED
    assert f(None, 0, 0, 4096, 4096, 32, 4, 64, None, None, None) == atk.OK
    # survivors that the library's own scratch array (16 MiB) cannot hold: refused before any launch
    assert f(FAKE, 0, 45, 150000, 150000, 100, 1, 50000, FAKE, FAKE, None) == atk.WORKSPACE_TOO_SMALL


def test_planner_choices_found_by_the_sweep_for_cliffs():
    # shapes outside the benchmark set on which a plausible plan was several times slower than
    # the one now taken (measured on the GPU; here the plan itself is pinned)
    f32 = torch.float32

    def plan(*a):
        st, text = atk.describe_plan(f32, *a)
        assert st == atk.OK
        return text

    # more survivors than a wavefront sorts: one row per workgroup and a lane per eight survivors
    # (rows sharing a workgroup would end in a full LDS sort of all their candidates)
    t = plan(16384, 4096, 64, 4, 1024)
    assert "lanes_per_row=512 rows_per_wg=1 " in t and "tail=2" in t, t
    t = plan(8192, 8192, 1024, 32, 64)
    assert t.startswith("fused batched") and "rows_per_wg=1 " in t and "tail=2" in t, t
    # few long rows with few buckets: as many segments as fill the chip (a row of 64 lanes streams
    # a quarter of what 256 lanes do), up to 128
    assert "grid=2x128 " in plan(8, 1 << 24, 64, 4, 64)
    assert "grid=3x64 " in plan(12, 1 << 20, 64, 4, 64)
    # 128 rows of 1024 lanes are 2048 wavefronts on half of the CUs: cut in two
    assert plan(128, 1 << 20, 128, 4, 1024).startswith("split") and "grid=128x2 " in plan(128, 1 << 20, 128, 4, 1024)
    assert plan(200, 1 << 19, 128, 4, 1024).startswith("fused")
    # long buckets: the variants with deferred insertion
    assert plan(256, 1 << 20, 128, 4, 1024).startswith("fused deferred")
    assert plan(1024, 65536, 256, 8, 256).startswith("fused deferred")
    assert plan(512, 256000, 64, 4, 512).startswith("fused KP=4")            # 500 steps: not worth it
    assert plan(256, 1 << 20, 128, 2, 1024).startswith("fused KP=2")          # nor are lists of two
    # 16-bit rows too long for keys that hold the position: packed keys of value and step in the
    # lists, the general keys from there on; without them, deferred insertion from 256 steps
    st, text = atk.describe_plan(torch.bfloat16, 4096, 131072, 256, 4, 256)
    assert st == atk.OK and text.startswith("fused lists32"), text
    atk.set_option("packed", 0)
    try:
        st, text = atk.describe_plan(torch.bfloat16, 4096, 131072, 256, 4, 256)
        assert st == atk.OK and text.startswith("fused deferred"), text
    finally:
        atk.set_option("packed", -1)
    st, text = atk.describe_plan(torch.float16, 3, 1 << 23, 64, 4, 64)        # more than 65535 steps
    assert st == atk.OK and "lists32" not in text, text
    # few rows: stage 2 by ranking on the slab route and on survivors beyond LDS
    assert "rank_finish=32x128" in plan(8, 262144, 1024, 4, 1024)
    assert "rank_finish=32x1024" in plan(64, 1 << 20, 1024, 4, 8192) and plan(64, 1 << 20, 1024, 4, 8192).startswith("unfused")
