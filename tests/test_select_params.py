"""Recall-target parameter selection (Section 6.3 last paragraph; appendix "Algorithm Parameter
Selection"): the library's closed-form sweep against the oracle's exhaustive enumeration in
exact arithmetic, and against the configurations the paper names."""
import ctypes

import pytest
import torch

from oracle import oracle
from paper_2506_04165_amd import binding as atk


def test_configurations_named_in_the_paper():
    # Section 7.1: for 95 % recall of the top 1024 of 262144, K'=1 needs 16384 survivors and
    # K'=4 only 2048; Section 7.2 / Table 1: the 99 % configuration is K'=4 with 1024 buckets,
    # against 65536 buckets for K'=1.  (Bucket counts are multiples of 128 there.)
    N, K = 262144, 1024
    kp, B, _ = atk.select_params(N, K, 0.95, max_kprime=1, bucket_multiple=128)
    assert (kp, B) == (1, 16384)
    kp, B, _ = atk.select_params(N, K, 0.95, max_kprime=4, bucket_multiple=128)
    assert (kp, B) == (4, 512) and kp * B == 2048
    kp, B, r = atk.select_params(N, K, 0.99, max_kprime=4, bucket_multiple=128)
    assert (kp, B) == (4, 1024) and r >= 0.99
    kp, B, _ = atk.select_params(N, K, 0.99, max_kprime=1, bucket_multiple=128)
    assert (kp, B) == (1, 65536)


@pytest.mark.parametrize("N,K", [(4096, 32), (14336, 287), (65536, 256), (15360, 480), (6000, 100)])
@pytest.mark.parametrize("target", [0.8, 0.9, 0.95, 0.99])
@pytest.mark.parametrize("max_kp,mult", [(1, 64), (4, 64), (8, 16), (4, 128)])
def test_matches_exhaustive_enumeration(N, K, target, max_kp, mult):
    want = oracle.select_parameters(N, K, target, tuple(range(1, max_kp + 1)), mult)
    kp, B, r = atk.select_params(N, K, target, max_kp, mult)
    if want is None:
        assert (kp, B) == (K, 1) and r == 1.0        # nothing approximate qualifies: exact
        return
    assert (kp, B) == want
    assert r >= target
    assert r == pytest.approx(oracle.expected_recall(N, B, K, kp), abs=1e-9)
    # minimality: the next smaller legal bucket count for this K' misses the target (or is illegal)
    smaller = [d for d in range(mult, B, mult) if N % d == 0 and d * kp >= K and kp <= N // d]
    if smaller:
        assert oracle.expected_recall(N, smaller[-1], K, kp) < target


def test_falls_back_to_exact_and_rejects_bad_arguments():
    assert atk.select_params(4096, 32, 1.0, 1, 64)[:2] in ((1, 4096), (32, 1))
    assert atk.select_params(1000, 10, 0.99, 4, 64)[:2] == (10, 1)    # no divisor of 1000 is a multiple of 64
    import ctypes
    a, c = ctypes.c_int(0), ctypes.c_int(0)
    f = atk.lib.atk_select_params
    assert f(0, 1, 0.9, 4, 64, ctypes.byref(a), ctypes.byref(c), None) == atk.INVALID_ARG
    assert f(4096, 0, 0.9, 4, 64, ctypes.byref(a), ctypes.byref(c), None) == atk.INVALID_ARG
    assert f(4096, 32, 0.0, 4, 64, ctypes.byref(a), ctypes.byref(c), None) == atk.INVALID_ARG
    assert f(4096, 32, 1.5, 4, 64, ctypes.byref(a), ctypes.byref(c), None) == atk.INVALID_ARG
    assert f(4096, 32, 0.9, 0, 64, ctypes.byref(a), ctypes.byref(c), None) == atk.INVALID_ARG
    assert f(4096, 32, 0.9, 4, 64, None, ctypes.byref(c), None) == atk.INVALID_ARG


@pytest.mark.gpu
def test_recall_target_entry_point_runs_the_selected_configuration():
    import numpy as np
    from paper_2506_04165_amd import workloads
    for dtype, N, K, target in [(torch.float32, 65536, 256, 0.95), (torch.bfloat16, 14336, 287, 0.95),
                                (torch.float16, 14336, 287, 0.95), (torch.float32, 430080, 3360, 0.999),
                                (torch.float32, 262144, 1024, 0.99), (torch.float32, 4096, 32, 1.0)]:
        x = workloads.gaussian(6, N, seed=77, dtype=dtype)
        xd = x.to("cuda:0")
        v, i, kp, B = atk.approx_topk_recall(xd, K, target)
        torch.cuda.synchronize()
        # the library's own choice, and the ceilings it documents (every configuration runs)
        assert (kp, B) == atk.recall_params(dtype, 6, N, K, target)[:2]
        xh = workloads.to_numpy_bits(x)
        if (kp, B) == (K, 1):
            ov, oi = oracle.topk(xh, K)
        else:
            ov, oi = oracle.approx_topk(xh, K, kp, B)
        assert np.array_equal(i.cpu().numpy(), oi)
        got = v.cpu().view(torch.int16).numpy().view(np.uint16) if x.element_size() == 2 else v.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, ov.view(np.uint16) if ov.dtype.itemsize == 2 else ov.view(np.uint32))
        # the realised recall on random data is close to the target's expectation
        _, ei = oracle.topk(xh, K)
        assert oracle.index_recall(oi, ei).mean() >= target - 0.03


def test_recall_params_is_the_sweep_with_the_chips_ceilings_over_what_runs():
    # 16-bit elements get the K' <= 8 ceiling whatever the format, 32-bit ones K' <= 4.  The choice:
    # the shortest lists for which some B keeps the survivors within a sixteenth of the row (512 to
    # 4096; 1024 for short 16-bit rows), the smallest sufficient power of two as B (doubled up to 1024
    # within the budget), else the smallest sufficient divisor; nothing within that budget: the fewest survivors (atk_select_params).
    memo = {}

    def expected(dtype, N, K, target, ceiling):
        es = 2 if dtype in (torch.bfloat16, torch.float16) else 4
        if (es, N, K, target) in memo:
            return memo[(es, N, K, target)]
        budget = min(max(N // 16, 512), 4096)
        if es == 2 and N <= 65536:
            budget = min(budget, 1024)
        answer = None
        for kp in range(1, min(ceiling, K) + 1):
            first = None
            for B in range(64, budget // kp + 1, 64):
                if N % B or B * kp < K or N // B < kp or (first and B & (B - 1)):
                    continue
                if oracle.expected_recall(N, B, K, kp) >= target:
                    first = first or B
                    if B & (B - 1) == 0:
                        first = B
                        break
            if first:
                while first & (first - 1) == 0 and first < 1024 and 2 * first * kp <= budget and N % (2 * first) == 0 \
                        and N // (2 * first) >= kp:
                    first *= 2
                answer = (kp, first)
                break
        memo[(es, N, K, target)] = answer or atk.select_params(N, K, target, ceiling, 64)[:2]
        return memo[(es, N, K, target)]

    for dtype, ceiling in [(torch.float32, 4), (torch.int32, 4), (torch.uint32, 4), (torch.bfloat16, 8),
                           (torch.float16, 8)]:
        for N, K, target in [(14336, 287, 0.95), (14336, 287, 0.99), (262144, 1024, 0.99), (65536, 256, 0.9),
                             (430080, 3360, 0.95), (4096, 32, 1.0), (1 << 20, 128, 0.95), (256000, 64, 0.99),
                             (32768, 100, 0.95)]:
            got = atk.recall_params(dtype, 8, N, K, target)
            assert got[:2] == expected(dtype, N, K, target, ceiling), (dtype, N, K, target, got)
            assert got == atk.recall_params(dtype, 8, N, K, target)            # (the cached answer)
            kp, b, r = got
            if (kp, b) != (K, 1):
                assert kp <= ceiling and atk.describe_plan(dtype, 8, N, K, kp, b)[0] == atk.OK
                assert r >= target and r == pytest.approx(oracle.expected_recall(N, b, K, kp), abs=1e-9)
    # what the paper's workloads get on this chip
    assert atk.recall_params(torch.float32, 256, 1 << 20, 128, 0.95)[:2] == (1, 2048)
    assert atk.recall_params(torch.float32, 512, 256000, 64, 0.99)[:2] == (1, 3200)
    assert atk.recall_params(torch.bfloat16, 16384, 14336, 287, 0.99)[:2] == (6, 128)       # nothing within 1024 survivors
    assert atk.recall_params(torch.float32, 8, 262144, 1024, 0.99)[:2] == (4, 1024)
    # nothing approximate reaches the target and the exact kernel does not cover K either
    kp, b = ctypes.c_int(), ctypes.c_int()
    assert atk.lib.atk_recall_params(0, 8, 1 << 20, 9000, 1.0, ctypes.byref(kp), ctypes.byref(b), None) == atk.UNSUPPORTED
    assert atk.lib.atk_recall_params(9, 8, 4096, 32, 0.9, ctypes.byref(kp), ctypes.byref(b), None) == atk.UNSUPPORTED
    assert atk.lib.atk_recall_params(0, -1, 4096, 32, 0.9, ctypes.byref(kp), ctypes.byref(b), None) == atk.INVALID_ARG
    assert atk.lib.atk_recall_params(0, 8, 4096, 32, 0.0, ctypes.byref(kp), ctypes.byref(b), None) == atk.INVALID_ARG


def test_options_are_validated():
    assert atk.lib.atk_set_option(b"no_such_option", 1) == atk.INVALID_ARG
    assert atk.lib.atk_set_option(None, 1) == atk.INVALID_ARG
    assert atk.lib.atk_set_option(b"lanes_per_row", 48) == atk.INVALID_ARG      # not a power of two
    assert atk.lib.atk_set_option(b"lanes_per_row", 2048) == atk.INVALID_ARG
    before = atk.describe_plan(torch.float32, 300, 65536, 64, 2, 512)
    atk.set_option("lanes_per_row", 128)
    assert "lanes_per_row=128" in atk.describe_plan(torch.float32, 300, 65536, 64, 2, 512)[1]
    atk.set_option("lanes_per_row", -1)
    assert atk.describe_plan(torch.float32, 300, 65536, 64, 2, 512) == before


@pytest.mark.parametrize("N,K,target", [(1 << 20, 1024, 0.99), (1 << 20, 1024, 0.95), (1 << 20, 128, 0.99),
                                        (65536, 64, 0.9), (262144, 1024, 0.99), (98304, 300, 0.97),
                                        (4096, 32, 0.999)])
def test_fusion_aware_choice_matches_plain_enumeration(N, K, target):
    ref = oracle.mips_select_parameters(N, K, target)
    if ref is None:
        with pytest.raises(atk.AtkError):
            atk.mips_select_params(N, K, target)
        return
    kp, b, r = atk.mips_select_params(N, K, target)
    assert (kp, b) == ref
    assert r == pytest.approx(oracle.expected_recall(N, b, K, kp), abs=1e-9) and r >= target
    # what the rule promises: no smaller K' has any legal B that reaches the target
    for smaller in range(1, kp):
        legal = [B for B in range(32, 16384 // smaller + 1, 32)
                 if N % B == 0 and B * smaller >= K and smaller <= N // B]
        assert all(atk.expected_recall(N, B, K, smaller) < target for B in legal)


def test_fusion_aware_choice_rejects_bad_arguments():
    kp, b, r = ctypes.c_int(), ctypes.c_int(), ctypes.c_double()
    f = atk.lib.atk_mips_select_params
    assert f(0, 1, 0.9, ctypes.byref(kp), ctypes.byref(b), None) == atk.INVALID_ARG
    assert f(4096, 32, 1.5, ctypes.byref(kp), ctypes.byref(b), None) == atk.INVALID_ARG
    assert f(4096, 32, 0.9, None, ctypes.byref(b), None) == atk.INVALID_ARG
    assert f(1 << 20, 1024, 0.999999, ctypes.byref(kp), ctypes.byref(b), ctypes.byref(r)) == atk.UNSUPPORTED
