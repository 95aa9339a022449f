"""The vector-throughput probe kernels (appendix "Estimating peak VPU throughput") against
their NumPy definition: integer work, so bit-exact."""
import numpy as np
import pytest
import torch

from oracle import oracle


@pytest.mark.gpu
@pytest.mark.parametrize("kind", [0, 1])
def test_probe_matches_definition(kind):
    from paper_2506_04165_amd import binding as atk
    rng = np.random.default_rng(3)
    for n in (1, 255, 4097, 100003):
        x = rng.integers(0, 2**32, size=n, dtype=np.uint32)
        y = rng.integers(0, 2**32, size=n, dtype=np.uint32)
        xd = torch.from_numpy(x.view(np.int32)).to("cuda:0")
        yd = torch.from_numpy(y.view(np.int32)).to("cuda:0")
        for ops in (0, 1, 2, 3, 4, 7, 64, 129):
            got = atk.valu_probe(kind, xd, yd, ops).cpu().numpy().view(np.uint32)
            with np.errstate(over="ignore"):
                want = oracle.valu_probe(kind, x, y, ops)
            assert np.array_equal(got, want), (kind, n, ops)


def test_probe_rejects_bad_arguments():
    from paper_2506_04165_amd import binding as atk
    f = atk.lib.atk_valu_probe
    assert f(2, 0x1000, 0x1000, 0x1000, 16, 1, None) == atk.INVALID_ARG
    assert f(0, 0x1000, None, 0x1000, 16, 1, None) == atk.INVALID_ARG
    assert f(1, None, None, 0x1000, 16, 1, None) == atk.INVALID_ARG
    assert f(1, 0x1000, None, 0x1000, 16, -1, None) == atk.INVALID_ARG
    assert f(1, 0x1002, None, 0x1000, 16, 1, None) == atk.INVALID_ARG
    assert f(1, 0x1000, None, 0x1000, 0, 1, None) == atk.OK
