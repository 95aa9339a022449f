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


@pytest.mark.gpu
def test_read_probe_folds_every_word_exactly_once():
    # the bandwidth-ceiling probe: exclusive-or of all 32-bit words, so a word read twice or
    # not at all shows
    from paper_2506_04165_amd import binding as atk
    rng = np.random.default_rng(4)
    for n_vec in (1, 7, 1000, 8 * 512 * 3 + 5, 2048 * 4096 + 123, (64 << 20) // 16):
        w = rng.integers(0, 2**32, size=n_vec * 4, dtype=np.uint32)
        d = torch.from_numpy(w.view(np.int32)).to("cuda:0")
        got = atk.read_probe(d)
        torch.cuda.synchronize()
        g = got.cpu().numpy().view(np.uint32)
        assert int(np.bitwise_xor.reduce(g)) == int(np.bitwise_xor.reduce(w)), n_vec
        # piece i is words [i*p, (i+1)*p) with p = ceil(n_vec / words) vectors of four words
        p = -(-n_vec // atk.READ_PROBE_WORDS) * 4
        for i in (0, 1, atk.READ_PROBE_WORDS - 1):
            assert int(g[i]) == int(np.bitwise_xor.reduce(w[i * p:(i + 1) * p], initial=np.uint32(0))), (n_vec, i)
    # accumulates into the caller's words
    acc = torch.full((atk.READ_PROBE_WORDS,), 0x5A5A, dtype=torch.int32, device="cuda:0")
    atk.read_probe(torch.zeros(64, dtype=torch.int32, device="cuda:0"), acc)
    torch.cuda.synchronize()
    assert bool((acc == 0x5A5A).all())


def test_read_probe_rejects_bad_arguments():
    from paper_2506_04165_amd import binding as atk
    f = atk.lib.atk_read_probe
    assert f(0x1000, 64, None, None) == atk.INVALID_ARG
    assert f(None, 64, 0x1000, None) == atk.INVALID_ARG
    assert f(0x1004, 64, 0x1000, None) == atk.INVALID_ARG       # data not 16-byte aligned
    assert f(0x1000, 60, 0x1000, None) == atk.INVALID_ARG       # not a multiple of 16
    assert f(0x1000, 64, 0x1002, None) == atk.INVALID_ARG
    assert f(None, 0, 0x1000, None) == atk.OK
