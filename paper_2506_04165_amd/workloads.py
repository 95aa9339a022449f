"""Seeded synthetic inputs for the five benchmark workloads.

This module only draws numbers and arranges them; it holds none of the
method's arithmetic (no bucketing, no selection) so both the HIP path and the
CPU oracle can be fed from it.  Everything is a function of (seed, shape,
device): a torch.Generator on the requested device is seeded explicitly.

The paper times its kernels on Gemma-2 FFN activations and on a 1M x 128-d MIPS
database (Sections 1 and 7.3); neither is available here, so inputs of the same
shape and value distribution stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    rows: int
    N: int
    dtype: torch.dtype
    K: int
    params: tuple  # ((B, K'), ...)
    note: str = ""
    extra: dict = field(default_factory=dict)


WORKLOADS = {
    "c1_tiny": Workload("c1_tiny", 4, 4096, torch.float32, 32, ((64, 4), (64, 32), (1, 32)),
                        "4 x 4096 fp32, i.i.d. N(0,1)"),
    "c2_ffn": Workload("c2_ffn", 16384, 14336, torch.bfloat16, 287, ((1024, 1), (128, 4), (64, 8)),
                       "FFN-activation sparsity: batch 8 x seqlen 2048 rows of 14336 bf16, top 2%"),
    "c3_vocab": Workload("c3_vocab", 512, 256000, torch.float32, 64, ((512, 2), (512, 4)),
                         "vocabulary logits N(0,3^2) + 64 spikes of +10 per row"),
    "c4_mips": Workload("c4_mips", 256, 1048576, torch.float32, 128, ((4096, 1), (1024, 4)),
                        "MIPS scores of unit-norm 128-d bf16 queries x database"),
    "c5_adversarial": Workload("c5_adversarial", 1024, 65536, torch.float32, 256,
                               ((256, 1), (256, 8), (256, 32)),
                               "first half: ascending rows with the top-K packed into 4 adjacent "
                               "buckets; second half: rows of 16 distinct values"),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def gaussian(rows: int, N: int, seed: int, device="cpu", dtype=torch.float32, scale: float = 1.0):
    """i.i.d. N(0, scale^2); bf16 by round-to-nearest-even of the fp32 draw."""
    x = torch.randn(rows, N, generator=_gen(seed, device), device=device, dtype=torch.float32)
    if scale != 1.0:
        x *= scale
    return x.to(dtype)


def vocab_logits(rows: int, N: int, seed: int, device="cpu", spikes: int = 64,
                 sigma: float = 3.0, boost: float = 10.0):
    """N(0, sigma^2) logits with `spikes` distinct seeded positions per row raised by `boost`."""
    g = _gen(seed, device)
    x = torch.randn(rows, N, generator=g, device=device, dtype=torch.float32) * sigma
    # distinct positions per row: the `spikes` smallest of N uniform draws
    u = torch.rand(rows, N, generator=g, device=device)
    pos = torch.topk(u, spikes, dim=1, largest=False).indices
    x.scatter_add_(1, pos, torch.full_like(pos, boost, dtype=torch.float32))
    return x


def mips_scores(rows: int, N: int, seed: int, device="cpu", dim: int = 128):
    """Inner products of unit-norm bf16-rounded queries and database vectors, fp32 accumulate.

    Computed once here; the same bytes then feed whichever implementation is
    being tested.
    """
    g = _gen(seed, device)
    q = torch.randn(rows, dim, generator=g, device=device, dtype=torch.float32)
    d = torch.randn(N, dim, generator=g, device=device, dtype=torch.float32)
    q = (q / q.norm(dim=1, keepdim=True)).to(torch.bfloat16).to(torch.float32)
    d = (d / d.norm(dim=1, keepdim=True)).to(torch.bfloat16).to(torch.float32)
    return (q @ d.t()).contiguous()


def mips_vectors(Q: int, N: int, seed: int, device="cpu", dim: int = 128, kind: str = "unit",
                 dtype=torch.bfloat16):
    """Query and database vectors for the matmul-fused entry point, as bf16 tensors [Q, dim] and
    [N, dim] (Section 7.3: one million 128-dimensional vectors, 1024 queries).

    kind "unit": Gaussian directions normalised to unit length, rounded to bf16 (inner products
    near N(0, 1/dim)).  kind "integer": entries drawn from {-2,...,2}; every product and every
    partial sum is a small integer, so the inner products are the same in any floating-point
    format and any summation order, and they tie heavily.
    """
    g = _gen(seed, device)
    if kind == "unit":
        q = torch.randn(Q, dim, generator=g, device=device, dtype=torch.float32)
        d = torch.randn(N, dim, generator=g, device=device, dtype=torch.float32)
        q = q / q.norm(dim=1, keepdim=True)
        d = d / d.norm(dim=1, keepdim=True)
    elif kind == "integer":
        q = torch.randint(-2, 3, (Q, dim), generator=g, device=device).to(torch.float32)
        d = torch.randint(-2, 3, (N, dim), generator=g, device=device).to(torch.float32)
    else:
        raise ValueError(kind)
    return q.to(dtype).contiguous(), d.to(dtype).contiguous()


def adversarial_sorted(rows: int, N: int, seed: int, device="cpu", K: int = 256, B: int = 256,
                       hot_buckets: int = 4):
    """Ascending-sorted N(0,1) rows whose K greatest values all sit in `hot_buckets` adjacent
    stride-B position classes (positions p with p mod B in [b0, b0+hot_buckets), b0 seeded per
    row), K/hot_buckets of them in each class; the other values fill the remaining positions
    in ascending order.
    """
    assert K % hot_buckets == 0 and N % B == 0 and K // hot_buckets <= N // B
    g = _gen(seed, device)
    v = torch.randn(rows, N, generator=g, device=device, dtype=torch.float32)
    v = torch.sort(v, dim=1).values
    b0 = torch.randint(0, B - hot_buckets + 1, (rows, 1), generator=g, device=device)
    per = K // hot_buckets
    j = torch.arange(per, device=device).repeat_interleave(hot_buckets)      # [K]
    c = torch.arange(hot_buckets, device=device).repeat(per)                  # [K]
    hot_pos = (b0 + c.unsqueeze(0)) + j.unsqueeze(0) * B                      # [rows, K] ascending
    is_hot = torch.zeros(rows, N, dtype=torch.bool, device=device)
    is_hot.scatter_(1, hot_pos, True)
    out = torch.empty_like(v)
    # positions in ascending order: cold first, then hot (stable argsort of the flag)
    order = torch.sort(is_hot.to(torch.uint8), dim=1, stable=True).indices    # [rows, N]
    out.scatter_(1, order, v)
    return out


def heavy_ties(rows: int, N: int, seed: int, device="cpu", symbols: int = 16):
    """Rows drawn uniformly from `symbols` distinct fp32 values."""
    g = _gen(seed, device)
    s = torch.randint(0, symbols, (rows, N), generator=g, device=device)
    return (s.to(torch.float32) - symbols / 2.0) * 0.25


def make(name: str, seed: int = 1, device="cpu", rows: int | None = None):
    """Build the input matrix of a named workload (optionally with fewer rows)."""
    w = WORKLOADS[name]
    r = w.rows if rows is None else rows
    if name == "c1_tiny":
        return gaussian(r, w.N, seed, device)
    if name == "c2_ffn":
        return gaussian(r, w.N, seed, device, dtype=torch.bfloat16)
    if name == "c3_vocab":
        return vocab_logits(r, w.N, seed, device)
    if name == "c4_mips":
        return mips_scores(r, w.N, seed, device)
    if name == "c5_adversarial":
        half = r // 2
        a = adversarial_sorted(r - half, w.N, seed, device, K=w.K, B=w.params[0][0])
        if half == 0:
            return a
        b = heavy_ties(half, w.N, seed + 1, device)
        return torch.cat([a, b], dim=0)
    raise KeyError(name)


def to_numpy_bits(x: torch.Tensor):
    """Host NumPy view for the oracle: bf16 as uint16 bit patterns, everything else as is."""
    import numpy as np
    x = x.detach().cpu().contiguous()
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16)
    if x.dtype == torch.uint32:
        return x.view(torch.int32).numpy().view(np.uint32)
    return x.numpy()
