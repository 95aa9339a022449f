"""Measure the vector-ALU throughput and the memory/compute ridge point of the GPU.

    python -m paper_2506_04165_amd.ridge [--words 268435456]

The method is the paper's (appendix "Estimating peak VPU throughput"): time two streaming
kernels for a growing number of dependent integer operations per element, fit a line to the
compute-bound region (time = ops / throughput + overhead); the inverse slope is the vector
throughput gamma, and gamma / (beta / 4) the number of vector operations that fit under one
4-byte element at the measured streaming bandwidth beta (Section 2.3).  Prints a small table
and one JSON line.
"""
import argparse
import json

import torch

from . import binding as atk


def time_ms(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b))
    return sorted(ts)[len(ts) // 2]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--words", type=int, default=1 << 28, help="int32 words per array (default 1 GiB)")
    args = ap.parse_args()
    n = args.words
    x = torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device="cuda:0")
    y = torch.randint(-2**31, 2**31 - 1, (n,), dtype=torch.int32, device="cuda:0")
    out = torch.empty_like(x)
    results = {}
    for kind, name, words_moved in ((0, "fibonacci (adds)", 3), (1, "squaring (muls)", 2)):
        rows = []
        for ops in (0, 4, 8, 16, 32, 64, 96, 128, 192, 256, 384, 512):
            ms = time_ms(lambda: atk.valu_probe(kind, x, y, ops, out=out))
            rows.append((ops, ms))
        # memory-bound plateau = the fastest times; compute-bound region = the last four points
        flat = min(ms for _, ms in rows)
        tail = rows[-4:]
        n_pts = len(tail)
        sx = sum(o for o, _ in tail); sy = sum(m for _, m in tail)
        sxx = sum(o * o for o, _ in tail); sxy = sum(o * m for o, m in tail)
        slope = (n_pts * sxy - sx * sy) / (n_pts * sxx - sx * sx)        # ms per op
        gamma = n / (slope * 1e-3)                                        # lane-ops per second
        beta = words_moved * 4 * n / (flat * 1e-3)                        # bytes per second
        results[name] = {"rows": rows, "plateau_ms": flat, "bandwidth_GBps": beta / 1e9,
                         "lane_ops_per_s": gamma, "ops_per_4_bytes": gamma / (beta / 4)}
        print(f"{name}: n = {n} words")
        for ops, ms in rows:
            print(f"  ops/element {ops:4d}   {ms:8.3f} ms")
        print(f"  plateau {flat:.3f} ms -> {beta / 1e9:.0f} GB/s moved;  slope {slope * 1e3:.3f} us/op -> "
              f"{gamma / 1e12:.1f} T lane-ops/s;  ridge {gamma / (beta / 4):.1f} ops per 4 bytes")
    print(json.dumps({"probe": "valu_ridge", "words": n,
                      "results": {k: {kk: vv for kk, vv in v.items() if kk != "rows"} for k, v in results.items()}}))


if __name__ == "__main__":
    main()
