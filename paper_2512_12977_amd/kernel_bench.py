"""Stand-alone timings of the HBM-bound C-ABI kernels at the sizes of the long-context batch
(7B-shaped K/V rows of 1 KB, 8 requests x 18432 slots): achieved GB/s against the 8 TB/s peak.

    python -m paper_2512_12977_amd.kernel_bench [--iters 20]

Prints one JSON object per kernel.  Algorithmic bytes: gather 2*H*e per row; scatter 4*Hkv*D*e per
row (K and V, read + write); RoPE shift 4*Hkv*D*e per reused token.
"""
from __future__ import annotations

import argparse
import json

import torch

from . import binding as B

PEAK_GBS = 8000.0


def timed(fn, iters):
    for _ in range(3):
        fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e-3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=20)
    args = ap.parse_args()
    dev, dt = "cuda", torch.bfloat16
    g = torch.Generator(device=dev)
    g.manual_seed(0)
    Hkv, D, H = 4, 128, 3584
    slots, pool = 8 * 18432, 8 * 16384
    out = []
    # RoPE shift: every reused image token of the batch (8 x 16064) from a pool into the packed cache
    n_tok = 8 * 16064
    kp = torch.randn((pool, Hkv, D), device=dev, generator=g).to(dt)
    vp = torch.randn((pool, Hkv, D), device=dev, generator=g).to(dt)
    kc = torch.zeros((slots, Hkv, D), device=dev, dtype=dt)
    vc = torch.zeros((slots, Hkv, D), device=dev, dtype=dt)
    src = torch.randperm(pool, device=dev, generator=g)[:n_tok].sort().values.to(torch.int32)
    dst = torch.randperm(slots, device=dev, generator=g)[:n_tok].sort().values.to(torch.int32)
    delta = torch.randint(-20000, 20000, (n_tok,), device=dev, generator=g, dtype=torch.int32)
    t = timed(lambda: B.vlc_rope_shift_kv(kp, vp, kc, vc, src, dst, delta, 1e6), args.iters)
    by = n_tok * 4.0 * Hkv * D * 2
    out.append({"kernel": "vlc_rope_shift_kv", "tokens": n_tok, "us": t * 1e6, "GB/s": by / t / 1e9})
    # gather: 18944 recomputed rows out of 147456 hidden rows
    n = 18944
    h = torch.randn((slots, H), device=dev, generator=g).to(dt)
    idx = torch.randperm(slots, device=dev, generator=g)[:n].sort().values.to(torch.int32)
    x = torch.empty((n, H), device=dev, dtype=dt)
    t = timed(lambda: B.vlc_gather_rows(h, idx, x), args.iters)
    by = n * 2.0 * H * 2
    out.append({"kernel": "vlc_gather_rows", "rows": n, "us": t * 1e6, "GB/s": by / t / 1e9})
    # a gather large enough to leave the launch-latency regime: all 147456 rows, permuted
    idx2 = torch.randperm(slots, device=dev, generator=g).to(torch.int32)
    x2 = torch.empty((slots, H), device=dev, dtype=dt)
    t = timed(lambda: B.vlc_gather_rows(h, idx2, x2), args.iters)
    by = slots * 2.0 * H * 2
    out.append({"kernel": "vlc_gather_rows (all rows permuted)", "rows": slots, "us": t * 1e6, "GB/s": by / t / 1e9})
    # scatter: fresh K/V of the 18944 rows into the packed cache
    kn = torch.randn((n, Hkv, D), device=dev, generator=g).to(dt)
    vn = torch.randn((n, Hkv, D), device=dev, generator=g).to(dt)
    t = timed(lambda: B.vlc_scatter_kv(kn, vn, idx, kc, vc), args.iters)
    by = n * 4.0 * Hkv * D * 2
    out.append({"kernel": "vlc_scatter_kv", "rows": n, "us": t * 1e6, "GB/s": by / t / 1e9})
    idx3 = torch.randperm(slots, device=dev, generator=g).to(torch.int32)
    kn3 = torch.randn((slots, Hkv, D), device=dev, generator=g).to(dt)
    t = timed(lambda: B.vlc_scatter_kv(kn3, kn3, idx3, kc, vc), args.iters)
    by = slots * 4.0 * Hkv * D * 2
    out.append({"kernel": "vlc_scatter_kv (all slots permuted)", "rows": slots, "us": t * 1e6, "GB/s": by / t / 1e9})
    for o in out:
        o["frac_of_8TBs"] = round(o["GB/s"] / PEAK_GBS, 4)
        o["us"] = round(o["us"], 2)
        o["GB/s"] = round(o["GB/s"], 1)
        print(json.dumps(o))


if __name__ == "__main__":
    main()
