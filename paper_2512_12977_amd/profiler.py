"""Layer-wise sensitivity scores S_i(r) (Sec. 3.2 and Sec. 4.1, Eq. 5) measured with the library's
own kernels: host orchestration only - every layer pass, the output scores and the squared error
run in libvlcache.so.

Procedure per sample (the three phases of Sec. 3.2):
  1. full prefill of the prompt the image was cached under; its image K/V per layer are the cache;
  2. full prefill of the evaluated prompt gives the reference scores of the answer rows;
  3. for every layer i and grid step k: a pass that computes every slot in every layer while the
     attention sees the cached image K/V (re-rotated by the position delta) in all layers, except
     the leading floor(k T / 500) tokens of each image in layer i, which keep their fresh k, v
     (rows with a negative slot entry are computed but not stored); mean squared error of the
     answer rows' scores against the reference.
The table this returns is what vlc_plan_layer_rates_blocks consumes (a measured table has a flat first layer, from
which the one-step greedy vlc_plan_layer_rates cannot start: it returns the all-zero plan).
"""
from __future__ import annotations

from typing import Sequence

import numpy as np
import torch

from . import binding as B
from . import runner as R


class _Prompt:
    """Index arrays of one prompt with every slot recomputed (host planner), on the device."""

    def __init__(self, request, device):
        self.segs = R.segments_of([request])
        self.S = request.S
        host = B.vlc_plan_token_indices(self.segs, 1, k=np.full(1, 500, dtype=np.int32))
        assert int(host["n_rows"][0]) == self.S
        self.slot_host = host["slot"][0, :self.S].copy()
        self.dev = {name: torch.from_numpy(host[name][0, :self.S].copy()).to(device)
                    for name in ("slot", "map", "pos", "kv_start", "kv_len")}
        self.device = device

    def plan(self, k_pool=None, v_pool=None, k_steps: int = 500) -> tuple:
        """(LayerPlan, tensors to keep alive): every slot a row; image tokens beyond the leading
        floor(k_steps T / 500) of each image take their K/V from the pool and do not store fresh ones."""
        d = dict(self.dev)
        n_reuse = 0
        keep = []
        if k_pool is not None and k_steps < 500:
            reuse = B.vlc_plan_reuse_rows(self.segs, 1, k=np.full(1, k_steps, dtype=np.int32))
            n_reuse = int(reuse["n_reuse"][0])
            slot = self.slot_host.copy()
            slot[reuse["dst_slot"][0, :n_reuse]] = -1          # slots of a single request are 0 .. S-1
            d["slot"] = torch.from_numpy(slot).to(self.device)
            for name in ("src_row", "dst_slot", "delta"):
                d[name] = torch.from_numpy(reuse[name][0, :n_reuse].copy()).to(self.device)
        p = lambda t: t.data_ptr() if t is not None and t.numel() else None
        rec = B.LayerPlan(self.S, self.S, p(d["map"]), p(d["slot"]), p(d["pos"]), p(d["kv_start"]), p(d["kv_len"]),
                          self.S, n_reuse, p(d.get("src_row")), p(d.get("dst_slot")), p(d.get("delta")),
                          p(k_pool) if n_reuse else None, p(v_pool) if n_reuse else None,
                          k_pool.shape[0] if n_reuse else 0, None)
        keep.append(d)
        return rec, keep


def sensitivity_profile(shape, weights: Sequence[R.DeviceWeights], w_norm_f, w_lm, samples: Sequence[dict],
                        steps: Sequence[int], device="cuda") -> np.ndarray:
    """S [L, len(steps)] (float64, host).  shape: a vlc_synth-style shape description; weights: one
    DeviceWeights per layer; w_norm_f [H], w_lm [vocab, H]: device tensors of the layer dtype; samples:
    dicts with cache_request, cache_emb, request, emb, answer_rows (1-D positions); steps: rates k/500."""
    L = len(weights)
    dt = R.torch_dtype(shape.dtype)
    rec = R.make_shape(shape)
    code = B.VLC_BF16 if shape.dtype == "bf16" else B.VLC_F32
    out = np.zeros((L, len(steps)), dtype=np.float64)
    mse_ws = torch.empty(B.vlc_mean_squared_error_workspace_bytes(), dtype=torch.uint8, device=device)
    for smp in samples:
        creq, req = smp["cache_request"], smp["request"]
        S_max = max(creq.S, req.S)
        ws = R.Workspace(rec, S_max, device)
        hbuf = [torch.empty((S_max, shape.H), device=device, dtype=dt) for _ in range(2)]

        def forward(prompt, emb, plans, kc, vc):
            h_in = emb
            for l in range(L):
                h_out = hbuf[l & 1][:prompt.S]
                R.run_layer(rec, weights[l], plans[l][0], h_in, h_out, kc[l], vc[l], ws)
                h_in = h_out
            return h_in

        def caches(S):
            return ([torch.zeros((S, shape.Hkv, shape.D), device=device, dtype=dt) for _ in range(L)],
                    [torch.zeros((S, shape.Hkv, shape.D), device=device, dtype=dt) for _ in range(L)])

        # phase 1: the cache
        cp = _Prompt(creq, device)
        ckc, cvc = caches(creq.S)
        forward(cp, torch.from_numpy(np.asarray(smp["cache_emb"], dtype=np.float32)).to(device).to(dt),
                [cp.plan() for _ in range(L)], ckc, cvc)
        img = np.concatenate([g.start + np.arange(g.length) for g in creq.segments if g.is_image])
        img_t = torch.from_numpy(img).to(device)
        kpool = [ckc[l][img_t].contiguous() for l in range(L)]
        vpool = [cvc[l][img_t].contiguous() for l in range(L)]
        # phase 2: reference scores of the answer rows
        ep = _Prompt(req, device)
        emb = torch.from_numpy(np.asarray(smp["emb"], dtype=np.float32)).to(device).to(dt)
        rows = torch.from_numpy(np.asarray(smp["answer_rows"], dtype=np.int32)).to(device)
        m, vocab = rows.numel(), w_lm.shape[0]
        ft_ws = torch.empty(max(256, B.vlc_first_token_workspace_bytes(shape.H, m, code)), dtype=torch.uint8, device=device)
        z_orig = torch.empty((m, vocab), device=device, dtype=torch.float32)
        z = torch.empty_like(z_orig)
        tok = torch.empty((m,), device=device, dtype=torch.int32)
        kc, vc = caches(req.S)
        h = forward(ep, emb, [ep.plan() for _ in range(L)], kc, vc)
        B.vlc_first_token(h, rows, shape.eps, w_norm_f, w_lm, z_orig, tok, ft_ws)
        # phase 3: one pass per (layer, rate)
        err = torch.zeros((L, len(steps)), device=device, dtype=torch.float64)
        pure = [ep.plan(kpool[l], vpool[l], 0) for l in range(L)]
        for i in range(L):
            for j, k in enumerate(steps):
                plans = list(pure)
                plans[i] = ep.plan(kpool[i], vpool[i], int(k))
                h = forward(ep, emb, plans, kc, vc)
                B.vlc_first_token(h, rows, shape.eps, w_norm_f, w_lm, z, tok, ft_ws)
                B.vlc_mean_squared_error(z, z_orig, err[i, j:j + 1], mse_ws)
                torch.cuda.synchronize()      # plans[i]'s index tensors are freed on the next iteration
        out += err.cpu().numpy()
    return out / max(len(samples), 1)


def main() -> int:
    """python -m paper_2512_12977_amd.profiler: the table of a synthetic sample at a named shape, the time
    one (layer, rate) pass takes, and the rates the planner derives from it.  One JSON line."""
    import argparse
    import json
    import time

    import vlc_synth as syn

    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="7b")
    ap.add_argument("--layers", type=int, default=4, help="layers of the synthetic stack (a full table costs L x steps passes)")
    ap.add_argument("--text", type=int, default=64)
    ap.add_argument("--cache-text", type=int, default=96)
    ap.add_argument("--image", type=int, default=1024)
    ap.add_argument("--answer", type=int, default=16)
    ap.add_argument("--steps", default="0,10,25,50,100,150")
    ap.add_argument("--budget-bp", type=int, default=500, help="mean rate in basis points for the derived plan")
    args = ap.parse_args()
    import dataclasses
    shape = dataclasses.replace(syn.SHAPES[args.shape], L=args.layers, vocab=min(syn.SHAPES[args.shape].vocab, 32768))
    if shape.mrope_section:
        raise SystemExit("the measurement uses 1-D positions; pick a shape without 3-axis RoPE")
    dt = R.torch_dtype(shape.dtype)
    dev = "cuda"
    weights = [R.DeviceWeights.random(shape, dt, 1000 + l) for l in range(args.layers)]
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    w_norm = (1.0 + 0.02 * torch.randn(shape.H, generator=g, device=dev)).to(dt)
    w_lm = (0.02 * torch.randn((shape.vocab, shape.H), generator=g, device=dev)).to(dt)
    smp = syn.profile_sample(shape, 7, args.cache_text, args.text, args.image, args.answer)
    steps = [int(v) for v in args.steps.split(",")]
    sensitivity_profile(shape, weights, w_norm, w_lm, [smp], steps[:1])        # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    S = sensitivity_profile(shape, weights, w_norm, w_lm, [smp], steps)
    dt_s = time.perf_counter() - t0
    passes = args.layers * len(steps) + 2
    # the planner wants every grid column 0..G; columns between the measured steps are interpolated
    G = max(steps)
    table = np.stack([np.interp(np.arange(G + 1), steps, S[i]) for i in range(args.layers)])
    budget = B.vlc_plan_budget_steps(args.budget_bp, args.layers)
    plan = B.vlc_plan_layer_rates(table, budget)
    plan_runs = B.vlc_plan_layer_rates_blocks(table, budget)   # the first layer's scores are flat: it has to be carried
    print(json.dumps({"shape": args.shape, "layers": args.layers, "slots": smp["request"].S, "steps": steps,
                      "S": [[float("%.6g" % v) for v in row] for row in S], "passes": passes,
                      "ms_per_pass": round(dt_s * 1e3 / passes, 3), "budget_steps": budget,
                      "plan": [int(v) for v in plan_runs], "planner": "vlc_plan_layer_rates_blocks",
                      "plan_one_step_greedy_for_comparison": [int(v) for v in plan]}))
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
