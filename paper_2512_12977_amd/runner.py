"""Host-side driver around the C ABI: uploads tensors, builds per-layer plans with the library's
own planner, and calls vlc_layer_forward layer by layer.  No arithmetic of the method lives here."""
from __future__ import annotations

import ctypes as C
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def torch_dtype(name: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def make_shape(sh) -> B.LayerShape:
    """sh: any object with H, Hq, Hkv, D, I, dtype ('f32'|'bf16'), eps, rope_base."""
    sec = tuple(getattr(sh, "mrope_section", ())) or (0, 0, 0)
    return B.LayerShape(sh.H, sh.Hq, sh.Hkv, sh.D, sh.I, B.VLC_BF16 if sh.dtype == "bf16" else B.VLC_F32,
                        float(sh.eps), float(sh.rope_base), int(sec[0]), int(sec[1]), int(sec[2]),
                        int(getattr(sh, "n_experts", 0)), int(getattr(sh, "top_k", 0)))


def segments_of(requests: Sequence) -> List[B.Segment]:
    """Flatten requests (with .segments, .kv_start, .pos_start) into the ABI's segment records."""
    out = []
    for r in requests:
        p3 = getattr(r, "pos3", None)
        for s in r.segments:
            # with 3-axis ids the segment's position is its first temporal id: an image's tokens share it,
            # so new - old is the shift of every axis of every token (the planner's reuse delta)
            pos = int(p3[s.start, 0]) if p3 is not None else r.pos_start + s.start
            out.append(B.Segment(r.kv_start + s.start, s.length, int(s.is_image), pos, s.old_pos, s.cache_row,
                                 r.kv_start))
    return out


_WEIGHT_FIELDS = ("w_ln1", "w_qkv", "b_qkv", "w_o", "w_ln2", "w_gate_up", "w_down", "w_qnorm", "w_knorm", "w_router")


class DeviceWeights:
    """One layer's weights on the GPU plus the pointer record the ABI takes."""

    def __init__(self, W: Dict[str, Optional[np.ndarray]], dtype, device="cuda"):
        self.t = {}
        for name, a in W.items():
            self.t[name] = None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dtype)
        self.rec = B.LayerWeights(*[None if self.t.get(n) is None else self.t[n].data_ptr() for n in _WEIGHT_FIELDS])

    @classmethod
    def random(cls, sh, dtype, seed: int, device="cuda") -> "DeviceWeights":
        """Random-init weights generated on the device (throughput runs; values do not affect timing)."""
        g = torch.Generator(device=device)
        g.manual_seed(seed)
        self = cls.__new__(cls)
        nq = (sh.Hq + 2 * sh.Hkv) * sh.D
        sizes = {"w_ln1": (sh.H,), "w_qkv": (nq, sh.H), "b_qkv": (nq,), "w_o": (sh.H, sh.Hq * sh.D),
                 "w_ln2": (sh.H,), "w_gate_up": (2 * sh.I, sh.H), "w_down": (sh.H, sh.I)}
        E = getattr(sh, "n_experts", 0)
        if E:
            sizes.update({"w_gate_up": (E, 2 * sh.I, sh.H), "w_down": (E, sh.H, sh.I), "w_router": (E, sh.H)})
        self.t = {}
        for name, size in sizes.items():
            if name == "b_qkv" and not sh.qkv_bias:
                self.t[name] = None
                continue
            w = torch.randn(size, generator=g, device=device, dtype=torch.float32)
            w *= getattr(sh, "residual_proj_scale", 0.02) if name in ("w_o", "w_down") else 0.02
            if name in ("w_ln1", "w_ln2"):
                w += 1.0
            self.t[name] = w.to(dtype)
        if getattr(sh, "qk_norm", False):
            for name in ("w_qnorm", "w_knorm"):
                self.t[name] = (1.0 + 0.02 * torch.randn((sh.D,), generator=g, device=device, dtype=torch.float32)).to(dtype)
        self.rec = B.LayerWeights(*[None if self.t.get(n) is None else self.t[n].data_ptr() for n in _WEIGHT_FIELDS])
        return self


class DevicePlans:
    """Per-layer index arrays on the GPU, built by the library's host planner."""

    def __init__(self, requests: Sequence, L: int, k=None, count_override=None, all_rows: bool = False,
                 device="cuda"):
        segs = segments_of(requests)
        if all_rows:   # full recompute: rate 1.0 in every layer, nothing reused
            k, count_override = np.full(L, 500, dtype=np.int32), None
        self.host = B.vlc_plan_token_indices(segs, L, k=k, count_override=count_override)
        self.reuse = B.vlc_plan_reuse_rows(segs, L, k=k, count_override=count_override)
        self.next_row = B.vlc_plan_next_rows(segs, L, k=k, count_override=count_override)
        self.L = L
        self.total_slots = sum(s.length for s in segs)
        self.n_rows = [int(v) for v in self.host["n_rows"]]
        self.n_reuse = [int(v) for v in self.reuse["n_reuse"]]
        self.dev = []
        for l in range(L):
            n, m = self.n_rows[l], self.n_reuse[l]
            d = {name: torch.from_numpy(self.host[name][l, :n].copy()).to(device)
                 for name in ("slot", "map", "pos", "kv_start", "kv_len")}
            d.update({name: torch.from_numpy(self.reuse[name][l, :m].copy()).to(device)
                      for name in ("src_row", "dst_slot", "delta")})
            d["pos3"] = None
            if any(getattr(r, "pos3", None) is not None for r in requests):
                # 3-axis ids of the recomputed rows: packed slot -> (request, local slot) -> its ids
                all3 = np.concatenate([np.asarray(r.pos3, dtype=np.int32) for r in requests])   # requests are packed in order
                d["pos3"] = torch.from_numpy(np.ascontiguousarray(all3[self.host["slot"][l, :n]])).to(device)
            self.dev.append(d)

    def record(self, l: int, n_in: int, kv_rows: int, k_pool=None, v_pool=None) -> B.LayerPlan:
        d = self.dev[l]
        n, m = self.n_rows[l], self.n_reuse[l]
        p = lambda t: t.data_ptr() if t is not None and t.numel() else None
        return B.LayerPlan(n_in, n, p(d["map"]), p(d["slot"]), p(d["pos"]), p(d["kv_start"]), p(d["kv_len"]),
                           kv_rows, m if k_pool is not None else 0, p(d["src_row"]), p(d["dst_slot"]),
                           p(d["delta"]), p(k_pool), p(v_pool), 0 if k_pool is None else k_pool.shape[0],
                           p(d["pos3"]))


class ShiftJobs:
    """The reused keys/values of all layers as one job table for vlc_rope_shift_kv_layers: layer l moves the
    rows plans.reuse lists for it from k_pool[l] / v_pool[l] into k_cache[l] / v_cache[l].  The layers are then
    run with records made with k_pool=None (n_reuse = 0)."""

    def __init__(self, plans: DevicePlans, k_pool, v_pool, k_cache, v_cache):
        jobs = []
        for l, d in enumerate(plans.dev):
            if plans.n_reuse[l] > 0:
                jobs.append((k_pool[l], v_pool[l], k_cache[l], v_cache[l], d["src_row"], d["dst_slot"], d["delta"]))
        self.keep = jobs
        self.n_jobs = len(jobs)
        self.max_n_tok = max([j[4].numel() for j in jobs] + [0])
        self.table = torch.from_numpy(B.shift_job_table(jobs)).to(k_cache[0].device) if jobs else None
        self.Hkv, self.D = k_cache[0].shape[-2], k_cache[0].shape[-1]
        self.dtype = B._dtype_code(k_cache[0])

    def run(self, rope_base: float, stream=None) -> None:
        if self.n_jobs:
            B.vlc_rope_shift_kv_layers(self.table, self.n_jobs, self.max_n_tok, self.Hkv, self.D, rope_base,
                                       self.dtype, stream)


class Workspace:
    def __init__(self, shape_rec: B.LayerShape, n_rows_max: int, device="cuda"):
        nbytes = B.vlc_layer_workspace_bytes(shape_rec, n_rows_max)
        self.t = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
        assert self.t.data_ptr() % 256 == 0


def run_layer(shape_rec, weights: DeviceWeights, plan_rec, h_in, h_out, k_cache, v_cache, ws: Workspace,
              stream=None) -> None:
    B.vlc_layer_forward(shape_rec, weights.rec, plan_rec, h_in, h_out, k_cache, v_cache, ws.t, stream)


def chain_link(plans: DevicePlans, l: int):
    """How layer l can hand the input norm to layer l + 1: (False, None) if it cannot (last layer, or one of the
    two has no rows), else (True, next_row) with next_row None if layer l + 1 keeps every row (same row count: its
    rows are a subset), else the planner's int32 list (vlc_plan_next_rows) on the device.  Uploaded once per plan."""
    links = plans.__dict__.setdefault("_links", {})
    if l not in links:
        if l + 1 >= plans.L or plans.n_rows[l] == 0 or plans.n_rows[l + 1] == 0:
            links[l] = (False, None)
        elif plans.n_rows[l + 1] == plans.n_rows[l]:
            links[l] = (True, None)
        else:
            links[l] = (True, torch.from_numpy(plans.next_row[l, :plans.n_rows[l]].copy()).to(plans.dev[l]["slot"].device))
    return links[l]


def run_layers(shape_rec, weights: Sequence[DeviceWeights], plans: DevicePlans, records: Sequence, h0, hbuf,
               k_cache, v_cache, ws: Workspace, stream=None, events=None, chain: bool = True):
    """All layers in order through vlc_layer_forward_chained: every layer hands its successor the input norm
    (chain=False: every layer norms its own input).  h0 [n_in, H] is the first layer's input, hbuf two
    [n_max, H] buffers the layers alternate between; events: per-layer stage-event arrays or None.
    Returns the buffer that holds the last layer's output rows."""
    h_in, ready = h0, False
    for l in range(plans.L):
        h_out = hbuf[l & 1]
        linked, next_row = chain_link(plans, l) if chain else (False, None)
        B.vlc_layer_forward_chained(shape_rec, weights[l].rec, records[l], h_in, h_out, k_cache[l], v_cache[l], ws.t,
                                    ready, weights[l + 1].t["w_ln1"] if linked else None, next_row,
                                    None if events is None else events[l], stream)
        h_in, ready = h_out, linked
    return h_in


def plan_for(wl):
    """(k per layer | None, explicit leading-token count per layer | None) of a workload description,
    through the library's planner (the budget conversion included)."""
    L = wl.shape.L
    if wl.plan == "static":
        return np.full(L, wl.static_k, dtype=np.int32), None
    if wl.plan == "explicit":
        return None, np.full(L, wl.explicit_counts, dtype=np.int32)
    import vlc_synth as syn
    sens = syn.sensitivity_table(L, 150, 1)
    return B.vlc_plan_layer_rates(sens, B.vlc_plan_budget_steps(int(wl.budget_bp), L)), None
