"""GPU parity of vlc_layer_forward against the CPU oracle (needs an MI355X).

Two kinds of check:
  * end to end: the layer stack's outputs (h, K, V per layer) against the oracle, element by
    element, at the stated tolerance: 1e-5 for the fp32 configuration, 2e-2 + 1e-2*|o| for bf16.
  * stage by stage (bf16 at the 7B shape): every intermediate the layer leaves in its workspace is
    compared, at the same element-wise tolerance, with the oracle's stage evaluated on the GPU's own
    input to that stage.  A chain of bf16 roundings decorrelates two correct implementations (one
    flipped rounding upstream moves every later pre-rounding value), and the text rows' tiny
    residual lets the MLP amplify that; so at the 7B shape the end-to-end h is additionally required
    to be as close to the oracle as the oracle's own bf16 result is to its unrounded float64 result.
"""
import numpy as np
import pytest
import torch

import vlc_synth as syn
from oracle import vlc_oracle as orc
import paper_2512_12977_amd as vlc
from paper_2512_12977_amd import runner as R
from helpers import plan_steps, counts_for, assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda"


def back(t):
    return t.float().cpu().numpy().astype(np.float64)


def oracle_stack(wl, weights, emb, caches, k, explicit, layers, store=None):
    """Oracle results per request: list over requests of selective_prefill outputs."""
    st = store or orc.STORE[wl.shape.dtype]
    res = []
    for req in wl.requests:
        counts = [counts_for(req, k, explicit, l) for l in range(layers)]
        e = emb[req.kv_start:req.kv_start + req.S]
        res.append(orc.selective_prefill(wl.shape, weights[:layers], e, req, counts, caches[:layers], st))
    return res


def run_gpu_stack(wl, weights, emb, caches, k, explicit, layers, teacher=None, all_rows=False, keep_ws=False,
                  shift_ahead=False, chain=False):
    """Runs `layers` layers on the GPU.  teacher: optional per-layer input rows (oracle outputs of the
    previous layer) to feed instead of the GPU's own previous output.  shift_ahead: the reused keys/values of all
    layers are placed by one vlc_rope_shift_kv_layers call before the first layer and the layers get no reuse
    list.  chain: layers go through vlc_layer_forward_chained, every layer leaving its successor's input norm in
    the workspace (plans.chained counts 1 per link and 10 more per link that drops rows).  Returns per-layer (h, K, V[, ws])."""
    sh = wl.shape
    dt = R.torch_dtype(sh.dtype)
    rec = R.make_shape(sh)
    plans = R.DevicePlans(wl.requests, layers, k=None if k is None else k[:layers],
                          count_override=None if explicit is None else explicit[:layers], all_rows=all_rows)
    ws = R.Workspace(rec, max(plans.n_rows + [1]))
    total = wl.total_slots
    h_prev = torch.from_numpy(emb).to(DEV).to(dt)
    n_prev = total
    out = []
    kps = [torch.from_numpy(caches[l][0]).to(DEV).to(dt) for l in range(layers)]
    vps = [torch.from_numpy(caches[l][1]).to(DEV).to(dt) for l in range(layers)]
    kcs = [torch.zeros((total, sh.Hkv, sh.D), device=DEV, dtype=dt) for l in range(layers)]
    vcs = [torch.zeros((total, sh.Hkv, sh.D), device=DEV, dtype=dt) for l in range(layers)]
    if shift_ahead:
        assert not all_rows
        jobs = R.ShiftJobs(plans, kps, vps, kcs, vcs)
        assert jobs.n_jobs == sum(1 for m in plans.n_reuse if m > 0)
        jobs.run(sh.rope_base)
    assert not (chain and teacher is not None)
    ready, chained = False, 0
    dws = [R.DeviceWeights(weights[l], dt) for l in range(layers)]
    for l in range(layers):
        W = dws[l]
        kp, vp, kc, vc = kps[l], vps[l], kcs[l], vcs[l]
        if shift_ahead:
            kp = vp = None
        if teacher is not None and l > 0:
            h_prev = torch.from_numpy(teacher[l - 1].astype(np.float32)).to(DEV).to(dt)
        n = plans.n_rows[l]
        h_out = torch.empty((n, sh.H), device=DEV, dtype=dt)
        prec = plans.record(l, n_prev, total, None if all_rows else kp, None if all_rows else vp)
        assert not shift_ahead or prec.n_reuse == 0
        if chain:
            linked, next_row = R.chain_link(plans, l)
            vlc.vlc_layer_forward_chained(rec, W.rec, prec, h_prev, h_out, kc, vc, ws.t, ready,
                                          dws[l + 1].t["w_ln1"] if linked else None, next_row)
            ready = linked
            chained += int(linked) + 10 * int(next_row is not None)
        else:
            R.run_layer(rec, W, prec, h_prev, h_out, kc, vc, ws)
        torch.cuda.synchronize()
        item = [back(h_out), back(kc), back(vc)]
        if keep_ws:
            item.append(read_workspace(sh, rec, ws, n))
        out.append(item)
        h_prev, n_prev = h_out, n
    if chain:
        plans.chained = chained
    return out, plans


def read_workspace(sh, rec, ws, n):
    """The layer's intermediates, by stage name, as float64 arrays."""
    off = vlc.vlc_layer_workspace_layout(rec, n)
    dt = R.torch_dtype(sh.dtype)
    es = 2 if sh.dtype == "bf16" else 4
    shapes = {"xn": (n, sh.H), "qkv": (n, sh.n_qkv), "q": (n, sh.Hq, sh.D), "o": (n, sh.Hq, sh.D),
              "h1": (n, sh.H), "n2": (n, sh.H), "act": (n, sh.I)}
    res = {}
    for name, shp in shapes.items():
        tdt, size = (torch.float32, 4) if name == "qkv" else (dt, es)
        nb = int(np.prod(shp)) * size
        res[name] = back(ws.t[off[name]:off[name] + nb].view(tdt).reshape(shp))
    return res


def check_against_oracle(wl, layers, teacher_forced, all_rows=False, shift_ahead=False, chain=False):
    sh = wl.shape
    k, explicit = plan_steps(wl)
    if all_rows:
        k, explicit = np.full(sh.L, 500, dtype=np.int32), None
    weights = [syn.layer_weights(sh, wl.seed, l) for l in range(layers)]
    emb = syn.embedding_rows(wl)
    caches = [syn.cached_kv(wl, l) for l in range(layers)]
    ref = oracle_stack(wl, weights, emb, caches, k, explicit, layers)
    teacher = None
    if teacher_forced:
        teacher = [np.concatenate([ref[r][l]["h"] for r in range(len(wl.requests))]) for l in range(layers)]
    got, plans = run_gpu_stack(wl, weights, emb, caches, k, explicit, layers, teacher, all_rows, shift_ahead=shift_ahead,
                               chain=chain)
    if chain:
        check_against_oracle.chained = plans.chained
    worst = 0.0
    for l in range(layers):
        want_h = np.concatenate([ref[r][l]["h"] for r in range(len(wl.requests))])
        want_K = np.concatenate([ref[r][l]["K"] for r in range(len(wl.requests))])
        want_V = np.concatenate([ref[r][l]["V"] for r in range(len(wl.requests))])
        assert got[l][0].shape == want_h.shape
        assert_close(got[l][1], want_K, sh.dtype, "%s layer %d K" % (wl.name, l))
        assert_close(got[l][2], want_V, sh.dtype, "%s layer %d V" % (wl.name, l))
        worst = max(worst, assert_close(got[l][0], want_h, sh.dtype, "%s layer %d h" % (wl.name, l)))
    return worst


def check_layer_stage_by_stage(wl, layer=0):
    """One layer of a single-request workload: strict per-stage parity + end-to-end noise-floor check."""
    sh = wl.shape
    st = orc.STORE[sh.dtype]
    assert len(wl.requests) == 1
    req = wl.requests[0]
    k, explicit = plan_steps(wl)
    W = syn.layer_weights(sh, wl.seed, layer)
    emb = syn.embedding_rows(wl)
    cache = syn.cached_kv(wl, layer)
    # teacher-forced input of this layer: rows the previous layer would hand over (layer 0: all slots)
    counts = counts_for(req, k, explicit, layer)
    got, plans = run_gpu_stack(wl, [W], emb, [cache], None if k is None else k[layer:layer + 1],
                               None if explicit is None else explicit[layer:layer + 1], 1, keep_ws=True)
    g_h, g_K, g_V, g = got[0]
    slots = orc.select_slots(req.segments, counts)
    x = st(emb)[slots]
    Kb, Vb = orc.blended_kv_before_scatter(sh, req, counts, st(cache[0]), st(cache[1]), st)
    forced = dict(g)
    forced["K"], forced["V"] = g_K, g_V
    r = orc.layer_stages(sh, W, x, slots, orc.positions_of(req, slots), Kb, Vb, st, forced=forced)
    # every stage, on the GPU's own inputs, element-wise at the stated tolerance
    assert_close(g["xn"], r["xn"], sh.dtype, "stage xn")
    assert_close(g["qkv"], r["qkv"], sh.dtype, "stage qkv")
    assert_close(g["q"], r["q"], sh.dtype, "stage q")
    assert_close(g_K, r["K"], sh.dtype, "stage K (reused keys rotated + fresh keys)")
    assert_close(g_V, r["V"], sh.dtype, "stage V")
    assert_close(g["o"], r["o"], sh.dtype, "stage attention")
    assert_close(g["h1"], r["h1"], sh.dtype, "stage o-proj + residual")
    assert_close(g["n2"], r["n2"], sh.dtype, "stage norm2")
    assert_close(g["act"], r["act"], sh.dtype, "stage SwiGLU")
    assert_close(g_h, r["h2"], sh.dtype, "stage down-proj + residual")
    # end to end against the free-running oracle, relative to the bf16 noise floor
    Kb, Vb = orc.blended_kv_before_scatter(sh, req, counts, st(cache[0]), st(cache[1]), st)
    o16 = orc.layer_stages(sh, W, x, slots, orc.positions_of(req, slots), Kb, Vb, st)
    ex = orc.store_exact
    Kb, Vb = orc.blended_kv_before_scatter(sh, req, counts, cache[0], cache[1], ex)
    o64 = orc.layer_stages(sh, W, np.asarray(emb, dtype=np.float64)[slots], slots, orc.positions_of(req, slots), Kb, Vb, ex)
    nrm = np.linalg.norm
    floor = nrm(o16["h2"] - o64["h2"]) / nrm(o64["h2"])       # what bf16 storage costs the oracle itself
    dev = nrm(g_h - o16["h2"]) / nrm(o16["h2"])
    dev64 = nrm(g_h - o64["h2"]) / nrm(o64["h2"])
    assert dev <= floor, ("GPU differs from the bf16 oracle by more than the bf16 noise floor", dev, floor)
    assert dev64 <= 1.25 * floor, ("GPU is further from the exact result than bf16 storage explains", dev64, floor)
    assert_close(g_K, o16["K"], sh.dtype, "K end to end")
    assert_close(g_V, o16["V"], sh.dtype, "V end to end")
    return dev, floor


@pytest.mark.parametrize("name", ["c1", "c1_bias"])
def test_tiny_fp32_stack_end_to_end(name):
    """Configuration 1: 2-layer fp32 decoder, 13 leading image tokens recomputed, within 1e-5."""
    check_against_oracle(syn.make_workload(name), layers=2, teacher_forced=False)


def test_tiny_fp32_full_recompute_equals_oracle_full_prefill():
    wl = syn.make_workload("c1")
    check_against_oracle(wl, layers=2, teacher_forced=False, all_rows=True)


def test_tiny_bf16_stack():
    wl = syn.make_workload("c1_bf16")
    check_against_oracle(wl, layers=2, teacher_forced=True)
    check_against_oracle(wl, layers=2, teacher_forced=False)
    check_layer_stage_by_stage(wl, layer=1)


def test_two_packed_requests_fp32():
    """A batch of two requests with different shifts, packed into one launch per kernel."""
    sh = syn.SHAPES["tiny_bias"]
    r0 = syn.Request([syn.Segment(0, 20, False), syn.Segment(20, 100, True, 3, 0), syn.Segment(120, 9, False)], 0)
    r1 = syn.Request([syn.Segment(0, 7, False), syn.Segment(7, 60, True, 50, 100), syn.Segment(67, 40, True, 0, 160),
                      syn.Segment(107, 5, False)], 129, pos_start=11)
    wl = syn.Workload("two", sh, [r0, r1], 200, "static", static_k=40, seed=12)
    check_against_oracle(wl, layers=2, teacher_forced=False)


@pytest.mark.parametrize("rows", [1, 2, 31, 33, 64, 65, 127, 129, 191, 193, 255, 257, 383, 385, 513, 641])
def test_bf16_layer_row_counts_around_tile_edges(rows):
    """One bf16 layer over `rows` text tokens (every row computed): row counts just below, at and above the 32-row
    MFMA tiles and the 128-row workgroup tiles, so that the clamped loads of a ragged last tile, its guarded
    stores, the ragged last column tile of the 96-column gate|up tiles and the key split of the attention (from
    257 rows on there are more than 4 key blocks) are all hit."""
    sh = syn.SHAPES["tiny_bf16"]
    req = syn.Request([syn.Segment(0, rows, False)], 0)
    wl = syn.Workload("rows_%d" % rows, sh, [req], 1, "static", static_k=0, seed=100 + rows)
    check_against_oracle(wl, layers=1, teacher_forced=False, all_rows=True)


def test_three_packed_requests_bf16_keys_shared_out_over_workgroups():
    """Few rows, so the bf16 attention shares the keys out in pieces of 4 blocks (1220 slots: 5 pieces): rows of three
    requests of 700, 130 and 390 slots share row tiles, the short request's rows fit one piece, the long one's
    need up to three, and the pieces beyond a tile's longest row are never written."""
    sh = syn.SHAPES["tiny_bf16"]
    r0 = syn.Request([syn.Segment(0, 40, False), syn.Segment(40, 600, True, 7, 0), syn.Segment(640, 60, False)], 0)
    r1 = syn.Request([syn.Segment(0, 30, False), syn.Segment(30, 80, True, 200, 600), syn.Segment(110, 20, False)], 700,
                     pos_start=5)
    r2 = syn.Request([syn.Segment(0, 90, False), syn.Segment(90, 300, True, 0, 680)], 830)
    wl = syn.Workload("three", sh, [r0, r1, r2], 980, "static", static_k=40, seed=17)
    check_against_oracle(wl, layers=2, teacher_forced=True)
    check_against_oracle(wl, layers=2, teacher_forced=False, shift_ahead=True)


def test_reused_keys_of_all_layers_placed_ahead_of_the_layer_loop():
    """vlc_rope_shift_kv_layers + layers without a reuse list give the oracle's stack: two packed requests in
    fp32, the bf16 tiny stack, and rates that fall with depth (a different reuse list in every layer)."""
    sh = syn.SHAPES["tiny_bias"]
    r0 = syn.Request([syn.Segment(0, 20, False), syn.Segment(20, 100, True, 3, 0), syn.Segment(120, 9, False)], 0)
    r1 = syn.Request([syn.Segment(0, 7, False), syn.Segment(7, 60, True, 50, 100), syn.Segment(67, 40, True, 0, 160),
                      syn.Segment(107, 5, False)], 129, pos_start=11)
    check_against_oracle(syn.Workload("two", sh, [r0, r1], 200, "static", static_k=40, seed=12), layers=2,
                         teacher_forced=False, shift_ahead=True)
    check_against_oracle(syn.make_workload("c1_bf16"), layers=2, teacher_forced=True, shift_ahead=True)
    wl = syn.Workload("falling", sh, [r0, r1], 200, "dynamic", budget_bp=2000, seed=13)
    k, _ = plan_steps(wl)
    assert len(set(k.tolist())) > 1
    check_against_oracle(wl, layers=sh.L, teacher_forced=False, shift_ahead=True)


def test_chained_layers_small_shapes():
    """vlc_layer_forward_chained over whole stacks against the oracle: the fp32 and bf16 tiny stacks and the packed
    pair with a uniform rate (the successor keeps every row), full recompute, and rates that fall with depth (the
    successor drops rows: the norm is written through the row list)."""
    for name in ("c1", "c1_bf16", "c1_q3"):
        check_against_oracle(syn.make_workload(name), layers=2, teacher_forced=False, chain=True)
        assert check_against_oracle.chained == 1
    check_against_oracle(syn.make_workload("c1"), layers=2, teacher_forced=False, all_rows=True, chain=True)
    assert check_against_oracle.chained == 1
    sh = syn.SHAPES["tiny_bias"]
    r0 = syn.Request([syn.Segment(0, 20, False), syn.Segment(20, 100, True, 3, 0), syn.Segment(120, 9, False)], 0)
    r1 = syn.Request([syn.Segment(0, 7, False), syn.Segment(7, 60, True, 50, 100), syn.Segment(67, 40, True, 0, 160),
                      syn.Segment(107, 5, False)], 129, pos_start=11)
    check_against_oracle(syn.Workload("two", sh, [r0, r1], 200, "static", static_k=40, seed=12), layers=2,
                         teacher_forced=False, shift_ahead=True, chain=True)
    assert check_against_oracle.chained == 1
    wl = syn.Workload("falling", sh, [r0, r1], 200, "dynamic", budget_bp=2000, seed=13)
    k, _ = plan_steps(wl)
    assert k[0] != k[1]
    check_against_oracle(wl, layers=sh.L, teacher_forced=False, chain=True)
    assert check_against_oracle.chained == 11
    wl = syn.Workload("falling_bf16", syn.SHAPES["tiny_bf16"], [r0, r1], 200, "dynamic", budget_bp=2000, seed=14)
    check_against_oracle(wl, layers=2, teacher_forced=False, chain=True)
    assert check_against_oracle.chained == 11


def test_7b_shape_layer_stage_by_stage():
    """Configuration 2 (7B-shaped bf16 layer, S=1600, 596 recomputed rows), layers 0 and 1."""
    wl = syn.make_workload("c2")
    for layer in (0, 1):
        dev, floor = check_layer_stage_by_stage(wl, layer)
        print("c2 layer %d: |gpu-oracle|/|oracle| = %.2e, bf16 noise floor %.2e" % (layer, dev, floor))


# ---- Qwen3-VL-shaped layer: per-head q/k RMSNorm before the rotation, interleaved 3-axis RoPE ----

def test_q3_tiny_fp32_stack_end_to_end():
    """2-layer fp32 decoder with q/k norm and grid position ids, 13 leading image tokens recomputed."""
    wl = syn.make_workload("c1_q3")
    check_against_oracle(wl, layers=2, teacher_forced=False)
    check_against_oracle(wl, layers=2, teacher_forced=False, all_rows=True)


def test_q3_tiny_bf16_stack():
    wl = syn.make_workload("c1_q3_bf16")
    check_against_oracle(wl, layers=2, teacher_forced=True)
    check_layer_stage_by_stage(wl, layer=0)
    check_layer_stage_by_stage(wl, layer=1)


def test_q3_two_packed_requests_images_moved_both_ways_fp32():
    """Two packed requests; images of different grids, moved forwards and backwards from their cached ids."""
    sh = syn.SHAPES["tiny_q3"]
    from vlc_synth.workloads import _grid_request
    r0 = _grid_request([("text", 20), ("image", 10, 7, 3, 0), ("text", 9)], 0)
    r1 = _grid_request([("text", 7), ("image", 6, 10, 50, 70), ("image", 5, 8, 0, 130), ("text", 5)], r0.S)
    wl = syn.Workload("two_q3", sh, [r0, r1], 170, "static", static_k=40, seed=13)
    check_against_oracle(wl, layers=2, teacher_forced=False)


def test_q3_8b_shape_layer_stage_by_stage():
    """Qwen3-VL 8B text-decoder shape (bf16, S=1600, 596 recomputed rows): every stage against the oracle."""
    wl = syn.make_workload("c2_q3")
    dev, floor = check_layer_stage_by_stage(wl, 0)
    print("c2_q3 layer 0: |gpu-oracle|/|oracle| = %.2e, bf16 noise floor %.2e" % (dev, floor))
