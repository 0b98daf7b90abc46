"""GPU parity of the mixture-of-experts layer against the CPU oracle (needs an MI355X).

The expert choice is an integer decided by floating point: both sides take it from the same values
(the GPU's float router scores), where it must then agree exactly, order included; the scores
themselves are compared with the oracle's at the layer's tolerance.  Everything downstream is
compared pair by pair through the grouped order the GPU reports (a permutation that is checked
for consistency, not for a particular order inside an expert).
"""
import numpy as np
import pytest
import torch

import vlc_synth as syn
from oracle import vlc_oracle as orc
import paper_2512_12977_amd as vlc
from paper_2512_12977_amd import runner as R
from helpers import plan_steps, counts_for, assert_close
from test_gpu_layer import run_gpu_stack, back, check_against_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"


def read_moe(sh, rec, ws, n):
    off = vlc.vlc_layer_workspace_layout(rec, n)
    dt = R.torch_dtype(sh.dtype)
    es = 2 if sh.dtype == "bf16" else 4
    K, E, P = sh.top_k, sh.n_experts, n * sh.top_k

    def take(name, tdt, shape, size):
        nb = int(np.prod(shape)) * size
        return ws.t[off[name]:off[name] + nb].view(tdt).reshape(shape)

    out = {name: back(take(name, dt, shp, es)) for name, shp in
           (("xn", (n, sh.H)), ("h1", (n, sh.H)), ("n2", (n, sh.H)), ("act", (P, sh.I)), ("moe_y", (P, sh.H)))}
    out["moe_logits"] = back(take("moe_logits", torch.float32, (n, E), 4))
    out["moe_w"] = back(take("moe_w", torch.float32, (n, K), 4))
    out["moe_idx"] = take("moe_idx", torch.int32, (n, K), 4).cpu().numpy().astype(np.int64)
    out["moe_pos"] = take("moe_pos", torch.int32, (n, K), 4).cpu().numpy().astype(np.int64)
    out["moe_offset"] = take("moe_offset", torch.int32, (E + 1,), 4).cpu().numpy().astype(np.int64)
    return out


def check_moe_layer(wl, layer=0):
    sh = wl.shape
    st = orc.STORE[sh.dtype]
    req = wl.requests[0]
    k, explicit = plan_steps(wl)
    W = syn.layer_weights(sh, wl.seed, layer)
    emb = syn.embedding_rows(wl)
    cache = syn.cached_kv(wl, layer)
    sh_rec = R.make_shape(sh)
    got, plans = run_gpu_stack(wl, [W], emb, [cache], None if k is None else k[layer:layer + 1],
                               None if explicit is None else explicit[layer:layer + 1], 1, keep_ws=False)
    # run_gpu_stack does not know the expert fields: run once more here keeping the workspace
    dt = R.torch_dtype(sh.dtype)
    n = plans.n_rows[0]
    ws = R.Workspace(sh_rec, n)
    total = wl.total_slots
    dW = R.DeviceWeights(W, dt)
    kp, vp = torch.from_numpy(cache[0]).to(DEV).to(dt), torch.from_numpy(cache[1]).to(DEV).to(dt)
    kc = torch.zeros((total, sh.Hkv, sh.D), device=DEV, dtype=dt)
    vc = torch.zeros_like(kc)
    h_in = torch.from_numpy(emb).to(DEV).to(dt)
    h_out = torch.empty((n, sh.H), device=DEV, dtype=dt)
    R.run_layer(sh_rec, dW, plans.record(0, total, total, kp, vp), h_in, h_out, kc, vc, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(back(h_out), got[0][0])            # two runs of the same layer agree bit for bit
    g = read_moe(sh, sh_rec, ws, n)
    K, E = sh.top_k, sh.n_experts
    Ws = {name: (None if w is None else st(w)) for name, w in W.items()}

    # router scores from the GPU's own normed rows
    assert_close(g["moe_logits"], orc.linear(g["n2"], Ws["w_router"]), sh.dtype, "router scores")
    # the choice, taken by both sides from the GPU's float scores: exact, order included
    want_idx, want_w = orc.route_top_k(g["moe_logits"], K)
    np.testing.assert_array_equal(g["moe_idx"], want_idx)
    np.testing.assert_allclose(g["moe_w"], want_w, rtol=2e-6, atol=1e-7)
    # grouped order: first pair of every expert = running count; every pair inside its expert's range; a permutation
    counts = np.bincount(g["moe_idx"].ravel(), minlength=E)
    np.testing.assert_array_equal(g["moe_offset"], np.concatenate([[0], np.cumsum(counts)]))
    pos = g["moe_pos"]
    assert np.array_equal(np.sort(pos.ravel()), np.arange(n * K))
    assert np.all(pos >= g["moe_offset"][g["moe_idx"]]) and np.all(pos < g["moe_offset"][g["moe_idx"] + 1])
    # experts, pair by pair, on the GPU's inputs
    forced = {"moe_idx": g["moe_idx"], "moe_w": g["moe_w"], "act": g["act"][pos], "y": g["moe_y"][pos]}
    r = orc.moe_mlp(sh, Ws, g["n2"], st, forced)
    assert_close(g["act"][pos], r["act"], sh.dtype, "SwiGLU product of the chosen experts")
    assert_close(g["moe_y"][pos], r["y"], sh.dtype, "expert outputs")
    assert_close(back(h_out), st(g["h1"] + r["mlp"]), sh.dtype, "weighted sum + residual")
    return g


def test_moe_tiny_fp32_stack_end_to_end():
    """2-layer fp32 decoder with 8 experts, 2 per token: every output against the free-running oracle."""
    check_against_oracle(syn.make_workload("c1_moe"), layers=2, teacher_forced=False)
    check_against_oracle(syn.make_workload("c1_moe"), layers=2, teacher_forced=False, chain=True)
    assert check_against_oracle.chained == 1


def stack_both_ways(wl, layers):
    """The first `layers` layers free-running on the GPU, layer by layer and chained; returns both results."""
    sh = wl.shape
    k, explicit = plan_steps(wl)
    weights = [syn.layer_weights(sh, wl.seed, l) for l in range(layers)]
    emb = syn.embedding_rows(wl)
    caches = [syn.cached_kv(wl, l) for l in range(layers)]
    plain, _ = run_gpu_stack(wl, weights, emb, caches, k, explicit, layers)
    chained, plans = run_gpu_stack(wl, weights, emb, caches, k, explicit, layers, chain=True)
    return plain, chained, plans


@pytest.mark.parametrize("name", ["c1_moe", "c1_moe_bf16", "falling", "c2_moe"])
def test_moe_chained_layers_equal_layer_by_layer(name):
    """With experts the chained call takes the next layer's input norm in the kernel that forms the weighted sum of
    the experts' outputs: h_out and K/V of every layer equal, bit for bit, those of vlc_layer_forward layer by layer
    (which the other tests compare with the oracle) - tiny fp32 and bf16 stacks, a bf16 stack whose second layer
    drops rows, and two layers at the 30B-A3B shape."""
    if name == "falling":
        from vlc_synth.workloads import _grid_request
        req = _grid_request([("text", 20), ("image", 10, 10, 3, 0), ("text", 9), ("image", 6, 10, 40, 100), ("text", 5)])
        wl = syn.Workload("falling_moe", syn.SHAPES["tiny_moe_bf16"], [req], 160, "dynamic", budget_bp=2000, seed=16)
    else:
        wl = syn.make_workload(name)
    plain, chained, plans = stack_both_ways(wl, 2)
    assert plans.chained == (11 if name == "falling" else 1)
    for l in range(2):
        for a, b, what in zip(plain[l], chained[l], ("h_out", "K", "V")):
            assert np.array_equal(a, b), "%s of layer %d" % (what, l)
    if name != "c2_moe":
        check_against_oracle(wl, layers=2, teacher_forced=False, chain=True)


@pytest.mark.parametrize("name", ["c1_moe", "c1_moe_bf16"])
def test_moe_tiny_layer_stage_by_stage(name):
    wl = syn.make_workload(name)
    g = check_moe_layer(wl, 0)
    assert len(np.unique(g["moe_idx"])) == wl.shape.n_experts        # every expert is used
    check_moe_layer(wl, 1)


def test_moe_30b_a3b_shape_layer_stage_by_stage():
    """Qwen3-VL-30B-A3B text-decoder shape (128 experts, 8 per token, bf16), 596 recomputed rows."""
    g = check_moe_layer(syn.make_workload("c2_moe"), 0)
    counts = np.bincount(g["moe_idx"].ravel(), minlength=128)
    print("pairs per expert: min %d median %d max %d" % (counts.min(), np.median(counts), counts.max()))


def test_moe_many_pairs_grouped_with_atomic_ranks():
    """More than 65536 (row, expert) pairs: ranks come from atomic counters in the choice kernel and the plan / fill
    kernels, and with 10000 rows per expert the grouped GEMMs run on 256-row tiles.  330 short text-only requests."""
    sh = syn.SHAPES["tiny_moe_bf16"]
    reqs = [syn.Request([syn.Segment(0, 124, False)], 124 * i, 0, syn.grid_positions([("text", 124)])) for i in range(330)]
    wl = syn.Workload("moe_many", sh, reqs, 1, "static", static_k=0, seed=14)
    g = check_moe_layer(wl, 0)
    assert g["moe_idx"].shape == (330 * 124, 2)


@pytest.mark.parametrize("rows", [250, 420, 700])
def test_moe_mid_sized_groups_on_128_row_tiles(rows):
    """62, 105 and 175 rows per expert on average (8 experts, 2 per token): the grouped GEMMs run on 128 x 128 tiles
    (56 to 191 rows per expert), with groups of one and of two row tiles, the last ragged."""
    sh = syn.SHAPES["tiny_moe_bf16"]
    req = syn.Request([syn.Segment(0, rows, False)], 0, 0, syn.grid_positions([("text", rows)]))
    wl = syn.Workload("moe_mid_%d" % rows, sh, [req], 1, "static", static_k=0, seed=18)
    g = check_moe_layer(wl, 0)
    assert g["moe_idx"].shape == (rows, 2)


def test_moe_more_pairs_than_2_gib_of_input_rows():
    """66000 rows at the 30B-A3B shape: 528000 (row, expert) pairs, so pairs x row bytes (2.2 GB) passes the 2 GiB
    that the grouped GEMM's 32-bit row offsets cover while the rows themselves (270 MB) do not - the bound that
    counts is the rows'.  Grouping invariants on everything; the experts' arithmetic on 48 sampled rows."""
    sh = syn.SHAPES["q3vl_30b_a3b"]
    st = orc.STORE[sh.dtype]
    dt = R.torch_dtype(sh.dtype)
    T, B = 1000, 66
    reqs = [syn.Request([syn.Segment(0, T, False)], T * i, 0, syn.grid_positions([("text", T)])) for i in range(B)]
    wl = syn.Workload("moe_wide", sh, reqs, 1, "static", static_k=0, seed=15)
    W = syn.layer_weights(sh, wl.seed, 0)
    emb = syn.embedding_rows(wl)
    rec = R.make_shape(sh)
    plans = R.DevicePlans(wl.requests, 1, k=np.zeros(1, dtype=np.int32))
    n, total = plans.n_rows[0], wl.total_slots
    assert n == T * B and n * sh.top_k * sh.H * 2 >= 2 ** 31 > n * sh.H * 2
    ws = R.Workspace(rec, n)
    dW = R.DeviceWeights(W, dt)
    kc = torch.zeros((total, sh.Hkv, sh.D), device=DEV, dtype=dt)
    vc = torch.zeros_like(kc)
    h_in = torch.from_numpy(emb).to(DEV).to(dt)
    h_out = torch.empty((n, sh.H), device=DEV, dtype=dt)
    R.run_layer(rec, dW, plans.record(0, total, total, None, None), h_in, h_out, kc, vc, ws)
    torch.cuda.synchronize()

    off = vlc.vlc_layer_workspace_layout(rec, n)
    K, E, P = sh.top_k, sh.n_experts, n * sh.top_k

    def take(name, tdt, shape, size):
        return ws.t[off[name]:off[name] + int(np.prod(shape)) * size].view(tdt).reshape(shape)

    idx = take("moe_idx", torch.int32, (n, K), 4).cpu().numpy().astype(np.int64)
    pos = take("moe_pos", torch.int32, (n, K), 4).cpu().numpy().astype(np.int64)
    offset = take("moe_offset", torch.int32, (E + 1,), 4).cpu().numpy().astype(np.int64)
    counts = np.bincount(idx.ravel(), minlength=E)
    np.testing.assert_array_equal(offset, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(np.sort(pos.ravel()), np.arange(P))
    assert np.all(pos >= offset[idx]) and np.all(pos < offset[idx + 1])

    sel = np.unique(np.concatenate([[0, 1, n - 1], np.random.default_rng(0).integers(0, n, size=45)]))
    sel_t = torch.from_numpy(sel).to(DEV)
    pos_t = torch.from_numpy(pos[sel]).to(DEV)
    n2 = back(take("n2", dt, (n, sh.H), 2)[sel_t])
    h1 = back(take("h1", dt, (n, sh.H), 2)[sel_t])
    logits = back(take("moe_logits", torch.float32, (n, E), 4)[sel_t])
    wts = back(take("moe_w", torch.float32, (n, K), 4)[sel_t])
    act = back(take("act", dt, (P, sh.I), 2)[pos_t])
    y = back(take("moe_y", dt, (P, sh.H), 2)[pos_t])
    Ws = {name: (None if w is None else st(w)) for name, w in W.items()}
    want_idx, want_w = orc.route_top_k(logits, K)
    np.testing.assert_array_equal(idx[sel], want_idx)
    np.testing.assert_allclose(wts, want_w, rtol=2e-6, atol=1e-7)
    r = orc.moe_mlp(sh, Ws, n2, st, {"moe_idx": idx[sel], "moe_w": wts, "act": act, "y": y})
    assert_close(act, r["act"], sh.dtype, "SwiGLU product of the chosen experts")
    assert_close(y, r["y"], sh.dtype, "expert outputs")
    assert_close(back(h_out[sel_t]), st(h1 + r["mlp"]), sh.dtype, "weighted sum + residual")


@pytest.mark.parametrize("seed", range(12))
def test_moe_random_expert_counts_widths_and_rows(seed):
    """Seeded random mixture-of-experts layers: 3-48 experts, 1-6 per token, expert widths 64-512, 5-1500 rows, fp32 and
    bf16 in turn - expert groups from empty to several row tiles, on all three tile sizes of the grouped GEMMs."""
    rng = np.random.default_rng(11000 + seed)
    bf16 = seed % 2 == 1
    D = 128 if bf16 else 64
    E = int(rng.integers(3, 49))
    if bf16:
        E = 4 * ((E + 3) // 4)          # bf16: the number of experts is a multiple of 4 (the library refuses others)
    top_k = int(rng.integers(1, min(E, 6) + 1))
    half = D // 2
    h_sec, w_sec = int(rng.integers(0, half // 2 + 1)), int(rng.integers(0, half // 2 + 1))
    sh = syn.Shape("moe_random%d" % seed, L=1, H=64 * int(rng.integers(2, 9)), Hq=4, Hkv=2, D=D, I=64 * int(rng.integers(1, 9)),
                   rope_base=1e4, dtype="bf16" if bf16 else "f32", qkv_bias=False, qk_norm=True,
                   mrope_section=(half - h_sec - w_sec, h_sec, w_sec), n_experts=E, top_k=top_k, text_scale=1.0,
                   residual_proj_scale=0.01)
    rows = int(rng.integers(5, 1500))
    req = syn.Request([syn.Segment(0, rows, False)], 0, 0, syn.grid_positions([("text", rows)]))
    wl = syn.Workload("moe_random%d" % seed, sh, [req], 1, "static", static_k=0, seed=300 + seed)
    g = check_moe_layer(wl, 0)
    assert g["moe_idx"].shape == (rows, top_k)
