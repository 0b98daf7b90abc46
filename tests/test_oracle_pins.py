"""Pins of the CPU oracle against things other than itself (no GPU).

Each test names what it pins and the passage of the paper (arxiv 2512.12977) that fixes it.
"""
import dataclasses
import itertools
import math

import numpy as np
import pytest
import torch

import vlc_synth as syn
from oracle import vlc_oracle as orc


# ------------------------------------------------------------------------------------------
# helpers (test side only)
# ------------------------------------------------------------------------------------------
def tiny_setup(shape_name="tiny", L=2, seed=0, parts=((32, False), (48, True), (16, False))):
    shape = syn.SHAPES[shape_name]
    segs, at, crow = [], 0, 0
    for n, is_img in parts:
        segs.append(syn.Segment(at, n, is_img, at if is_img else 0, crow if is_img else 0))
        if is_img:
            crow += n
        at += n
    req = syn.Request(segs, 0)
    W = [syn.layer_weights(shape, seed, l) for l in range(L)]
    rng = np.random.default_rng(seed + 100)
    emb = rng.standard_normal((at, shape.H))
    return shape, req, W, emb, crow


def img_counts(req, value):
    return [min(value, s.length) if value is not None else s.length for s in req.segments if s.is_image]


# ------------------------------------------------------------------------------------------
# storage rounding
# ------------------------------------------------------------------------------------------
def test_bf16_round_matches_torch_and_known_ties():
    """bf16 round-to-nearest-even: library conversion (torch CPU) and hand-picked tie cases."""
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000), rng.standard_normal(2000) * 1e-3,
                        rng.standard_normal(2000) * 300.0]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    got = orc.store_bf16(x.astype(np.float64))
    np.testing.assert_array_equal(got, want)
    # 8 significant bits: 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0)
    assert orc.store_bf16(1.0 + 2.0 ** -8) == 1.0
    assert orc.store_bf16(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
    assert orc.store_bf16(-(1.0 + 2.0 ** -8 + 2.0 ** -20)) == -(1.0 + 2.0 ** -7)
    assert orc.store_bf16(0.0) == 0.0


# ------------------------------------------------------------------------------------------
# RoPE (Sec. 4.2: keys are stored position-free and rotated for the new position)
# ------------------------------------------------------------------------------------------
def test_rope_hand_values():
    """D=2: a single pair (x0, x1) at position p is the plane rotation by p radians
    (frequency base^0 = 1).  Fixes the sign of the rotation."""
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])             # [2 tokens, 1 head, D=2]
    y = orc.rope_rotate(x, np.array([1, 2]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [math.cos(1.0), math.sin(1.0)], atol=1e-15)
    np.testing.assert_allclose(y[1, 0], [-math.sin(2.0), math.cos(2.0)], atol=1e-15)


def test_rope_frequency_values():
    """D=4, base 10000: pair 0 = (x0, x2) turns by p, pair 1 = (x1, x3) by p * 10000^(-1/2) = p/100."""
    x = np.array([[[1.0, 1.0, 0.0, 0.0]]])
    y = orc.rope_rotate(x, np.array([50]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [math.cos(50.0), math.cos(0.5), math.sin(50.0), math.sin(0.5)],
                               atol=1e-13)


def test_rope_is_complex_multiplication():
    """Rotation of the pair (lo_i, hi_i) equals multiplying lo_i + j hi_i by exp(j p theta_i)."""
    rng = np.random.default_rng(1)
    D, n, Hh = 64, 7, 3
    x = rng.standard_normal((n, Hh, D))
    pos = rng.integers(-5000, 5000, size=n)
    z = x[..., :D // 2] + 1j * x[..., D // 2:]
    theta = 1e6 ** (-np.arange(0, D, 2) / D)
    z2 = z * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    y = orc.rope_rotate(x, pos, 1e6)
    np.testing.assert_allclose(y[..., :D // 2], z2.real, atol=1e-11)
    np.testing.assert_allclose(y[..., D // 2:], z2.imag, atol=1e-11)


def test_rope_shift_group_properties():
    """shift(d) then shift(-d) is the identity; shifts add; shifting un-rotated keys by p is RoPE at p;
    each pair keeps its norm."""
    rng = np.random.default_rng(2)
    D, n, Hh, base = 128, 33, 4, 1e6
    x = rng.standard_normal((n, Hh, D))
    d1 = rng.integers(-20000, 20000, size=n)
    d2 = rng.integers(-20000, 20000, size=n)
    a = orc.rope_rotate(orc.rope_rotate(x, d1, base), -d1, base)
    np.testing.assert_allclose(a, x, atol=1e-10)
    b = orc.rope_rotate(orc.rope_rotate(x, d1, base), d2, base)
    np.testing.assert_allclose(b, orc.rope_rotate(x, d1 + d2, base), atol=1e-9)
    y = orc.rope_rotate(x, d1, base)
    np.testing.assert_allclose(y[..., :64] ** 2 + y[..., 64:] ** 2, x[..., :64] ** 2 + x[..., 64:] ** 2,
                               rtol=1e-12)
    # zero shift is exactly the identity
    np.testing.assert_array_equal(orc.rope_rotate(x, np.zeros(n, dtype=np.int64), base), x)


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 1, 64))
    k = rng.standard_normal((1, 1, 64))
    s0 = np.sum(orc.rope_rotate(q, [17], 1e4) * orc.rope_rotate(k, [5], 1e4))
    s1 = np.sum(orc.rope_rotate(q, [1017], 1e4) * orc.rope_rotate(k, [1005], 1e4))
    assert abs(s0 - s1) < 1e-10


# ------------------------------------------------------------------------------------------
# attention for selected rows (Fig. 4)
# ------------------------------------------------------------------------------------------
def brute_attention(q, K, V, kv_len, scale):
    n, Hq, D = q.shape
    g = Hq // K.shape[1]
    out = np.zeros_like(q)
    for i in range(n):
        for h in range(Hq):
            c = int(kv_len[i])
            if c == 0:
                continue
            s = [scale * sum(q[i, h, d] * K[j, h // g, d] for d in range(D)) for j in range(c)]
            m = max(s)
            w = [math.exp(v - m) for v in s]
            tot = sum(w)
            for d in range(D):
                out[i, h, d] = sum(w[j] * V[j, h // g, d] for j in range(c)) / tot
    return out


def test_attention_rows_vs_brute_force_loops():
    rng = np.random.default_rng(4)
    S, Hq, Hkv, D = 11, 4, 2, 8
    K = rng.standard_normal((S, Hkv, D))
    V = rng.standard_normal((S, Hkv, D))
    slots = np.array([0, 3, 4, 10])
    q = rng.standard_normal((len(slots), Hq, D))
    got = orc.attention_rows(q, K, V, slots + 1, 0.37)
    np.testing.assert_allclose(got, brute_attention(q, K, V, slots + 1, 0.37), atol=1e-13)


def test_attention_rows_vs_torch_sdpa_row_selection():
    """Dense causal S x S attention by the library routine, rows picked afterwards."""
    rng = np.random.default_rng(5)
    S, Hq, Hkv, D = 40, 6, 2, 16
    Q = rng.standard_normal((S, Hq, D))
    K = rng.standard_normal((S, Hkv, D))
    V = rng.standard_normal((S, Hkv, D))
    tq, tk, tv = (torch.from_numpy(a).permute(1, 0, 2)[None] for a in (Q, K, V))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, enable_gqa=True)
    ref = ref[0].permute(1, 0, 2).numpy()
    rows = np.array([0, 1, 7, 8, 9, 30, 39])
    got = orc.attention_rows(Q[rows], K, V, rows + 1, 1.0 / math.sqrt(D))
    np.testing.assert_allclose(got, ref[rows], atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(6)
    S, Hq, Hkv, D = 9, 4, 4, 8
    K = rng.standard_normal((S, Hkv, D))
    q = rng.standard_normal((3, Hq, D))
    # V = ones -> output ones (softmax weights sum to one)
    o = orc.attention_rows(q, K, np.ones((S, Hkv, D)), [1, 5, 9], 1.0)
    np.testing.assert_allclose(o, 1.0, atol=1e-14)
    # a single visible key -> output is that key's V
    V = rng.standard_normal((S, Hkv, D))
    o = orc.attention_rows(q[:1], K, V, [1], 1.0)
    np.testing.assert_allclose(o[0], V[0], atol=1e-14)
    # no visible key -> zeros
    o = orc.attention_rows(q[:1], K, V, [0], 1.0)
    assert np.all(o == 0.0)
    # GQA mapping: heads 2g..2g+g-1 read kv head 2
    K2 = rng.standard_normal((S, 2, D))
    V2 = np.zeros((S, 2, D))
    V2[:, 1, :] = 1.0
    o = orc.attention_rows(q, K2, V2, [9, 9, 9], 1.0)
    np.testing.assert_allclose(o[:, :2], 0.0, atol=1e-14)
    np.testing.assert_allclose(o[:, 2:], 1.0, atol=1e-14)


# ------------------------------------------------------------------------------------------
# decoder layer: full prefill equals the Qwen2 decoder layer of the `transformers` library
# ------------------------------------------------------------------------------------------
def load_qwen2_layer(layer, shape, W, bias):
    """Copy one layer of vlc_synth weights into a `transformers` Qwen2DecoderLayer (float64)."""
    Hq, Hkv, D = shape.Hq, shape.Hkv, shape.D
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    wq, wk, wv = np.split(W["w_qkv"], [Hq * D, (Hq + Hkv) * D], axis=0)
    layer.self_attn.q_proj.weight.copy_(t(wq))
    layer.self_attn.k_proj.weight.copy_(t(wk))
    layer.self_attn.v_proj.weight.copy_(t(wv))
    b = W["b_qkv"] if bias else np.zeros(shape.n_qkv)
    bq, bk, bv = np.split(b, [Hq * D, (Hq + Hkv) * D])
    layer.self_attn.q_proj.bias.copy_(t(bq))
    layer.self_attn.k_proj.bias.copy_(t(bk))
    layer.self_attn.v_proj.bias.copy_(t(bv))
    layer.self_attn.o_proj.weight.copy_(t(W["w_o"]))
    layer.mlp.gate_proj.weight.copy_(t(W["w_gate_up"][:shape.I]))
    layer.mlp.up_proj.weight.copy_(t(W["w_gate_up"][shape.I:]))
    layer.mlp.down_proj.weight.copy_(t(W["w_down"]))
    layer.input_layernorm.weight.copy_(t(W["w_ln1"]))
    layer.post_attention_layernorm.weight.copy_(t(W["w_ln2"]))


@pytest.mark.parametrize("bias", [False, True])
def test_full_prefill_layer_vs_transformers_qwen2(bias):
    """The paper evaluates on Qwen-VL decoders and leaves layer details to that family; the
    oracle's full prefill must equal the library's own Qwen2 decoder layer (fp64, eager)."""
    from transformers import Qwen2Config
    from transformers.models.qwen2.modeling_qwen2 import Qwen2DecoderLayer, Qwen2RotaryEmbedding

    shape = syn.SHAPES["tiny_bias" if bias else "tiny"]
    W = syn.layer_weights(shape, 11, 0)
    S = 37
    rng = np.random.default_rng(12)
    emb = rng.standard_normal((S, shape.H))
    cfg = Qwen2Config(hidden_size=shape.H, num_attention_heads=shape.Hq, num_key_value_heads=shape.Hkv,
                      intermediate_size=shape.I, num_hidden_layers=1, rope_theta=shape.rope_base,
                      rms_norm_eps=shape.eps, vocab_size=8, max_position_embeddings=4096)
    cfg._attn_implementation = "eager"
    layer = Qwen2DecoderLayer(cfg, 0).double()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        load_qwen2_layer(layer, shape, W, bias)
        x = t(emb)[None]
        pos = torch.arange(5, 5 + S)[None]
        cos, sin = Qwen2RotaryEmbedding(cfg)(x, pos)
        mask = torch.full((S, S), float("-inf"), dtype=torch.float64).triu(1)[None, None]
        ref = layer(x, attention_mask=mask, position_ids=pos,
                    position_embeddings=(cos.double(), sin.double()))
        ref = (ref[0] if isinstance(ref, tuple) else ref)[0].numpy()
    req = syn.Request([syn.Segment(0, S, False)], 0, pos_start=5)
    got = orc.full_prefill(shape, [W], emb, req, orc.store_exact)[0]["h"]
    # the library builds cos/sin in float32, hence 1e-6 rather than 1e-12
    np.testing.assert_allclose(got, ref, atol=2e-6, rtol=0)


# ------------------------------------------------------------------------------------------
# Qwen3-VL-shaped variant: per-head q/k RMSNorm and interleaved 3-axis RoPE
# ------------------------------------------------------------------------------------------
def q3_setup(d=0):
    """text 7 | image 4 x 6 | text 5 | image 3 x 3 | text 6 with grid position ids, all ids moved by d."""
    shape = syn.SHAPES["tiny_q3"]
    parts = [("text", 7), ("image", 4, 6), ("text", 5), ("image", 3, 3), ("text", 6)]
    pos3 = syn.grid_positions(parts, start=d)
    segs, at, crow = [], 0, 0
    for prt in parts:
        n = prt[1] if prt[0] == "text" else prt[1] * prt[2]
        if prt[0] == "image":
            segs.append(syn.Segment(at, n, True, int(syn.grid_positions(parts)[at, 0]), crow))   # cached at shift 0
            crow += n
        else:
            segs.append(syn.Segment(at, n, False))
        at += n
    req = syn.Request(segs, 0, 0, pos3)
    W = [syn.layer_weights(shape, 41, l) for l in range(2)]
    emb = np.random.default_rng(42).standard_normal((at, shape.H))
    return shape, req, W, emb


def test_grid_positions_layout():
    p = syn.grid_positions([("text", 3), ("image", 2, 3), ("text", 2)], start=10)
    want = [[10, 10, 10], [11, 11, 11], [12, 12, 12],
            [13, 13, 13], [13, 13, 14], [13, 13, 15], [13, 14, 13], [13, 14, 14], [13, 14, 15],
            [16, 16, 16], [17, 17, 17]]
    np.testing.assert_array_equal(p, want)


def test_rope_axes_vs_transformers_interleaved_mrope():
    from transformers.models.qwen3_vl.modeling_qwen3_vl import Qwen3VLTextRotaryEmbedding
    for D, section in ((128, (24, 20, 20)), (64, (12, 10, 10)), (64, (16, 8, 8))):
        freqs = torch.stack([torch.full((1, 2, D // 2), float(a)) for a in range(3)])    # axis id as the value
        got = Qwen3VLTextRotaryEmbedding.apply_interleaved_mrope(None, freqs.clone(), list(section))[0, 0].numpy()
        np.testing.assert_array_equal(orc.rope_axes(D, section), got.astype(np.int64))
    np.testing.assert_array_equal(orc.rope_axes(8, ()), [0, 0, 0, 0])
    # one id on all axes is ordinary RoPE whatever the section
    x = np.random.default_rng(5).standard_normal((3, 2, 64))
    p = np.array([3, 17, 400])
    np.testing.assert_array_equal(orc.rope_rotate(x, np.stack([p, p, p], 1), 1e4, (12, 10, 10)), orc.rope_rotate(x, p, 1e4))


def test_full_prefill_layer_vs_transformers_qwen3_vl():
    """Oracle layer with q/k norm and 3-axis positions against the library's Qwen3-VL text decoder layer (fp64)."""
    from transformers.models.qwen3_vl.modeling_qwen3_vl import (Qwen3VLTextConfig, Qwen3VLTextDecoderLayer,
                                                                Qwen3VLTextRotaryEmbedding)
    shape, req, Ws, emb = q3_setup(d=3)
    W = Ws[0]
    S = emb.shape[0]
    cfg = Qwen3VLTextConfig(hidden_size=shape.H, num_attention_heads=shape.Hq, num_key_value_heads=shape.Hkv,
                            head_dim=shape.D, intermediate_size=shape.I, num_hidden_layers=1, rms_norm_eps=shape.eps,
                            vocab_size=8, max_position_embeddings=4096, attention_bias=False,
                            rope_parameters={"rope_type": "default", "rope_theta": shape.rope_base,
                                             "mrope_section": list(shape.mrope_section)})
    cfg._attn_implementation = "eager"
    layer = Qwen3VLTextDecoderLayer(cfg, 0).double()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    Hq, Hkv, D = shape.Hq, shape.Hkv, shape.D
    with torch.no_grad():
        wq, wk, wv = np.split(W["w_qkv"], [Hq * D, (Hq + Hkv) * D], axis=0)
        layer.self_attn.q_proj.weight.copy_(t(wq))
        layer.self_attn.k_proj.weight.copy_(t(wk))
        layer.self_attn.v_proj.weight.copy_(t(wv))
        layer.self_attn.o_proj.weight.copy_(t(W["w_o"]))
        layer.self_attn.q_norm.weight.copy_(t(W["w_qnorm"]))
        layer.self_attn.k_norm.weight.copy_(t(W["w_knorm"]))
        layer.mlp.gate_proj.weight.copy_(t(W["w_gate_up"][:shape.I]))
        layer.mlp.up_proj.weight.copy_(t(W["w_gate_up"][shape.I:]))
        layer.mlp.down_proj.weight.copy_(t(W["w_down"]))
        layer.input_layernorm.weight.copy_(t(W["w_ln1"]))
        layer.post_attention_layernorm.weight.copy_(t(W["w_ln2"]))
        x = t(emb)[None]
        pos = torch.from_numpy(req.pos3.T.copy())[:, None, :]                    # [3, batch, S]
        cos, sin = Qwen3VLTextRotaryEmbedding(cfg)(x, pos)
        mask = torch.full((S, S), float("-inf"), dtype=torch.float64).triu(1)[None, None]
        ref = layer(x, attention_mask=mask, position_ids=pos, position_embeddings=(cos.double(), sin.double()))
        ref = (ref[0] if isinstance(ref, tuple) else ref)
        ref = ref[0].numpy() if ref.dim() == 3 else ref.numpy()
    got = orc.full_prefill(shape, [W], emb, req, orc.store_exact)[0]["h"]
    np.testing.assert_allclose(got, ref, atol=2e-6, rtol=0)                        # the library's cos/sin are float32
    # the norm and the axis layout matter: dropping either moves the result
    no_norm = dict(W, w_qnorm=None, w_knorm=None)
    assert np.max(np.abs(orc.full_prefill(shape, [no_norm], emb, req, orc.store_exact)[0]["h"] - ref)) > 1e-3
    flat = syn.Request(req.segments, 0, 0, np.repeat(req.pos3[:, :1], 3, axis=1))
    assert np.max(np.abs(orc.full_prefill(shape, [W], emb, flat, orc.store_exact)[0]["h"] - ref)) > 1e-4


@pytest.mark.parametrize("d", [0, 19, -3])
def test_three_axis_reuse_equals_full_prefill(d):
    """The limits that fix the method also hold with 3-axis ids: a cache taken from a full prefill of
    the same prompt, every id moved by d on all axes, nothing or little recomputed."""
    shape, req0, W, emb = q3_setup(d=0)
    full = orc.full_prefill(shape, W, emb, req0, orc.store_exact)
    cache = cache_from_full_prefill(shape, W, emb, req0, full)
    _, moved, _, _ = q3_setup(d=d)
    for counts in ([img_counts(req0, 0)] * 2, [img_counts(req0, 5), img_counts(req0, 2)], [img_counts(req0, None)] * 2):
        sel = orc.selective_prefill(shape, W, emb, moved, counts, cache, orc.store_exact)
        for l in range(2):
            np.testing.assert_allclose(sel[l]["h"], full[l]["h"][sel[l]["slots"]], atol=1e-9)
    # moving the axes by different amounts is not a reuse the method covers: the temporal shift alone is applied
    bad = syn.Request(moved.segments, 0, 0, moved.pos3 + np.array([0, 1, 0]))
    if d != 0:
        sel = orc.selective_prefill(shape, W, emb, bad, [img_counts(req0, 0)] * 2, cache, orc.store_exact)
        assert np.max(np.abs(sel[-1]["h"] - full[-1]["h"][sel[-1]["slots"]])) > 1e-6


# ------------------------------------------------------------------------------------------
# first output token: final norm + output matrix + greedy choice
# ------------------------------------------------------------------------------------------
def test_first_token_vs_transformers_qwen2_causal_lm():
    """Whole stack: two oracle layers of full prefill, then the first-token head, against the
    library's Qwen2ForCausalLM with the same weights (scores of the last position, fp64)."""
    from transformers import Qwen2Config, Qwen2ForCausalLM

    shape = syn.SHAPES["tiny_bias"]
    Ws = [syn.layer_weights(shape, 21, l) for l in range(shape.L)]
    Wh = syn.head_weights(shape, 21)
    S = 29
    emb = np.random.default_rng(22).standard_normal((S, shape.H))
    cfg = Qwen2Config(hidden_size=shape.H, num_attention_heads=shape.Hq, num_key_value_heads=shape.Hkv,
                      intermediate_size=shape.I, num_hidden_layers=shape.L, rope_theta=shape.rope_base,
                      rms_norm_eps=shape.eps, vocab_size=shape.vocab, max_position_embeddings=4096,
                      tie_word_embeddings=False)
    cfg._attn_implementation = "eager"
    model = Qwen2ForCausalLM(cfg).double().eval()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        for l in range(shape.L):
            load_qwen2_layer(model.model.layers[l], shape, Ws[l], True)
        model.model.norm.weight.copy_(t(Wh["w_norm_f"]))
        model.lm_head.weight.copy_(t(Wh["w_lm"]))
        ref = model(inputs_embeds=t(emb)[None], position_ids=torch.arange(S)[None]).logits[0, -1].numpy()
    req = syn.Request([syn.Segment(0, S, False)], 0)
    h = orc.full_prefill(shape, Ws, emb, req, orc.store_exact)[-1]["h"]
    got = orc.first_token_logits(shape, Wh, h[-1:], orc.store_exact)[0]
    assert got.shape == (shape.vocab,)
    np.testing.assert_allclose(got, ref, atol=5e-6, rtol=0)     # the library's cos/sin are float32
    assert orc.first_token(got[None])[0] == int(np.argmax(ref))


def test_first_token_head_closed_forms():
    shape = syn.SHAPES["tiny"]
    H = shape.H
    rng = np.random.default_rng(23)
    x = rng.standard_normal((3, H))
    # unit norm weight, output matrix = signed unit rows: score v is +-x[v] / rms(x)
    Wh = {"w_norm_f": np.ones(H), "w_lm": np.concatenate([np.eye(H), -np.eye(H)])}
    lg = orc.first_token_logits(shape, Wh, x, orc.store_exact)
    rms = np.sqrt(np.mean(x * x, axis=1, keepdims=True) + shape.eps)
    np.testing.assert_allclose(lg[:, :H], x / rms, atol=1e-13)
    np.testing.assert_allclose(lg[:, H:], -x / rms, atol=1e-13)
    tok = orc.first_token(lg)
    j = np.argmax(np.abs(x), axis=1)
    want = np.where(x[np.arange(3), j] > 0, j, j + H)
    np.testing.assert_array_equal(tok, want)
    # the norm weight scales column-wise before the product (not after)
    w = rng.uniform(0.5, 2.0, H)
    Wh2 = {"w_norm_f": w, "w_lm": rng.standard_normal((7, H))}
    lg2 = orc.first_token_logits(shape, Wh2, x, orc.store_exact)
    np.testing.assert_allclose(lg2, ((x / rms) * w) @ Wh2["w_lm"].T, atol=1e-12)
    # scaling a row leaves its scores unchanged up to eps (RMSNorm), so it keeps its token
    lg3 = orc.first_token_logits(shape, Wh2, 3.0 * x, orc.store_exact)
    np.testing.assert_allclose(lg3, lg2, rtol=2e-6, atol=1e-9)


def test_first_token_ties_take_lowest_index():
    lg = np.array([[0.0, 2.0, 2.0, -1.0], [5.0, 5.0, 5.0, 5.0], [-3.0, -2.0, -2.0, -2.0]])
    np.testing.assert_array_equal(orc.first_token(lg), [1, 0, 1])


def test_first_token_bf16_contract_rounds_inputs_not_scores():
    shape = syn.SHAPES["tiny_bf16"]
    Wh = syn.head_weights(shape, 24)
    x = np.random.default_rng(25).standard_normal((2, shape.H))
    lg = orc.first_token_logits(shape, Wh, x, orc.store_bf16)
    xn = orc.store_bf16(orc.rmsnorm(orc.store_bf16(x), orc.store_bf16(Wh["w_norm_f"]), shape.eps))
    np.testing.assert_array_equal(lg, xn @ orc.store_bf16(Wh["w_lm"]).T)
    assert np.any(lg != orc.store_bf16(lg))          # scores themselves stay unrounded


# ------------------------------------------------------------------------------------------
# selective recompute reduces to full prefill in the two limits the paper fixes
# ------------------------------------------------------------------------------------------
def random_cache(shape, rows, L, seed):
    rng = np.random.default_rng(seed)
    return [(rng.standard_normal((rows, shape.Hkv, shape.D)), rng.standard_normal((rows, shape.Hkv, shape.D)))
            for _ in range(L)]


@pytest.mark.parametrize("store", ["f32", "bf16"])
def test_rate_one_equals_full_prefill(store):
    """r = 1.0 is 'full-recompute' (accuracy tables, last column): every cached value is
    overwritten, so any cache content gives the full-prefill result."""
    shape, req, W, emb, crow = tiny_setup(parts=((5, False), (20, True), (3, False), (9, True), (4, False)))
    st = orc.STORE[store]
    cache = random_cache(shape, crow, len(W), 3)
    counts = [img_counts(req, None)] * len(W)
    sel = orc.selective_prefill(shape, W, emb, req, counts, cache, st)
    full = orc.full_prefill(shape, W, emb, req, st)
    for a, b in zip(sel, full):
        np.testing.assert_array_equal(a["slots"], b["slots"])
        np.testing.assert_array_equal(a["h"], b["h"])
        np.testing.assert_array_equal(a["K"], b["K"])
        np.testing.assert_array_equal(a["V"], b["V"])


def cache_from_full_prefill(shape, W, emb, req, full):
    """Cache pools holding the image tokens' K/V exactly as a full prefill produced them."""
    rows = sum(s.length for s in req.segments if s.is_image)
    cache = []
    for l in range(len(W)):
        Kc = np.zeros((rows, shape.Hkv, shape.D))
        Vc = np.zeros_like(Kc)
        for s in req.segments:
            if s.is_image:
                Kc[s.cache_row:s.cache_row + s.length] = full[l]["K"][s.start:s.start + s.length]
                Vc[s.cache_row:s.cache_row + s.length] = full[l]["V"][s.start:s.start + s.length]
        cache.append((Kc, Vc))
    return cache


def test_exact_prefix_reuse_rate_zero_equals_full_prefill():
    """Sec. 1 / 2.2: with an exactly matching prefix, reuse is lossless.  Cache = the image K/V of
    a full prefill of the same request, delta 0, nothing recomputed: all text rows equal full prefill."""
    shape, req, W, emb, crow = tiny_setup()
    full = orc.full_prefill(shape, W, emb, req, orc.store_exact)
    cache = cache_from_full_prefill(shape, W, emb, req, full)
    sel = orc.selective_prefill(shape, W, emb, req, [img_counts(req, 0)] * len(W), cache, orc.store_exact)
    for l in range(len(W)):
        sl = sel[l]["slots"]
        assert len(sl) == 48           # 32 + 16 text rows, no image rows
        np.testing.assert_allclose(sel[l]["h"], full[l]["h"][sl], atol=1e-12)
        np.testing.assert_allclose(sel[l]["K"], full[l]["K"], atol=1e-12)


@pytest.mark.parametrize("d", [32, -7, 4097])
def test_shifted_reuse_equals_full_prefill(d):
    """Position-independent reuse (Sec. 2.2, 4.2): the whole request moves by d positions, the
    cache (rotated at the old positions) is re-rotated by d.  RoPE attention only sees position
    differences, so the text rows still equal the full prefill.  Pins the direction of the
    key re-rotation end to end: rotating by -d instead fails this test."""
    shape, req, W, emb, crow = tiny_setup()
    full = orc.full_prefill(shape, W, emb, req, orc.store_exact)
    cache = cache_from_full_prefill(shape, W, emb, req, full)
    moved = syn.Request(req.segments, 0, pos_start=d)
    sel = orc.selective_prefill(shape, W, emb, moved, [img_counts(req, 0)] * len(W), cache, orc.store_exact)
    for l in range(len(W)):
        np.testing.assert_allclose(sel[l]["h"], full[l]["h"][sel[l]["slots"]], atol=1e-9)
    # a partially recomputed image stays exact too, because recomputed rows see exact inputs
    sel = orc.selective_prefill(shape, W, emb, moved, [img_counts(req, 10), img_counts(req, 4)], cache,
                                orc.store_exact)
    for l in range(len(W)):
        np.testing.assert_allclose(sel[l]["h"], full[l]["h"][sel[l]["slots"]], atol=1e-9)


def test_wrong_direction_shift_is_detected():
    """Negative control on the CPU: a cache re-rotated the wrong way does NOT reproduce full prefill."""
    shape, req, W, emb, crow = tiny_setup()
    full = orc.full_prefill(shape, W, emb, req, orc.store_exact)
    cache = cache_from_full_prefill(shape, W, emb, req, full)
    bad = [(orc.rope_rotate(Kc, np.full(Kc.shape[0], -64), shape.rope_base), Vc) for Kc, Vc in cache]
    moved = syn.Request(req.segments, 0, pos_start=32)
    sel = orc.selective_prefill(shape, W, emb, moved, [img_counts(req, 0)] * len(W), bad, orc.store_exact)
    assert np.max(np.abs(sel[-1]["h"] - full[-1]["h"][sel[-1]["slots"]])) > 1e-4


def test_mismatched_prefix_gives_reuse_error_that_recompute_reduces():
    """Sec. 3.1: a cache built under another prefix carries reuse error.  Recomputing every image
    token removes it entirely (rate 1.0); this only checks the two ends and that error is non-zero
    at rate 0 (the size of the error depends on trained weights and is not pinned)."""
    shape, req, W, emb, crow = tiny_setup()
    emb2 = emb.copy()
    emb2[:32] = np.random.default_rng(9).standard_normal((32, shape.H))
    full = orc.full_prefill(shape, W, emb, req, orc.store_exact)
    other = orc.full_prefill(shape, W, emb2, req, orc.store_exact)
    cache = cache_from_full_prefill(shape, W, emb2, req, other)
    sel0 = orc.selective_prefill(shape, W, emb, req, [img_counts(req, 0)] * 2, cache, orc.store_exact)
    sel1 = orc.selective_prefill(shape, W, emb, req, [img_counts(req, None)] * 2, cache, orc.store_exact)
    e0 = np.max(np.abs(sel0[-1]["h"] - full[-1]["h"][sel0[-1]["slots"]]))
    e1 = np.max(np.abs(sel1[-1]["h"] - full[-1]["h"][sel1[-1]["slots"]]))
    assert e0 > 1e-8 and e1 == 0.0


def test_increasing_rate_is_rejected():
    """Sec. 4.1 last paragraph: a deeper layer cannot recompute a token the layer above dropped."""
    shape, req, W, emb, crow = tiny_setup()
    cache = random_cache(shape, crow, 2, 0)
    with pytest.raises(ValueError):
        orc.selective_prefill(shape, W, emb, req, [img_counts(req, 2), img_counts(req, 3)], cache,
                              orc.store_exact)


# ------------------------------------------------------------------------------------------
# token selection (Sec. 4.2)
# ------------------------------------------------------------------------------------------
def test_leading_count_is_floor_r_times_T():
    for k in range(0, 501, 7):
        for T in (1, 49, 256, 1024, 1296):
            assert orc.leading_count(k, T) == math.floor(k * T / 500 + 1e-12)
    # counts the workloads rely on
    assert orc.leading_count(10, 1024) == 20 and orc.leading_count(25, 1024) == 51
    assert orc.leading_count(10, 1296) == 25 and orc.leading_count(25, 1296) == 64
    assert orc.leading_count(500, 777) == 777 and orc.leading_count(0, 777) == 0


def test_selected_slots_structure():
    wl = syn.make_workload("c3")
    req = wl.requests[0]
    prev = None
    for k in (150, 150, 40, 3, 0):
        counts = orc.image_counts(req.segments, k=k)
        sl = orc.select_slots(req.segments, counts)
        assert np.all(np.diff(sl) > 0)
        n_text = sum(s.length for s in req.segments if not s.is_image)
        assert len(sl) == n_text + sum(counts)
        for s, c in zip([s for s in req.segments if s.is_image], counts):
            inside = sl[(sl >= s.start) & (sl < s.start + s.length)]
            np.testing.assert_array_equal(inside, np.arange(s.start, s.start + c))
        if prev is not None:
            assert set(sl.tolist()) <= set(prev.tolist())
        reused, rows, old = orc.reused_slots(req.segments, counts)
        assert len(reused) + len(sl) == req.S
        assert not set(reused.tolist()) & set(sl.tolist())
        prev = sl


# ------------------------------------------------------------------------------------------
# layer-rate allocation (Sec. 4.1 Eq. 6-9)
# ------------------------------------------------------------------------------------------
def feasible(k, budget, G):
    k = list(k)
    return sum(k) <= budget and all(0 <= v <= G for v in k) and all(a >= b for a, b in zip(k, k[1:]))


def test_planner_feasibility_random_tables():
    rng = np.random.default_rng(0)
    for trial in range(30):
        L, G = int(rng.integers(1, 12)), int(rng.integers(1, 20))
        sens = rng.random((L, G + 1))           # arbitrary, not even monotone
        B = int(rng.integers(0, L * G + 5))
        k = orc.plan_layer_rates(sens, B)
        assert feasible(k, B, G)


def test_planner_closed_forms():
    L, G = 6, 10
    sens = syn.sensitivity_table(L, G, 3)
    assert list(orc.plan_layer_rates(sens, 0)) == [0] * L
    assert list(orc.plan_layer_rates(sens, L * G)) == [G] * L
    assert list(orc.plan_layer_rates(sens, L * G + 50)) == [G] * L
    # identical strictly convex rows: steps are dealt round-robin from the shallowest layer
    row = 1.0 / (1.0 + np.arange(G + 1))
    same = np.tile(row, (L, 1))
    for B in (1, 5, 6, 7, 23, 59):
        want = [B // L + (1 if i < B % L else 0) for i in range(L)]
        assert list(orc.plan_layer_rates(same, B)) == want
    # a flat table offers no gain: nothing is spent
    assert list(orc.plan_layer_rates(np.ones((L, G + 1)), 17)) == [0] * L
    # budget conversion: mean 5 % over 28 layers = 700 grid steps, 3 % over 80 layers = 1200
    assert orc.budget_steps_from_mean_rate(500, 28) == 700
    assert orc.budget_steps_from_mean_rate(300, 80) == 1200


def exhaustive_optimum(sens, B):
    L, G = sens.shape[0], sens.shape[1] - 1
    best = None
    for k in itertools.product(range(G + 1), repeat=L):
        if not feasible(k, B, G):
            continue
        val = sum(sens[i][k[i]] for i in range(L))
        if best is None or val < best - 1e-15:
            best = val
    return best


def test_planner_matches_exhaustive_optimum_on_convex_ordered_tables():
    """With diminishing returns per layer and gains ordered by depth the greedy solves Eq. 6-9
    exactly; checked against enumeration of every monotone sequence (L <= 4, G <= 6)."""
    rng = np.random.default_rng(5)
    for trial in range(12):
        L, G = int(rng.integers(2, 5)), int(rng.integers(2, 7))
        w = np.sort(rng.random(L) + 0.1)[::-1] * 3.0
        sens = w[:, None] / (1.0 + np.arange(G + 1))[None, :]
        for B in range(0, L * G + 1, max(1, (L * G) // 5)):
            k = orc.plan_layer_rates(sens, B)
            val = sum(sens[i][k[i]] for i in range(L))
            assert abs(val - exhaustive_optimum(sens, B)) < 1e-12


def test_planner_weights_early_layers_on_benchmark_table():
    sens = syn.sensitivity_table(28, 150, 1)
    k = orc.plan_layer_rates(sens, 700)
    assert feasible(k, 700, 150) and int(k.sum()) == 700
    assert k[0] > k[-1]


def objective(sens, k):
    return sum(sens[i][k[i]] for i in range(len(k)))


def test_block_planner_feasible_and_never_worse_than_starting_point():
    rng = np.random.default_rng(1)
    for trial in range(30):
        L, G = int(rng.integers(1, 12)), int(rng.integers(1, 20))
        sens = rng.random((L, G + 1))
        B = int(rng.integers(0, L * G + 5))
        k = orc.plan_layer_rates_blocks(sens, B)
        assert feasible(k, B, G)
        assert objective(sens, k) <= objective(sens, [0] * L) + 1e-15      # every move has positive gain


def test_block_planner_closed_forms():
    L, G = 5, 8
    row = 1.0 / (1.0 + np.arange(G + 1))
    same = np.tile(row, (L, 1))
    assert list(orc.plan_layer_rates_blocks(same, 0)) == [0] * L
    assert list(orc.plan_layer_rates_blocks(same, L * G + 9)) == [G] * L
    assert list(orc.plan_layer_rates_blocks(np.ones((L, G + 1)), 17)) == [0] * L
    # identical convex rows: gain per step of a run equals that of its first layer alone, ties go to the
    # smallest j, so steps are dealt exactly as by the one-step greedy
    for B in (1, 4, 5, 6, 23, 39):
        np.testing.assert_array_equal(orc.plan_layer_rates_blocks(same, B), orc.plan_layer_rates(same, B))
    # A first layer that gains nothing (its cached keys/values are exact) blocks the one-step greedy at zero;
    # runs carry it along.  Layers 1, 2 gain 1.0 and 0.6 per step, layer 0 nothing: the run 0..1 gains 0.5 per
    # step, the run 0..2 gains 1.6 / 3 per step > 0.5, so all three rise together while the budget lasts.
    flat0 = np.stack([np.zeros(G + 1), -1.0 * np.arange(G + 1), -0.6 * np.arange(G + 1)])
    assert list(orc.plan_layer_rates(flat0, 12)) == [0, 0, 0]
    assert list(orc.plan_layer_rates_blocks(flat0, 12)) == [4, 4, 4]
    assert list(orc.plan_layer_rates_blocks(flat0, 14)) == [5, 5, 4]      # 2 steps left: the run 0..1
    assert list(orc.plan_layer_rates_blocks(flat0, 13)) == [4, 4, 4]      # 1 step left: layer 0 alone gains nothing


def test_block_planner_reaches_the_exhaustive_optimum_where_the_one_step_greedy_cannot():
    """Tables whose first layer is flat and whose other layers are convex with gains ordered by depth: the
    optimum raises layer 0 only as far as the layers behind it need; enumeration over every monotone sequence
    (L <= 4, G <= 5) agrees with the run-based greedy whenever the budget is a multiple of what a full run costs."""
    rng = np.random.default_rng(7)
    hits = 0
    for trial in range(10):
        L, G = int(rng.integers(2, 5)), int(rng.integers(2, 6))
        w = np.sort(rng.random(L - 1) + 0.1)[::-1] * 3.0
        sens = np.concatenate([np.zeros((1, G + 1)), w[:, None] / (1.0 + np.arange(G + 1))[None, :]])
        for B in range(0, L * G + 1):
            k = orc.plan_layer_rates_blocks(sens, B)
            assert feasible(k, B, G)
            best = exhaustive_optimum(sens, B)
            val = objective(sens, k)
            assert val >= best - 1e-12
            assert objective(sens, orc.plan_layer_rates(sens, B)) == objective(sens, [0] * L)   # stuck at zero
            if B >= 2:
                assert val < objective(sens, [0] * L)
            hits += abs(val - best) < 1e-12
    assert hits > 60           # optimal in most cases; the greedy is an approximation (Sec. 4.1)
    # on convex tables ordered by depth (no flat layer) both greedies solve the problem exactly
    for trial in range(8):
        L, G = int(rng.integers(2, 5)), int(rng.integers(2, 6))
        w = np.sort(rng.random(L) + 0.1)[::-1] * 3.0
        sens = w[:, None] / (1.0 + np.arange(G + 1))[None, :]
        for B in range(0, L * G + 1, 3):
            assert abs(objective(sens, orc.plan_layer_rates_blocks(sens, B)) - exhaustive_optimum(sens, B)) < 1e-12


# ---- mixture-of-experts MLP (Qwen3-VL-30B-A3B-shaped layer) -----------------------------------

def test_route_top_k_by_hand():
    """Scores 0, ln 2, ln 4 -> probabilities 1/7, 2/7, 4/7; the two largest renormalised are 2/3 and 1/3."""
    idx, w = orc.route_top_k(np.array([[0.0, np.log(2.0), np.log(4.0)], [np.log(4.0), 0.0, np.log(2.0)]]), 2)
    np.testing.assert_array_equal(idx, [[2, 1], [0, 2]])
    np.testing.assert_allclose(w, [[2 / 3, 1 / 3], [2 / 3, 1 / 3]], rtol=1e-15)
    # equal scores: the lower expert index comes first
    idx, w = orc.route_top_k(np.array([[1.0, 3.0, 3.0, 1.0, 3.0]]), 2)
    np.testing.assert_array_equal(idx, [[1, 2]])
    np.testing.assert_allclose(w, [[0.5, 0.5]])
    # top_k = all experts: the weights are the softmax itself
    z = np.random.default_rng(0).standard_normal((4, 6))
    idx, w = orc.route_top_k(z, 6)
    p = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    np.testing.assert_allclose(w, np.take_along_axis(p, idx, 1), rtol=1e-14)
    assert np.all(np.diff(w, axis=1) <= 0)


def moe_setup(n=37):
    shape = syn.SHAPES["tiny_moe"]
    W = syn.layer_weights(shape, 51, 0)
    n2 = np.random.default_rng(52).standard_normal((n, shape.H))
    return shape, W, n2


def test_moe_block_vs_transformers():
    from transformers.models.qwen3_vl_moe.modeling_qwen3_vl_moe import Qwen3VLMoeTextConfig, Qwen3VLMoeTextSparseMoeBlock
    shape, W, n2 = moe_setup()
    cfg = Qwen3VLMoeTextConfig(hidden_size=shape.H, moe_intermediate_size=shape.I, num_experts=shape.n_experts,
                               num_experts_per_tok=shape.top_k, hidden_act="silu")
    blk = Qwen3VLMoeTextSparseMoeBlock(cfg).double()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    with torch.no_grad():
        blk.gate.weight.copy_(t(W["w_router"]))
        blk.experts.gate_up_proj.copy_(t(W["w_gate_up"]))
        blk.experts.down_proj.copy_(t(W["w_down"]))
        ref = blk(t(n2)[None])[0].numpy()
        _, ref_w, ref_idx = blk.gate(t(n2))
    got = orc.moe_mlp(shape, W, n2, orc.store_exact)
    np.testing.assert_array_equal(np.sort(got["moe_idx"], 1), np.sort(ref_idx.numpy(), 1))
    np.testing.assert_allclose(np.sort(got["moe_w"], 1), np.sort(ref_w.numpy(), 1), rtol=1e-6)   # the library's softmax is float32
    np.testing.assert_allclose(got["mlp"], ref, atol=1e-8, rtol=1e-6)
    assert len(np.unique(got["moe_idx"])) == shape.n_experts          # the sample exercises every expert
    # without the renormalisation, or with gate and up swapped, the result moves
    raw = orc.route_top_k(orc.linear(n2, W["w_router"]), shape.n_experts)
    p_sel = np.stack([raw[1][i][np.isin(raw[0][i], got["moe_idx"][i])] for i in range(len(n2))])
    unnorm = orc.moe_mlp(shape, W, n2, orc.store_exact, forced={"moe_w": p_sel})
    assert np.max(np.abs(unnorm["mlp"] - ref)) > 1e-3
    swapped = dict(W, w_gate_up=np.concatenate([W["w_gate_up"][:, shape.I:], W["w_gate_up"][:, :shape.I]], axis=1))
    assert np.max(np.abs(orc.moe_mlp(shape, swapped, n2, orc.store_exact)["mlp"] - ref)) > 1e-3


def test_moe_with_identical_experts_is_the_dense_mlp():
    """The weights sum to one, so experts that all hold the same matrices give the ordinary SwiGLU MLP,
    whatever the router does."""
    shape, W, n2 = moe_setup()
    same = dict(W, w_gate_up=np.repeat(W["w_gate_up"][:1], shape.n_experts, 0), w_down=np.repeat(W["w_down"][:1], shape.n_experts, 0))
    got = orc.moe_mlp(shape, same, n2, orc.store_exact)["mlp"]
    gu = n2 @ W["w_gate_up"][0].T.astype(np.float64)
    dense = (torch.nn.functional.silu(torch.from_numpy(gu[:, :shape.I])).numpy() * gu[:, shape.I:]) @ W["w_down"][0].T.astype(np.float64)
    np.testing.assert_allclose(got, dense, atol=1e-12, rtol=1e-10)
    # one expert per token and a router that can only pick expert 3: that expert's MLP alone
    one = dataclasses.replace(shape, top_k=1)
    router = np.zeros_like(W["w_router"])
    router[3] = 1.0
    pos = np.abs(n2)                                                 # positive rows: expert 3's score is the largest
    got = orc.moe_mlp(one, dict(W, w_router=router), pos, orc.store_exact)
    assert np.all(got["moe_idx"] == 3) and np.all(got["moe_w"] == 1.0)
    gu = pos @ W["w_gate_up"][3].T.astype(np.float64)
    want = (torch.nn.functional.silu(torch.from_numpy(gu[:, :shape.I])).numpy() * gu[:, shape.I:]) @ W["w_down"][3].T.astype(np.float64)
    np.testing.assert_allclose(got["mlp"], want, atol=1e-12, rtol=1e-10)


def test_full_prefill_moe_layer_vs_transformers():
    """Oracle layer (q/k norm, 3-axis positions, mixture-of-experts MLP) against the library's Qwen3-VL-MoE text decoder layer (fp64)."""
    from transformers.models.qwen3_vl_moe.modeling_qwen3_vl_moe import (Qwen3VLMoeTextConfig, Qwen3VLMoeTextDecoderLayer,
                                                                        Qwen3VLMoeTextRotaryEmbedding)
    _, req, _, emb = q3_setup(d=3)
    shape = syn.SHAPES["tiny_moe"]
    W = syn.layer_weights(shape, 53, 0)
    S = emb.shape[0]
    cfg = Qwen3VLMoeTextConfig(hidden_size=shape.H, num_attention_heads=shape.Hq, num_key_value_heads=shape.Hkv,
                               head_dim=shape.D, moe_intermediate_size=shape.I, num_experts=shape.n_experts,
                               num_experts_per_tok=shape.top_k, num_hidden_layers=1, rms_norm_eps=shape.eps,
                               vocab_size=8, max_position_embeddings=4096, attention_bias=False, hidden_act="silu",
                               rope_parameters={"rope_type": "default", "rope_theta": shape.rope_base,
                                                "mrope_section": list(shape.mrope_section)})
    cfg._attn_implementation = "eager"
    layer = Qwen3VLMoeTextDecoderLayer(cfg, 0).double()
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    Hq, Hkv, D = shape.Hq, shape.Hkv, shape.D
    with torch.no_grad():
        wq, wk, wv = np.split(W["w_qkv"], [Hq * D, (Hq + Hkv) * D], axis=0)
        layer.self_attn.q_proj.weight.copy_(t(wq))
        layer.self_attn.k_proj.weight.copy_(t(wk))
        layer.self_attn.v_proj.weight.copy_(t(wv))
        layer.self_attn.o_proj.weight.copy_(t(W["w_o"]))
        layer.self_attn.q_norm.weight.copy_(t(W["w_qnorm"]))
        layer.self_attn.k_norm.weight.copy_(t(W["w_knorm"]))
        layer.mlp.gate.weight.copy_(t(W["w_router"]))
        layer.mlp.experts.gate_up_proj.copy_(t(W["w_gate_up"]))
        layer.mlp.experts.down_proj.copy_(t(W["w_down"]))
        layer.input_layernorm.weight.copy_(t(W["w_ln1"]))
        layer.post_attention_layernorm.weight.copy_(t(W["w_ln2"]))
        x = t(emb)[None]
        pos = torch.from_numpy(req.pos3.T.copy())[:, None, :]
        cos, sin = Qwen3VLMoeTextRotaryEmbedding(cfg)(x, pos)
        mask = torch.full((S, S), float("-inf"), dtype=torch.float64).triu(1)[None, None]
        ref = layer(x, attention_mask=mask, position_ids=pos, position_embeddings=(cos.double(), sin.double()))
        ref = (ref[0] if isinstance(ref, tuple) else ref)
        ref = ref[0].numpy() if ref.dim() == 3 else ref.numpy()
    got = orc.full_prefill(shape, [W], emb, req, orc.store_exact)[0]["h"]
    np.testing.assert_allclose(got, ref, atol=2e-6, rtol=0)


# ---- layer-wise sensitivity measurement (Sec. 3.2, Eq. 5) --------------------------------------

def profile_setup(L=2, same_prompt=False, shift=5):
    shape = dataclasses.replace(syn.SHAPES["tiny"], L=L)
    W = [syn.layer_weights(shape, 61, l) for l in range(L)]
    head = syn.head_weights(shape, 61)
    smp = syn.profile_sample(shape, 62, t_cache_text=9 + shift, t_text=9, t_image=40, t_answer=6)
    if same_prompt:     # the cache is built under the evaluated prompt's own text
        smp = dict(smp, cache_emb=smp["emb"][:9 + 40].copy(),
                   cache_request=syn.Request([syn.Segment(0, 9, False), syn.Segment(9, 40, True, 9, 0)], 0),
                   request=syn.Request([syn.Segment(0, 9, False), syn.Segment(9, 40, True, 9, 0), syn.Segment(49, 6, False)], 0))
    return shape, W, head, smp


def test_sensitivity_is_zero_when_the_cache_matches():
    """A cache built under the same text and positions holds exactly the keys/values a forward pass computes,
    so no layer and no rate changes the scores."""
    shape, W, head, smp = profile_setup(same_prompt=True)
    S = orc.sensitivity_profile(shape, W, head, [smp], [0, 100, 500], orc.store_exact)
    assert S.shape == (2, 3)
    np.testing.assert_allclose(S, 0.0, atol=1e-24)


def test_sensitivity_mismatched_cache():
    shape, W, head, smp = profile_setup(L=3)
    steps = [0, 150, 500]
    S = orc.sensitivity_profile(shape, W, head, [smp], steps, orc.store_exact)
    assert np.all(S[:, 0] > 1e-10)                      # pure reuse of a mismatched cache costs something
    np.testing.assert_allclose(S[:, 0], S[0, 0], rtol=1e-12)      # rate 0: the layer index is immaterial
    # The first layer's keys/values of an image do not depend on the prompt (they come from the image rows
    # alone, re-rotated to the new position), so recomputing there changes nothing ...
    np.testing.assert_allclose(S[0], S[0, 0], rtol=1e-9)
    # ... deeper layers do depend on it, and recomputing ALL image tokens in the last layer restores the scores
    # only if no other layer is mismatched: not so here (layer 1 still is), but it must help
    assert S[2, 2] < S[2, 0] and S[1, 2] != pytest.approx(S[1, 0], rel=1e-3)
    # the mean over samples: the same sample twice gives the same table
    np.testing.assert_allclose(orc.sensitivity_profile(shape, W[:2], head, [smp, smp], steps, orc.store_exact),
                               orc.sensitivity_profile(shape, W[:2], head, [smp], steps, orc.store_exact), rtol=1e-12)


def test_sensitivity_one_and_two_layer_models():
    """One layer: its cached image keys/values equal the fresh ones, every entry is zero.  Two layers: only layer 1
    is mismatched, so recomputing all image tokens there is the original forward pass (S = 0).  And on the text
    rows the measurement pass of a one-layer model is the fast path (image rows' outputs feed nothing)."""
    shape, W, head, smp = profile_setup(L=1)
    S = orc.sensitivity_profile(shape, W, head, [smp], [0, 500], orc.store_exact)
    np.testing.assert_allclose(S, 0.0, atol=1e-24)
    shape2, W2, head2, smp2 = profile_setup(L=2)
    S2 = orc.sensitivity_profile(shape2, W2, head2, [smp2], [0, 250, 500], orc.store_exact)
    assert S2[1, 0] > 1e-10 and S2[1, 2] < 1e-24 and 0 < S2[1, 1]
    req = smp["request"]
    full_c = orc.full_prefill(shape, W, smp["cache_emb"], smp["cache_request"], orc.store_exact)
    img = np.arange(14, 54)
    cache = [(full_c[0]["K"][img], full_c[0]["V"][img])]
    for k in (0, 120):
        counts = orc.image_counts(req.segments, k=k)
        h_prof = orc.profile_prefill(shape, W, smp["emb"], req, 0, counts, cache, orc.store_exact)
        sel = orc.selective_prefill(shape, W, smp["emb"], req, [counts], cache, orc.store_exact)[0]
        np.testing.assert_allclose(h_prof[sel["slots"]][-6:], sel["h"][-6:], atol=1e-12)
