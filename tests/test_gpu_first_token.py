"""GPU parity of the first-token head (final RMSNorm + output matrix + greedy choice) against the oracle."""
import numpy as np
import pytest
import torch

import vlc_synth as syn
from oracle import vlc_oracle as orc
import paper_2512_12977_amd as vlc

pytestmark = pytest.mark.gpu
DEV = "cuda"
TD = {"f32": torch.float32, "bf16": torch.bfloat16}
# scores are sums of H products of O(1) x O(0.02) terms accumulated in float; a one-ulp flip of a
# bf16-rounded normed value (the GPU norm runs in float, the oracle in double) moves a score by
# |w| * 2^-8 ~ 1e-4; the fp32 configuration differs only by float accumulation order
# (absolute, relative): the fp32 bound is the stated one, |g - o| <= 1e-5 + 1e-5 |o|
TOL = {"f32": (1e-5, 1e-5), "bf16": (2e-3, 0.0)}


def run_gpu(h, rows, Wh, shape):
    dt = TD[shape.dtype]
    d_h = torch.from_numpy(np.ascontiguousarray(h, dtype=np.float32)).to(DEV).to(dt)
    d_rows = torch.from_numpy(np.ascontiguousarray(rows, dtype=np.int32)).to(DEV)
    d_wn = torch.from_numpy(Wh["w_norm_f"]).to(DEV).to(dt)
    d_wo = torch.from_numpy(Wh["w_lm"]).to(DEV).to(dt)
    m = len(rows)
    logits = torch.full((m, shape.vocab), float("nan"), device=DEV, dtype=torch.float32)
    token = torch.full((m,), -1, device=DEV, dtype=torch.int32)
    code = vlc.VLC_BF16 if shape.dtype == "bf16" else vlc.VLC_F32
    ws = torch.empty(max(256, vlc.vlc_first_token_workspace_bytes(shape.H, m, code)), device=DEV, dtype=torch.uint8)
    vlc.vlc_first_token(d_h, d_rows, shape.eps, d_wn, d_wo, logits, token, ws)
    torch.cuda.synchronize()
    return logits.cpu().numpy().astype(np.float64), token.cpu().numpy().astype(np.int64)


def check(h, rows, Wh, shape, chunk=16384):
    g_logits, g_tok = run_gpu(h, rows, Wh, shape)
    st = orc.STORE[shape.dtype]
    hs = np.asarray(h, dtype=np.float32).astype(np.float64)[np.asarray(rows)]
    tol, rtol = TOL[shape.dtype]
    o_best = np.full(len(rows), -np.inf)
    for v0 in range(0, shape.vocab, chunk):                      # the oracle, a slab of the output matrix at a time
        part = {"w_norm_f": Wh["w_norm_f"], "w_lm": Wh["w_lm"][v0:v0 + chunk]}
        o = orc.first_token_logits(shape, part, hs, st)
        np.testing.assert_allclose(g_logits[:, v0:v0 + chunk], o, atol=tol, rtol=rtol)
        o_best = np.maximum(o_best, o.max(axis=1))
        for r in range(len(rows)):
            if v0 <= g_tok[r] < v0 + chunk:
                g_tok_score = o[r, g_tok[r] - v0]
                assert g_tok_score >= o.max(axis=1)[r] - 2 * tol
    # the choice itself is index work on the float scores the kernel produced: exact, first of equals
    np.testing.assert_array_equal(g_tok, orc.first_token(g_logits))
    # and it is a largest score of the oracle too, up to the score tolerance
    for r in range(len(rows)):
        part = {"w_norm_f": Wh["w_norm_f"], "w_lm": Wh["w_lm"][g_tok[r]:g_tok[r] + 1]}
        assert orc.first_token_logits(shape, part, hs[r:r + 1], st)[0, 0] >= o_best[r] - 2 * tol
    return g_logits, g_tok


@pytest.mark.parametrize("name", ["tiny", "tiny_bf16"])
def test_first_token_small(name):
    shape = syn.SHAPES[name]
    Wh = syn.head_weights(shape, 31)
    h = np.random.default_rng(32).standard_normal((61, shape.H)).astype(np.float32)
    check(h, [60, 3, 17], Wh, shape)
    check(h, [0], Wh, shape)                                      # a single request
    check(h, [5, 9, 60, 1, 2, 33, 34, 35, 8, 7, 6], Wh, shape)    # more than 8 requests: the GEMM path


@pytest.mark.parametrize("seed", range(10))
def test_first_token_random_widths_vocabularies_and_batches(seed):
    """Seeded random heads: H 64-2048 (multiples of 64), vocabularies of 4-9000 entries (multiples of 4, so also fewer
    entries than one tile and than the 64 slices of the greedy choice), 1-70 requests whose rows repeat and come in any order."""
    import dataclasses
    rng = np.random.default_rng(17000 + seed)
    base = syn.SHAPES["tiny_bf16" if seed % 2 else "tiny"]
    shape = dataclasses.replace(base, H=64 * int(rng.integers(1, 33)), vocab=4 * int(rng.integers(1, 2251)))
    Wh = syn.head_weights(shape, 400 + seed)
    n = int(rng.integers(1, 300))
    h = rng.standard_normal((n, shape.H)).astype(np.float32)
    rows = [int(r) for r in rng.integers(0, n, size=int(rng.integers(1, 71)))]
    check(h, rows, Wh, shape)


def test_first_token_equal_scores_take_lowest_index():
    shape = syn.SHAPES["tiny_bf16"]
    Wh = syn.head_weights(shape, 33)
    h = np.random.default_rng(34).standard_normal((5, shape.H)).astype(np.float32)
    _, tok = run_gpu(h, [4], Wh, shape)
    w = Wh["w_lm"].copy()
    v = int(tok[0])
    for dup in (v + 129, (v + 300) % shape.vocab, 2):             # copies of the winning row, other tiles too
        if dup < shape.vocab:
            w[dup] = w[v]
    lg, tok2 = run_gpu(h, [4], {"w_norm_f": Wh["w_norm_f"], "w_lm": w}, shape)
    winners = np.flatnonzero(lg[0] == lg[0].max())
    assert len(winners) >= 2                                      # identical rows give identical scores
    assert tok2[0] == winners[0] == min(2, v)


def test_first_token_empty_batch_is_a_no_op():
    shape = syn.SHAPES["tiny"]
    h = torch.zeros((4, shape.H), device=DEV)
    rows = torch.zeros((0,), device=DEV, dtype=torch.int32)
    logits = torch.zeros((0, shape.vocab), device=DEV)
    token = torch.zeros((0,), device=DEV, dtype=torch.int32)
    ws = torch.empty(256, device=DEV, dtype=torch.uint8)
    vlc.vlc_first_token(h, rows, shape.eps, torch.ones(shape.H, device=DEV), torch.zeros((shape.vocab, shape.H), device=DEV),
                        logits, token, ws)
    with pytest.raises(vlc.VlcError) as e:                         # workspace too small
        vlc.vlc_first_token(h, torch.zeros((2,), device=DEV, dtype=torch.int32), shape.eps, torch.ones(shape.H, device=DEV),
                            torch.zeros((shape.vocab, shape.H), device=DEV), torch.zeros((2, shape.vocab), device=DEV),
                            torch.zeros((2,), device=DEV, dtype=torch.int32), ws)
    assert e.value.code == 5


def test_first_token_full_vocabulary_7b():
    """The 7B head at full size (152064 x 3584 output matrix, 8 requests as in the long-context batch)."""
    shape = syn.SHAPES["7b"]
    Wh = syn.head_weights(shape, 35)
    h = np.random.default_rng(36).standard_normal((40, shape.H)).astype(np.float32)
    rows = [39, 0, 7, 13, 21, 22, 30, 38]
    print("first-token head 7b: oracle in slabs of 16384 output rows", flush=True)
    check(h, rows, Wh, shape)
