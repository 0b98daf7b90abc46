"""vlc_first_token_noalloc (scratch in a device array built into the library, for callers that cannot
allocate) against vlc_first_token with a caller-owned workspace: same kernels, so the float scores and the
chosen tokens must agree bit for bit.  Two calls in a row share the array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import vlc_synth as syn
import paper_2512_12977_amd as vlc

pytestmark = pytest.mark.gpu
DEV = "cuda"
TD = {"f32": torch.float32, "bf16": torch.bfloat16}


def both_ways(d_h, rows, Wd, shape):
    dt = TD[shape.dtype]
    code = vlc.VLC_BF16 if shape.dtype == "bf16" else vlc.VLC_F32
    d_rows = torch.tensor(rows, device=DEV, dtype=torch.int32)
    m = len(rows)
    out = []
    for noalloc in (False, True):
        logits = torch.full((m, shape.vocab), float("nan"), device=DEV, dtype=torch.float32)
        token = torch.full((m,), -1, device=DEV, dtype=torch.int32)
        if noalloc:
            vlc.vlc_first_token_noalloc(d_h, d_rows, shape.eps, Wd["w_norm_f"], Wd["w_lm"], logits, token)
        else:
            ws = torch.empty(max(256, vlc.vlc_first_token_workspace_bytes(shape.H, m, code)), device=DEV, dtype=torch.uint8)
            vlc.vlc_first_token(d_h, d_rows, shape.eps, Wd["w_norm_f"], Wd["w_lm"], logits, token, ws)
        torch.cuda.synchronize()
        out.append((logits.cpu().numpy(), token.cpu().numpy()))
    (l0, t0), (l1, t1) = out
    assert not np.isnan(l1).any() and (t1 >= 0).all()
    np.testing.assert_array_equal(l1.view(np.uint32), l0.view(np.uint32))
    np.testing.assert_array_equal(t1, t0)


@pytest.mark.parametrize("name", ["tiny", "tiny_bf16"])
def test_noalloc_first_token_equals_the_workspace_entry_point(name):
    shape = syn.SHAPES[name]
    dt = TD[shape.dtype]
    Wh = syn.head_weights(shape, 41)
    Wd = {k: torch.from_numpy(v).to(DEV).to(dt) for k, v in Wh.items()}
    h = np.random.default_rng(42).standard_normal((80, shape.H)).astype(np.float32)
    d_h = torch.from_numpy(h).to(DEV).to(dt)
    print("no-alloc first token:", name, "12 requests, then 3", flush=True)
    both_ways(d_h, [79, 3, 17, 5, 9, 60, 1, 2, 33, 34, 35, 8], Wd, shape)    # more than 8 requests: the GEMM path
    both_ways(d_h, [60, 0, 44], Wd, shape)                                     # smaller, right after, same array


def test_noalloc_first_token_at_the_7b_head_and_its_limit():
    shape = syn.SHAPES["7b"]
    dt = torch.bfloat16
    g = torch.Generator(device=DEV)
    g.manual_seed(43)
    Wd = {"w_norm_f": (1.0 + 0.02 * torch.randn(shape.H, generator=g, device=DEV)).to(dt),
          "w_lm": (0.02 * torch.randn((16384, shape.H), generator=g, device=DEV)).to(dt)}
    import dataclasses
    sh = dataclasses.replace(shape, vocab=16384)
    d_h = torch.randn((200, shape.H), generator=g, device=DEV).to(dt)
    print("no-alloc first token: 7b rows, 8 requests, then 1, then 128 (the limit), then 129 (refused)", flush=True)
    both_ways(d_h, [199, 0, 7, 13, 21, 22, 30, 38], Wd, sh)
    both_ways(d_h, [5], Wd, sh)
    both_ways(d_h, list(range(128)), Wd, sh)
    rows = torch.arange(129, device=DEV, dtype=torch.int32)
    logits = torch.zeros((129, sh.vocab), device=DEV)
    token = torch.zeros((129,), device=DEV, dtype=torch.int32)
    with pytest.raises(vlc.VlcError) as e:
        vlc.vlc_first_token_noalloc(d_h, rows, sh.eps, Wd["w_norm_f"], Wd["w_lm"], logits, token)
    assert e.value.code == 5 and "scratch" in str(e.value)
    assert vlc.vlc_first_token_noalloc_max_bytes() == 1 << 20
