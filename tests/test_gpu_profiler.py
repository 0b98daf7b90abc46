"""The layer-wise sensitivity measurement (Sec. 3.2, Eq. 5) driven through the library against the CPU oracle."""
import dataclasses

import numpy as np
import pytest
import torch

import vlc_synth as syn
from oracle import vlc_oracle as orc
import paper_2512_12977_amd as vlc
from paper_2512_12977_amd import runner as R
from paper_2512_12977_amd import profiler as P

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_mean_squared_error_entry_point():
    g = torch.Generator(device=DEV)
    g.manual_seed(0)
    for n in (1, 255, 256, 1000003):
        a = torch.randn(n, generator=g, device=DEV)
        b = torch.randn(n, generator=g, device=DEV)
        out = torch.zeros(1, device=DEV, dtype=torch.float64)
        ws = torch.empty(vlc.vlc_mean_squared_error_workspace_bytes(), dtype=torch.uint8, device=DEV)
        vlc.vlc_mean_squared_error(a, b, out, ws)
        torch.cuda.synchronize()
        want = float(np.mean((a.cpu().numpy().astype(np.float64) - b.cpu().numpy().astype(np.float64)) ** 2))
        assert abs(out.item() - want) <= 1e-12 * want


@pytest.mark.parametrize("name,L", [("tiny", 3), ("tiny_bias", 2)])
def test_sensitivity_table_fp32_vs_oracle(name, L):
    """fp32 decoder: S[i, j] of the GPU pass against the oracle's.  The table is a mean of squared
    differences of scores that agree to ~1e-5 each, so its entries agree to a few 1e-3 relative
    (difference of nearly equal numbers) plus an absolute floor of the squared score error."""
    shape = dataclasses.replace(syn.SHAPES[name], L=L)
    Wn = [syn.layer_weights(shape, 71, l) for l in range(L)]
    head = syn.head_weights(shape, 71)
    samples = [syn.profile_sample(shape, 72 + s, t_cache_text=17 - 4 * s, t_text=11, t_image=48, t_answer=7) for s in range(2)]
    steps = [0, 60, 150, 500]
    want = orc.sensitivity_profile(shape, Wn, head, samples, steps, orc.store_exact)
    dt = R.torch_dtype(shape.dtype)
    Wd = [R.DeviceWeights(w, dt) for w in Wn]
    got = P.sensitivity_profile(shape, Wd, torch.from_numpy(head["w_norm_f"]).to(DEV).to(dt),
                                torch.from_numpy(head["w_lm"]).to(DEV).to(dt), samples, steps)
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=1e-2, atol=1e-9)
    assert want[:, 0].min() > 1e-7                                   # the mismatch is far above that floor
    # the planner takes the measured table as it is
    k = vlc.vlc_plan_layer_rates(got, 40)
    np.testing.assert_array_equal(k, orc.plan_layer_rates(got, 40))


def test_sensitivity_table_bf16_matching_cache_and_first_layer():
    """bf16: what must hold exactly.  A cache built under the evaluated prompt itself reproduces the
    reference scores bit for bit in every layer at every rate (S = 0); with a mismatched cache the first
    layer's row does not depend on the rate beyond the rounding of the key re-rotation."""
    shape = dataclasses.replace(syn.SHAPES["tiny_bf16"], L=3)
    Wn = [syn.layer_weights(shape, 81, l) for l in range(3)]
    head = syn.head_weights(shape, 81)
    dt = R.torch_dtype(shape.dtype)
    Wd = [R.DeviceWeights(w, dt) for w in Wn]
    wn, wl = torch.from_numpy(head["w_norm_f"]).to(DEV).to(dt), torch.from_numpy(head["w_lm"]).to(DEV).to(dt)
    smp = syn.profile_sample(shape, 82, t_cache_text=12, t_text=12, t_image=64, t_answer=5)
    same = dict(smp, cache_emb=smp["emb"][:12 + 64].copy())
    S = P.sensitivity_profile(shape, Wd, wn, wl, [same], [0, 100, 500])
    np.testing.assert_array_equal(S, 0.0)
    moved = syn.profile_sample(shape, 82, t_cache_text=20, t_text=12, t_image=64, t_answer=5)
    S = P.sensitivity_profile(shape, Wd, wn, wl, [moved], [0, 100, 500])
    assert S[1:, 0].min() > 0
    np.testing.assert_allclose(S[:, 0], S[0, 0], rtol=0, atol=0)     # rate 0: same pass whatever the layer
    assert np.ptp(S[0]) <= 0.05 * S[0, 0]
