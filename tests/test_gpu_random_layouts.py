"""GPU parity on seeded random decoder shapes and prompt layouts (needs an MI355X).

The named workloads fix their head counts, widths and layouts; here they are drawn: 1-3 packed requests whose
parts are text runs and images in any order (an image first, images side by side, a request that ends on an image),
position ids that start anywhere, cached positions before or behind the new ones, head groups of 1-8 query heads
per kv head, widths that are not powers of two, three layers whose rates fall with depth down to zero; a third of the
cases use the Qwen3-VL-shaped layer with random frequency sections and images as grids of 1-17 rows and columns.  Every
layer's h, K and V are compared with the oracle element by element at the stated tolerance (fp32: free running;
bf16: each layer fed the oracle's previous output, as the tolerance is a per-layer statement).
"""
import os

import numpy as np
import pytest

import vlc_synth as syn
from helpers import assert_close
from test_gpu_layer import oracle_stack, run_gpu_stack

pytestmark = pytest.mark.gpu


def random_workload(seed):
    rng = np.random.default_rng(7000 + seed)
    bf16 = seed % 2 == 1
    D = 128 if bf16 else int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3]))
    g = int(rng.choice([1, 2, 3, 4, 7, 8]))
    grid = seed % 36 >= 24  # the Qwen3-VL-shaped layer: q/k norm, three position ids per token, images as grids
    extra = {}
    if grid:
        h_sec = int(rng.integers(0, D // 4 + 1))
        w_sec = int(rng.integers(0, D // 4 + 1))
        extra = dict(qk_norm=True, mrope_section=(D // 2 - h_sec - w_sec, h_sec, w_sec))
    shape = syn.Shape("random%d" % seed, L=3, H=64 * int(rng.integers(2, 6)), Hq=Hkv * g, Hkv=Hkv, D=D,
                      I=64 * int(rng.integers(2, 9)), rope_base=float(rng.choice([1e4, 1e6])),
                      dtype="bf16" if bf16 else "f32", qkv_bias=bool(rng.integers(2)) and not grid, **extra)
    requests, at, cache_row = [], 0, 0
    for b in range(int(rng.integers(1, 4))):
        parts, texts = [], 0
        for p in range(int(rng.integers(1, 7))):
            if rng.random() < 0.5:
                n = int(rng.integers(1, 50))
                parts.append(("text", n))
                texts += n
            elif grid:
                rows, cols = int(rng.integers(1, 18)), int(rng.integers(1, 18))
                parts.append(("image", rows, cols, int(rng.integers(0, 5000)), cache_row))
                cache_row += rows * cols
            else:
                T = int(rng.integers(3, 300))
                parts.append(("image", T, int(rng.integers(0, 5000)), cache_row))
                cache_row += T
        if texts == 0:
            parts.append(("text", int(rng.integers(1, 9))))
        if grid:
            req = syn.workloads._grid_request(parts, at)
        else:
            req = syn.Request(syn.workloads._layout(parts), at, pos_start=int(rng.integers(0, 3000)))
        requests.append(req)
        at += req.S
    k = np.sort(rng.integers(0, 501, size=3))[::-1].astype(np.int32)
    if seed % 4 == 3:
        k[2] = 0            # the deepest layer recomputes text only
    if seed % 6 == 0:
        k[0] = 500          # the first layer recomputes everything
    wl = syn.Workload("random%d" % seed, shape, requests, max(cache_row, 1), "static", static_k=int(k[0]), seed=100 + seed)
    return wl, k


N_SEEDS = int(os.environ.get("VLC_RANDOM_LAYOUTS", "36"))   # more seeds for a longer soak of the same check


@pytest.mark.parametrize("seed", range(N_SEEDS))
def test_random_shape_and_layout_against_oracle(seed):
    wl, k = random_workload(seed)
    sh, L = wl.shape, 3
    weights = [syn.layer_weights(sh, wl.seed, l) for l in range(L)]
    emb = syn.embedding_rows(wl)
    caches = [syn.cached_kv(wl, l) for l in range(L)]
    ref = oracle_stack(wl, weights, emb, caches, k, None, L)
    cat = lambda l, key: np.concatenate([ref[r][l][key] for r in range(len(wl.requests))])
    teacher = [cat(l, "h") for l in range(L)] if sh.dtype == "bf16" else None
    got, plans = run_gpu_stack(wl, weights, emb, caches, k, None, L, teacher, shift_ahead=seed % 3 == 0,
                               chain=sh.dtype != "bf16" and seed % 4 == 2)
    what = "seed %d (%s, H %d, %d/%d heads of %d, I %d, %d requests, %d slots, k %s)" % (
        seed, sh.dtype, sh.H, sh.Hq, sh.Hkv, sh.D, sh.I, len(wl.requests), wl.total_slots, k.tolist())
    for l in range(L):
        assert got[l][0].shape == cat(l, "h").shape, what
        assert_close(got[l][1], cat(l, "K"), sh.dtype, "%s layer %d K" % (what, l))
        assert_close(got[l][2], cat(l, "V"), sh.dtype, "%s layer %d V" % (what, l))
        assert_close(got[l][0], cat(l, "h"), sh.dtype, "%s layer %d h" % (what, l))


@pytest.mark.parametrize("seed", range(16))
def test_random_row_counts_at_mid_sized_shapes_stage_by_stage(seed):
    """One bf16 layer at shapes between the tiny and the 7B ones (H 1024-2048, MLP width 2048-6144), with 1-2600
    recomputed rows: the GEMM dispatcher's choices (tile, k ranges, split of the last round) and the attention's
    key-range split change with every case.  Every stage is compared with the oracle on the GPU's own inputs."""
    from test_gpu_layer import check_layer_stage_by_stage
    rng = np.random.default_rng(9000 + seed)
    Hkv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 4, 7]))
    shape = syn.Shape("mid%d" % seed, L=1, H=256 * int(rng.integers(4, 9)), Hq=Hkv * g, Hkv=Hkv, D=128,
                      I=256 * int(rng.integers(8, 25)), rope_base=1e6, dtype="bf16", qkv_bias=bool(rng.integers(2)))
    n_text = int(rng.integers(1, 1200))
    T = int(rng.integers(16, 3000))
    k = int(rng.integers(0, 501))
    segs = syn.workloads._layout([("text", n_text // 2 + 1), ("image", T, int(rng.integers(0, 4000)), 0), ("text", n_text - n_text // 2)])
    wl = syn.Workload("mid%d" % seed, shape, [syn.Request(segs, 0, pos_start=int(rng.integers(0, 2000)))], T, "static",
                      static_k=k, seed=200 + seed)
    dev, floor = check_layer_stage_by_stage(wl)
    assert dev <= floor
