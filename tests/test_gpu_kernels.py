"""GPU parity of the individual C-ABI kernels against the CPU oracle (needs an MI355X)."""
import math

import numpy as np
import pytest
import torch

from oracle import vlc_oracle as orc
import paper_2512_12977_amd as vlc
from helpers import assert_close

pytestmark = pytest.mark.gpu
DEV = "cuda"
TD = {"f32": torch.float32, "bf16": torch.bfloat16}


def to_dev(a, dtype):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(TD[dtype])


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def back(t):
    return t.float().cpu().numpy().astype(np.float64)


def stored(a, dtype):
    """What the device holds after upload: the oracle's storage rounding of the float32 data."""
    return orc.STORE[dtype](np.asarray(a, dtype=np.float32).astype(np.float64))


# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("rows,elems,n", [(37, 256, 61), (1600, 3584, 596), (5, 8, 1), (300, 8192, 257)])
def test_gather_rows_bit_exact(dtype, rows, elems, n):
    rng = np.random.default_rng(rows + n)
    src = rng.standard_normal((rows, elems)).astype(np.float32)
    idx = rng.integers(0, rows, size=n)
    d_src = to_dev(src, dtype)
    d_dst = torch.full((n, elems), 7.0, device=DEV, dtype=TD[dtype])
    vlc.vlc_gather_rows(d_src, i32(idx), d_dst)
    torch.cuda.synchronize()
    # the selection itself is exact: compare bit patterns with plain indexing of the uploaded rows
    assert torch.equal(d_dst, d_src[torch.from_numpy(idx).to(DEV)])
    np.testing.assert_array_equal(back(d_dst), stored(src, dtype)[idx])


def test_gather_rows_empty_and_errors():
    src = torch.zeros((4, 8), device=DEV)
    dst = torch.zeros((0, 8), device=DEV)
    vlc.vlc_gather_rows(src, i32([]), dst)          # n = 0: no-op
    with pytest.raises(vlc.VlcError) as e:          # 12-byte rows are not a multiple of 16
        vlc.vlc_gather_rows(torch.zeros((4, 3), device=DEV), i32([0]), torch.zeros((1, 3), device=DEV))
    assert e.value.code == 2


# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("Hkv,D,base", [(2, 64, 1e4), (4, 128, 1e6), (8, 128, 1e6)])
def test_rope_shift_kv_vs_oracle(dtype, Hkv, D, base):
    rng = np.random.default_rng(Hkv * D)
    pool, S, n = 300, 517, 211
    ks = rng.standard_normal((pool, Hkv, D)).astype(np.float32)
    vs = rng.standard_normal((pool, Hkv, D)).astype(np.float32)
    src = rng.permutation(pool)[:n]
    dst = rng.permutation(S)[:n]
    delta = rng.integers(-20000, 20000, size=n)
    delta[:3] = [0, 1, -1]
    d_k = torch.zeros((S, Hkv, D), device=DEV, dtype=TD[dtype])
    d_v = torch.zeros((S, Hkv, D), device=DEV, dtype=TD[dtype])
    vlc.vlc_rope_shift_kv(to_dev(ks, dtype), to_dev(vs, dtype), d_k, d_v, i32(src), i32(dst), i32(delta), base)
    torch.cuda.synchronize()
    want_k = np.zeros((S, Hkv, D))
    want_v = np.zeros((S, Hkv, D))
    want_k[dst] = orc.STORE[dtype](orc.rope_rotate(stored(ks, dtype)[src], delta, base))
    want_v[dst] = stored(vs, dtype)[src]
    assert_close(back(d_k), want_k, dtype, "shifted K")
    np.testing.assert_array_equal(back(d_v), want_v)            # values are copied, bit-exact
    # delta 0 leaves keys bit-identical
    np.testing.assert_array_equal(back(d_k)[dst[0]], stored(ks, dtype)[src[0]])


@pytest.mark.parametrize("seed", range(16))
def test_streaming_entry_points_random_sizes(seed):
    """RoPE shift, gather and scatter on seeded random sizes: 1-8 kv heads, head dimension 64 or 128, 1-6000 tokens or
    rows, row widths that are any multiple of 8 elements, deltas up to +-2^20 positions, both storage types."""
    rng = np.random.default_rng(15000 + seed)
    dtype = "bf16" if seed % 2 else "f32"
    Hkv, D = int(rng.integers(1, 9)), int(rng.choice([64, 128]))
    base = float(rng.choice([1e4, 1e6, 5e6]))
    n = int(rng.integers(1, 6000))
    pool, S = n + int(rng.integers(0, 500)), n + int(rng.integers(0, 500))
    ks = rng.standard_normal((pool, Hkv, D)).astype(np.float32)
    vs = rng.standard_normal((pool, Hkv, D)).astype(np.float32)
    src, dst = rng.permutation(pool)[:n], rng.permutation(S)[:n]
    delta = rng.integers(-(1 << 20), 1 << 20, size=n)
    d_k = torch.zeros((S, Hkv, D), device=DEV, dtype=TD[dtype])
    d_v = torch.zeros((S, Hkv, D), device=DEV, dtype=TD[dtype])
    vlc.vlc_rope_shift_kv(to_dev(ks, dtype), to_dev(vs, dtype), d_k, d_v, i32(src), i32(dst), i32(delta), base)
    torch.cuda.synchronize()
    want_k, want_v = np.zeros((S, Hkv, D)), np.zeros((S, Hkv, D))
    want_k[dst] = orc.STORE[dtype](orc.rope_rotate(stored(ks, dtype)[src], delta, base))
    want_v[dst] = stored(vs, dtype)[src]
    assert_close(back(d_k), want_k, dtype, "shifted K (seed %d: %d tokens, %d heads of %d)" % (seed, n, Hkv, D))
    np.testing.assert_array_equal(back(d_v), want_v)
    # scatter of fresh rows into the same caches, gather of rows of a matrix of odd width: bit-exact
    m = int(rng.integers(1, n + 1))
    kn = rng.standard_normal((m, Hkv, D)).astype(np.float32)
    vn = rng.standard_normal((m, Hkv, D)).astype(np.float32)
    rows = rng.permutation(S)[:m]
    vlc.vlc_scatter_kv(to_dev(kn, dtype), to_dev(vn, dtype), i32(rows), d_k, d_v)
    elems = 8 * int(rng.integers(1, 700))
    x = rng.standard_normal((pool, elems)).astype(np.float32)
    idx = rng.integers(0, pool, size=m)
    out = torch.empty((m, elems), device=DEV, dtype=TD[dtype])
    vlc.vlc_gather_rows(to_dev(x, dtype), i32(idx), out)
    torch.cuda.synchronize()
    want_k2, want_v2 = back(d_k).copy(), back(d_v).copy()
    np.testing.assert_array_equal(back(d_k)[rows], stored(kn, dtype))
    np.testing.assert_array_equal(back(d_v)[rows], stored(vn, dtype))
    keep = np.setdiff1d(np.arange(S), rows)
    np.testing.assert_array_equal(back(d_v)[keep], want_v[keep])          # rows not scattered to are untouched
    np.testing.assert_array_equal(back(out), stored(x, dtype)[idx])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rope_shift_in_place_and_inverse(dtype):
    """In-place use, and shift(d) followed by shift(-d) returns the keys (to storage rounding)."""
    rng = np.random.default_rng(5)
    S, Hkv, D, base = 130, 4, 128, 1e6
    k0 = rng.standard_normal((S, Hkv, D)).astype(np.float32)
    d_k = to_dev(k0, dtype)
    rows = np.arange(S)
    delta = rng.integers(-4000, 4000, size=S)
    vlc.vlc_rope_shift_kv(d_k, None, d_k, None, i32(rows), i32(rows), i32(delta), base)
    torch.cuda.synchronize()
    assert_close(back(d_k), orc.STORE[dtype](orc.rope_rotate(stored(k0, dtype), delta, base)), dtype, "in place")
    vlc.vlc_rope_shift_kv(d_k, None, d_k, None, i32(rows), i32(rows), i32(-delta), base)
    torch.cuda.synchronize()
    assert_close(back(d_k), stored(k0, dtype), dtype, "round trip")
    if dtype == "f32":
        assert np.max(np.abs(back(d_k) - k0)) < 5e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("Hkv,D,base,counts", [(2, 64, 1e4, (211, 0, 37, 1)), (4, 128, 1e6, (20, 517, 300, 64, 3)),
                                               (8, 128, 1e6, (4000, 2500))])
def test_rope_shift_kv_layers_vs_oracle(dtype, Hkv, D, base, counts):
    """Several layers' reused keys in one launch (job table), token counts differing per job (one
    table entry has n_tok = 0): against the oracle, and bit for
    bit against the per-layer entry point."""
    rng = np.random.default_rng(Hkv * D + len(counts))
    pool, S = max(counts) + 90, max(counts) + 301
    jobs, keep, want, single = [], [], [], []
    for n in counts:
        ks = rng.standard_normal((pool, Hkv, D)).astype(np.float32)
        vs = rng.standard_normal((pool, Hkv, D)).astype(np.float32)
        src, dst = rng.permutation(pool)[:n], rng.permutation(S)[:n]
        delta = rng.integers(-20000, 20000, size=n)
        d_ks, d_vs = to_dev(ks, dtype), to_dev(vs, dtype)
        d_k = torch.zeros((S, Hkv, D), device=DEV, dtype=TD[dtype])
        d_v = torch.zeros((S, Hkv, D), device=DEV, dtype=TD[dtype])
        idx = (i32(src), i32(dst), i32(delta))
        jobs.append((d_ks, d_vs, d_k, d_v) + idx)
        want_k, want_v = np.zeros((S, Hkv, D)), np.zeros((S, Hkv, D))
        want_k[dst] = orc.STORE[dtype](orc.rope_rotate(stored(ks, dtype)[src], delta, base))
        want_v[dst] = stored(vs, dtype)[src]
        want.append((want_k, want_v))
        s_k, s_v = torch.zeros_like(d_k), torch.zeros_like(d_v)
        if n:
            vlc.vlc_rope_shift_kv(d_ks, d_vs, s_k, s_v, *idx, base)
        single.append((s_k, s_v))
    table = torch.from_numpy(vlc.shift_job_table(jobs)).to(DEV)
    assert table.numel() == 64 * len(counts)
    vlc.vlc_rope_shift_kv_layers(table, len(jobs), max(counts), Hkv, D, base, vlc.VLC_BF16 if dtype == "bf16" else vlc.VLC_F32)
    torch.cuda.synchronize()
    for j, (wk, wv) in zip(jobs, want):
        assert_close(back(j[2]), wk, dtype, "shifted K")
        np.testing.assert_array_equal(back(j[3]), wv)
    for j, (s_k, s_v) in zip(jobs, single):
        assert torch.equal(j[2], s_k) and torch.equal(j[3], s_v)


def test_rope_shift_kv_layers_bound_and_keys_only():
    """max_n_tok below a job's n_tok: only the first max_n_tok tokens move; v pointers NULL: keys only."""
    rng = np.random.default_rng(77)
    Hkv, D, base, n = 4, 128, 1e6, 100
    ks = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    d_k = torch.zeros((n, Hkv, D), device=DEV, dtype=torch.float32)
    rows, delta = np.arange(n), rng.integers(-500, 500, size=n)
    job = (to_dev(ks, "f32"), None, d_k, None, i32(rows), i32(rows), i32(delta))
    table = torch.from_numpy(vlc.shift_job_table([job])).to(DEV)
    vlc.vlc_rope_shift_kv_layers(table, 1, 40, Hkv, D, base, vlc.VLC_F32)
    torch.cuda.synchronize()
    got = back(d_k)
    assert_close(got[:40], orc.rope_rotate(ks[:40].astype(np.float64), delta[:40], base), "f32", "first 40")
    assert not got[40:].any()
    vlc.vlc_rope_shift_kv_layers(table, 0, 40, Hkv, D, base, vlc.VLC_F32)      # no jobs: nothing launched
    vlc.vlc_rope_shift_kv_layers(table, 1, 0, Hkv, D, base, vlc.VLC_F32)       # no tokens: nothing launched
    with pytest.raises(vlc.VlcError):
        vlc.vlc_rope_shift_kv_layers(table, 1, 40, Hkv, 96, base, vlc.VLC_F32)


# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scatter_kv_bit_exact(dtype):
    rng = np.random.default_rng(9)
    S, n, Hkv, D = 1600, 596, 4, 128
    kn = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    vn = rng.standard_normal((n, Hkv, D)).astype(np.float32)
    kc = rng.standard_normal((S, Hkv, D)).astype(np.float32)
    vc = rng.standard_normal((S, Hkv, D)).astype(np.float32)
    dst = np.sort(rng.permutation(S)[:n])
    d_kc, d_vc = to_dev(kc, dtype), to_dev(vc, dtype)
    vlc.vlc_scatter_kv(to_dev(kn, dtype), to_dev(vn, dtype), i32(dst), d_kc, d_vc)
    torch.cuda.synchronize()
    want_k, want_v = stored(kc, dtype), stored(vc, dtype)
    want_k[dst] = stored(kn, dtype)
    want_v[dst] = stored(vn, dtype)
    np.testing.assert_array_equal(back(d_kc), want_k)
    np.testing.assert_array_equal(back(d_vc), want_v)


# ------------------------------------------------------------------------------------------
def attention_case(dtype, Hq, Hkv, D, requests, seed, lens_sorted=True):
    """requests: list of (S, [query slots]).  Packed KV, per-row start/len, oracle per request."""
    rng = np.random.default_rng(seed)
    total = sum(S for S, _ in requests)
    K = rng.standard_normal((total, Hkv, D)).astype(np.float32)
    V = rng.standard_normal((total, Hkv, D)).astype(np.float32)
    starts, lens, base = [], [], 0
    for S, slots in requests:
        for s in slots:
            starts.append(base)
            lens.append(s + 1 if s >= 0 else 0)
        base += S
    n = len(starts)
    q = rng.standard_normal((n, Hq, D)).astype(np.float32)
    d_out = torch.full((n, Hq, D), 3.0, device=DEV, dtype=TD[dtype])
    scale = 1.0 / math.sqrt(D)
    vlc.vlc_sparse_q_attention(to_dev(q, dtype), to_dev(K, dtype), to_dev(V, dtype), i32(starts), i32(lens),
                               scale, d_out)
    torch.cuda.synchronize()
    want = np.zeros((n, Hq, D))
    row, base = 0, 0
    for S, slots in requests:
        m = len(slots)
        want[row:row + m] = orc.attention_rows(stored(q[row:row + m], dtype), stored(K[base:base + S], dtype),
                                               stored(V[base:base + S], dtype),
                                               np.asarray(lens[row:row + m]), scale)
        row += m
        base += S
    want = orc.STORE[dtype](want)
    return assert_close(back(d_out), want, dtype, "attention")


@pytest.mark.parametrize("dtype,Hq,Hkv,D", [("f32", 4, 2, 64), ("f32", 4, 4, 128), ("bf16", 28, 4, 128),
                                           ("bf16", 64, 8, 128), ("bf16", 4, 2, 128), ("bf16", 3, 3, 128)])
def test_attention_single_request_ragged(dtype, Hq, Hkv, D):
    S = 333
    slots = list(range(0, 40)) + [41, 44, 100, 101, 102, 199, 200] + list(range(310, 333))
    attention_case(dtype, Hq, Hkv, D, [(S, slots)], seed=Hq * 7 + D)


@pytest.mark.parametrize("dtype,Hq,Hkv,D", [("f32", 4, 2, 64), ("bf16", 28, 4, 128), ("bf16", 16, 2, 128)])
def test_attention_packed_requests_share_tiles(dtype, Hq, Hkv, D):
    """Three requests whose few rows land in the same row tile; includes a zero-length row and
    a single-key row."""
    reqs = [(70, [0, 5, 69]), (130, [-1, 0, 64, 65, 129]), (64, [63]), (200, list(range(150, 200)))]
    attention_case(dtype, Hq, Hkv, D, reqs, seed=11)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_unsorted_lengths_and_one_row(dtype):
    D = 64 if dtype == "f32" else 128
    attention_case(dtype, 4, 2, D, [(257, [256, 3, 128, 0, 77])], seed=3)
    attention_case(dtype, 4, 2, D, [(65, [64])], seed=4)


def test_attention_long_context_bf16():
    """7B head layout, S = 4500: rows at the start of each 'image' and a trailing text run."""
    S = 4500
    slots = list(range(0, 30)) + [s for b in range(30, 4000, 1024) for s in range(b, b + 20)] + \
        list(range(S - 120, S))
    attention_case("bf16", 28, 4, 128, [(S, slots)], seed=21)


@pytest.mark.parametrize("Hq,Hkv,reqs", [
    # one query head per kv head, 256 rows per tile: runs of three requests share tiles, a zero-length row,
    # single-key rows, rows out of order
    (64, 64, [(700, [-1, 0, 0] + list(range(0, 700, 1)) + [5, 699, 3]), (300, list(range(300))), (1000, list(range(1000)))]),
    # two query heads per kv head, 128 rows per tile, ragged tail
    (32, 16, [(2500, list(range(2500))), (1723, list(range(0, 1723)))]),
    # seven query heads per kv head (7B layout): 36 rows and 252 of 256 lanes per tile of the many-row kernel,
    # rows of one request out of order, a zero-length row and single-key rows among them
    (28, 4, [(1500, list(range(1500))), (1800, [-1, 0, 0, 1799, 2] + list(range(1800))), (1400, list(range(1399, -1, -1)))]),
])
def test_attention_many_rows(Hq, Hkv, reqs):
    """Thousands of rows, several requests, more than 512 workgroups."""
    attention_case("bf16", Hq, Hkv, 128, reqs, seed=31)


@pytest.mark.parametrize("seed", range(24))
def test_attention_random_heads_requests_and_rows(seed):
    """Seeded random head layouts (1-8 kv heads, 1-16 query heads per kv head), 1-5 packed requests of 1-3000 slots,
    rows that are runs, scattered slots, duplicates and zero-length rows in any order; fp32 (D 64 or 128) and bf16."""
    rng = np.random.default_rng(13000 + seed)
    dtype = "bf16" if seed % 3 else "f32"
    D = 128 if dtype == "bf16" else int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    g = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16]))
    reqs = []
    for _ in range(int(rng.integers(1, 6))):
        S = int(rng.integers(1, 3000 if dtype == "bf16" else 700))
        kind = int(rng.integers(0, 4))
        if kind == 0:      # a trailing run (the text behind the images)
            slots = list(range(max(0, S - int(rng.integers(1, 200))), S))
        elif kind == 1:    # scattered slots, unsorted, with duplicates
            slots = [int(x) for x in rng.integers(0, S, size=int(rng.integers(1, 150)))]
        elif kind == 2:    # leading runs of several "images" and a zero-length row
            slots = [-1] + [s for b in range(0, S, max(1, S // 5)) for s in range(b, min(S, b + int(rng.integers(1, 40))))]
        else:              # every slot
            slots = list(range(S)) if S <= 1200 else list(range(0, S, 3))
        reqs.append((S, slots))
    attention_case(dtype, Hkv * g, Hkv, D, reqs, seed=seed)


def test_attention_errors():
    q = torch.zeros((2, 4, 128), device=DEV, dtype=torch.bfloat16)
    kv = torch.zeros((8, 3, 128), device=DEV, dtype=torch.bfloat16)
    with pytest.raises(vlc.VlcError) as e:      # 4 query heads over 3 kv heads
        vlc.vlc_sparse_q_attention(q, kv, kv, i32([0, 0]), i32([1, 2]), 1.0, torch.zeros_like(q))
    assert e.value.code == 2
