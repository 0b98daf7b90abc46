"""Workload descriptions and seeded random tensors (no method arithmetic).

The paper times prompts of the form <text><image_1>...<image_n> with a short
text part and 1K-20K image tokens on Qwen-VL decoders (Sec. 5.1); its images,
prompts and checkpoints are not available here, so the workloads below keep
the *shapes* (decoder dimensions, image-token counts, text/image interleaving,
position shifts of the reused images) and fill every tensor from
numpy.random.default_rng with per-tensor child seeds.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Optional, Sequence

import numpy as np


@dataclasses.dataclass(frozen=True)
class Shape:
    """Decoder-layer dimensions."""
    name: str
    L: int            # layers
    H: int            # hidden size
    Hq: int           # query heads
    Hkv: int          # key/value heads
    D: int            # head dim
    I: int            # MLP width
    rope_base: float
    dtype: str        # "f32" | "bf16"  (storage type of the GPU path)
    qkv_bias: bool
    eps: float = 1e-6
    vocab: int = 512  # rows of the output (LM head) matrix
    qk_norm: bool = False                 # per-head RMSNorm of q and k before RoPE (Qwen3 family)
    mrope_section: tuple = ()             # (t, h, w) frequency counts of 3-axis RoPE; () = 1-D RoPE
    n_experts: int = 0                    # > 0: mixture-of-experts MLP; I is then the width of ONE expert
    top_k: int = 0                        # experts per token
    # Scale of the synthetic inputs.  With experts the rows must stay as different from one another as a
    # trained model's are, or the router sends every row to the same few experts (a trained router is
    # balanced): text rows are then drawn at the scale of the image rows (1.0 instead of 0.02) and the
    # two projections that write into the residual stream (w_o, w_down) at 0.02 / sqrt(2 L) instead
    # of 0.02, so that the residual stream is not taken over by the mean of the values that uniform
    # attention over random keys adds to every row.
    text_scale: float = 0.02
    residual_proj_scale: float = 0.02

    @property
    def g(self) -> int:
        return self.Hq // self.Hkv

    @property
    def n_qkv(self) -> int:
        return (self.Hq + 2 * self.Hkv) * self.D


SHAPES: Dict[str, Shape] = {
    "tiny": Shape("tiny", L=2, H=256, Hq=4, Hkv=2, D=64, I=512, rope_base=1e4,
                  dtype="f32", qkv_bias=False),
    "tiny_bias": Shape("tiny_bias", L=2, H=256, Hq=4, Hkv=2, D=64, I=512, rope_base=1e4,
                       dtype="f32", qkv_bias=True),
    "tiny_bf16": Shape("tiny_bf16", L=2, H=256, Hq=4, Hkv=2, D=128, I=512, rope_base=1e4,
                       dtype="bf16", qkv_bias=True),
    # Qwen3-VL-shaped variants: q/k norm, interleaved 3-axis RoPE, no q|k|v bias
    "tiny_q3": Shape("tiny_q3", L=2, H=256, Hq=4, Hkv=2, D=64, I=512, rope_base=1e4,
                     dtype="f32", qkv_bias=False, qk_norm=True, mrope_section=(12, 10, 10)),
    "tiny_q3_bf16": Shape("tiny_q3_bf16", L=2, H=256, Hq=4, Hkv=2, D=128, I=512, rope_base=1e4,
                          dtype="bf16", qkv_bias=False, qk_norm=True, mrope_section=(24, 20, 20)),
    "q3vl_8b": Shape("q3vl_8b", L=36, H=4096, Hq=32, Hkv=8, D=128, I=12288, rope_base=5e6,
                     dtype="bf16", qkv_bias=False, vocab=151936, qk_norm=True, mrope_section=(24, 20, 20)),
    # mixture-of-experts MLP on top of the Qwen3-VL-shaped attention
    "tiny_moe": Shape("tiny_moe", L=2, H=256, Hq=4, Hkv=2, D=64, I=128, rope_base=1e4, dtype="f32", qkv_bias=False,
                      qk_norm=True, mrope_section=(12, 10, 10), n_experts=8, top_k=2, text_scale=1.0,
                      residual_proj_scale=0.01),
    "tiny_moe_bf16": Shape("tiny_moe_bf16", L=2, H=256, Hq=4, Hkv=2, D=128, I=128, rope_base=1e4, dtype="bf16",
                           qkv_bias=False, qk_norm=True, mrope_section=(24, 20, 20), n_experts=8, top_k=2,
                           text_scale=1.0, residual_proj_scale=0.01),
    "q3vl_30b_a3b": Shape("q3vl_30b_a3b", L=48, H=2048, Hq=32, Hkv=4, D=128, I=768, rope_base=5e6, dtype="bf16",
                          qkv_bias=False, vocab=151936, qk_norm=True, mrope_section=(24, 20, 20), n_experts=128,
                          top_k=8, text_scale=1.0, residual_proj_scale=0.02 / 96 ** 0.5),
    "7b": Shape("7b", L=28, H=3584, Hq=28, Hkv=4, D=128, I=18944, rope_base=1e6,
                dtype="bf16", qkv_bias=True, vocab=152064),
    "72b": Shape("72b", L=80, H=8192, Hq=64, Hkv=8, D=128, I=29568, rope_base=1e6,
                 dtype="bf16", qkv_bias=True, vocab=152064),
}


@dataclasses.dataclass(frozen=True)
class Segment:
    """A run of consecutive slots of one request.

    start     first slot, relative to the request's first slot
    length    number of tokens
    is_image  True: vision tokens whose K/V exist in the cache pool
    old_pos   position id the cached keys of the first token were rotated at
    cache_row row of the first token inside the cache pool
    """
    start: int
    length: int
    is_image: bool
    old_pos: int = 0
    cache_row: int = 0


@dataclasses.dataclass(frozen=True)
class Request:
    segments: Sequence[Segment]
    kv_start: int     # first slot of this request in the packed KV of the batch
    pos_start: int = 0  # position id of the request's first slot (slot s has pos_start + s)
    # 3-axis position ids [S, 3] (temporal, height, width) when the decoder uses 3-axis RoPE, else
    # None.  Text slots carry the same id on all axes; an image's tokens share the temporal id and
    # count rows / columns of its grid on the other two.  A reused image whose first position moved
    # from Segment.old_pos to pos3[start, 0] has every axis of every token shifted by that difference.
    pos3: Optional[np.ndarray] = None

    @property
    def S(self) -> int:
        return sum(s.length for s in self.segments)


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    shape: Shape
    requests: Sequence[Request]
    cache_rows: int                  # rows of the cached-image K/V pool (per layer)
    plan: str                        # "static" | "dynamic" | "explicit"
    static_k: Optional[int] = None   # grid steps (rate = k/500) when plan == "static"
    budget_bp: Optional[int] = None  # mean rate in basis points when plan == "dynamic"
    explicit_counts: Optional[int] = None  # leading tokens per image when plan == "explicit"
    seed: int = 0

    @property
    def total_slots(self) -> int:
        return sum(r.S for r in self.requests)


def _layout(parts: Sequence[tuple]) -> List[Segment]:
    """parts: ("text", n) or ("image", n, old_pos, cache_row)."""
    segs, at = [], 0
    for p in parts:
        if p[0] == "text":
            segs.append(Segment(at, p[1], False))
        else:
            segs.append(Segment(at, p[1], True, p[2], p[3]))
        at += p[1]
    return segs


def _grid_request(parts: Sequence[tuple], kv_start: int = 0) -> "Request":
    """A request with 3-axis position ids.  parts: ("text", n) or ("image", rows, cols, old_pos, cache_row),
    old_pos being the temporal id the image was cached at."""
    flat = [p if p[0] == "text" else ("image", p[1] * p[2], p[3], p[4]) for p in parts]
    grid = [p if p[0] == "text" else ("image", p[1], p[2]) for p in parts]
    return Request(_layout(flat), kv_start, 0, grid_positions(grid))


def make_workload(name: str) -> Workload:
    """The benchmark/parity workloads, by short name.

    c1  tiny fp32 decoder, one 256-token image after 32 text tokens (+32 shift), 16 new text tokens,
        13 leading image tokens recomputed in both layers
    c2  7B shape, 512 text | 1024-token image (shift +512) | 64 text, uniform 2 %
    c3  7B shape, four 1296-token images between 128-token text runs, images placed in a shuffled
        order relative to the layout they were cached under, dynamic 5 % budget
    c4  7B shape, batch of 8: text a_b | 16 x 1024-token images | text 2048-a_b, uniform 2 %
    c4_5  as c4 with uniform 5 %
    c5  72B shape, 8 x 1296-token images | 256 text, dynamic 3 % budget
    c1_q3, c1_q3_bf16, c2_q3, c3_q3  the same prompts for the Qwen3-VL-shaped layer (q/k norm, 3-axis position ids)
    c1_moe, c1_moe_bf16, c2_moe, c4_moe  the same with a mixture-of-experts MLP (c2_moe, c4_moe: 30B-A3B shape)
    """
    if name == "c1":
        segs = _layout([("text", 32), ("image", 256, 0, 0), ("text", 16)])
        return Workload("c1", SHAPES["tiny"], [Request(segs, 0)], 256, "explicit",
                        explicit_counts=13, seed=0)
    if name == "c1_bias":
        segs = _layout([("text", 32), ("image", 256, 0, 0), ("text", 16)])
        return Workload("c1_bias", SHAPES["tiny_bias"], [Request(segs, 0)], 256, "explicit",
                        explicit_counts=13, seed=0)
    if name == "c1_bf16":
        segs = _layout([("text", 32), ("image", 256, 0, 0), ("text", 16)])
        return Workload("c1_bf16", SHAPES["tiny_bf16"], [Request(segs, 0)], 256, "explicit",
                        explicit_counts=13, seed=0)
    if name in ("c1_q3", "c1_q3_bf16"):
        # as c1 with the Qwen3-VL-shaped layer: the image is a 16 x 16 grid cached at temporal id 0
        req = _grid_request([("text", 32), ("image", 16, 16, 0, 0), ("text", 16)])
        return Workload(name, SHAPES["tiny_q3" if name == "c1_q3" else "tiny_q3_bf16"], [req], 256, "explicit",
                        explicit_counts=13, seed=6)
    if name in ("c1_moe", "c1_moe_bf16"):
        # as c1_q3 with a mixture-of-experts MLP (8 experts, 2 per token)
        req = _grid_request([("text", 32), ("image", 16, 16, 0, 0), ("text", 16)])
        return Workload(name, SHAPES["tiny_moe" if name == "c1_moe" else "tiny_moe_bf16"], [req], 256, "explicit",
                        explicit_counts=13, seed=9)
    if name == "c2_moe":
        # as c2_q3 at the Qwen3-VL-30B-A3B text-decoder shape (128 experts, 8 per token)
        req = _grid_request([("text", 512), ("image", 32, 32, 0, 0), ("text", 64)])
        return Workload("c2_moe", SHAPES["q3vl_30b_a3b"], [req], 1024, "static", static_k=10, seed=10)
    if name == "c4_moe":
        # a batch of 8 long prompts at the 30B-A3B shape: text a_b | 16 images of 32 x 32 tokens | text 2048 - a_b
        NI, X, B = 16, 2048, 8
        a = np.random.default_rng(11).choice(np.arange(1, 1025), size=B, replace=False)
        reqs, at = [], 0
        for b in range(B):
            parts = [("text", int(a[b]))] + [("image", 32, 32, j * 32, j * 1024) for j in range(NI)] + [("text", X - int(a[b]))]
            reqs.append(_grid_request(parts, at))
            at += X + NI * 1024
        return Workload("c4_moe", SHAPES["q3vl_30b_a3b"], reqs, NI * 1024, "static", static_k=10, seed=11)
    if name == "c2_q3":
        # as c2 at the Qwen3-VL 8B text-decoder shape: a 32 x 32-token image cached at temporal id 0
        req = _grid_request([("text", 512), ("image", 32, 32, 0, 0), ("text", 64)])
        return Workload("c2_q3", SHAPES["q3vl_8b"], [req], 1024, "static", static_k=10, seed=7)
    if name == "c3_q3":
        # as c3 at the Qwen3-VL 8B shape: four 36 x 36 images, reused in a shuffled order.  Cached
        # under text|img0|text|img1|... where an image advances the ids by max(rows, cols) = 36.
        G, X = 36, 128
        old_pos = [X + i * (G + X) for i in range(4)]
        parts = [("text", X)]
        for i, j in enumerate((2, 0, 3, 1)):
            parts += [("image", G, G, old_pos[j], j * G * G), ("text", X)]
        return Workload("c3_q3", SHAPES["q3vl_8b"], [_grid_request(parts)], 4 * G * G, "dynamic", budget_bp=500, seed=8)
    if name == "c2":
        segs = _layout([("text", 512), ("image", 1024, 0, 0), ("text", 64)])
        return Workload("c2", SHAPES["7b"], [Request(segs, 0)], 1024, "static", static_k=10, seed=2)
    if name == "c3":
        # cached under the layout text|img0|text|img1|text|img2|text|img3|text ; reused with the
        # four images in a permuted order, so the position deltas have both signs.
        T, X = 1296, 128
        old_pos = [X + i * (T + X) for i in range(4)]
        rng = np.random.default_rng(1)
        perm = rng.permutation(4)
        while np.any(perm == np.arange(4)):      # every image must move (non-zero delta)
            perm = rng.permutation(4)
        parts = [("text", X)]
        for i in range(4):
            j = int(perm[i])
            parts += [("image", T, old_pos[j], j * T), ("text", X)]
        return Workload("c3", SHAPES["7b"], [Request(_layout(parts), 0)], 4 * T, "dynamic",
                        budget_bp=500, seed=3)
    if name in ("c4", "c4_5"):
        T, NI, X, B = 1024, 16, 2048, 8
        a = np.random.default_rng(4).choice(np.arange(1, 1025), size=B, replace=False)
        reqs, at = [], 0
        for b in range(B):
            parts = [("text", int(a[b]))]
            parts += [("image", T, j * T, j * T) for j in range(NI)]
            parts += [("text", X - int(a[b]))]
            reqs.append(Request(_layout(parts), at))
            at += X + NI * T
        return Workload(name, SHAPES["7b"], reqs, NI * T, "static",
                        static_k=10 if name == "c4" else 25, seed=4)
    if name == "c5":
        T, NI = 1296, 8
        d = np.random.default_rng(5).integers(0, 4096, size=NI)
        parts = [("image", T, int(j * T + d[j]), j * T) for j in range(NI)] + [("text", 256)]
        return Workload("c5", SHAPES["72b"], [Request(_layout(parts), 0)], NI * T, "dynamic",
                        budget_bp=300, seed=5)
    raise KeyError(name)


# ----------------------------------------------------------------------------------------------
# random tensors
# ----------------------------------------------------------------------------------------------
_CHUNK = 1 << 22   # elements per independently seeded chunk (fixed: results do not depend on threads)


def normal_f32(seed_key: Sequence[int], n: int, scale: float = 1.0, threads: int = 8) -> np.ndarray:
    """n float32 samples of N(0, scale^2); chunk c is drawn from default_rng([*seed_key, c])."""
    out = np.empty(n, dtype=np.float32)
    n_chunks = (n + _CHUNK - 1) // _CHUNK

    def fill(c: int) -> None:
        lo, hi = c * _CHUNK, min(n, (c + 1) * _CHUNK)
        np.random.default_rng([*seed_key, c]).standard_normal(hi - lo, dtype=np.float32, out=out[lo:hi])

    if n_chunks <= 1 or threads <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(n_chunks)))
    if scale != 1.0:
        out *= np.float32(scale)
    return out


WEIGHT_NAMES = ("w_ln1", "w_qkv", "b_qkv", "w_o", "w_ln2", "w_gate_up", "w_down")
QK_NORM_NAMES = ("w_qnorm", "w_knorm")   # only for shapes with qk_norm


def layer_weights(shape: Shape, seed: int, layer: int) -> Dict[str, Optional[np.ndarray]]:
    """Weights of one decoder layer, float32, torch-Linear layout [out, in].

    w_qkv rows: q heads, then k heads, then v heads.  w_gate_up rows: gate (I rows) then up (I rows).
    Linear weights ~ N(0, 0.02^2) (w_o and w_down: N(0, shape.residual_proj_scale^2), the same unless the shape
    says otherwise); norm weights 1 + N(0, 0.02^2); qkv bias N(0, 0.02^2) or None.
    Mixture-of-experts shapes: w_gate_up [E, 2I, H], w_down [E, H, I] and the router matrix
    w_router [E, H] ~ N(0, 0.02^2) (else w_router is None).
    """
    H, I, nq, E = shape.H, shape.I, shape.n_qkv, shape.n_experts
    sizes = {"w_ln1": (H,), "w_qkv": (nq, H), "b_qkv": (nq,), "w_o": (H, shape.Hq * shape.D),
             "w_ln2": (H,), "w_gate_up": (2 * I, H), "w_down": (H, I)}
    if E:
        sizes["w_gate_up"], sizes["w_down"] = (E, 2 * I, H), (E, H, I)
    out: Dict[str, Optional[np.ndarray]] = {}
    for t, nm in enumerate(WEIGHT_NAMES):
        if nm == "b_qkv" and not shape.qkv_bias:
            out[nm] = None
            continue
        n = int(np.prod(sizes[nm]))
        w = normal_f32([seed, 1000 + layer, t], n, shape.residual_proj_scale if nm in ("w_o", "w_down") else 0.02).reshape(sizes[nm])
        if nm in ("w_ln1", "w_ln2"):
            w += np.float32(1.0)
        out[nm] = w
    for t, nm in enumerate(QK_NORM_NAMES):
        out[nm] = (normal_f32([seed, 1000 + layer, 100 + t], shape.D, 0.02) + np.float32(1.0)) if shape.qk_norm else None
    out["w_router"] = normal_f32([seed, 1000 + layer, 200], E * H, 0.02).reshape(E, H) if E else None
    return out


def grid_positions(parts: Sequence[tuple], start: int = 0) -> np.ndarray:
    """3-axis position ids [S, 3] of a prompt made of ("text", n) and ("image", rows, cols) parts, the
    way the Qwen-VL family numbers them: text advances all three axes together; an image starting
    at id p gives its tokens (p, p + row, p + col) in row-major order and the next part starts at
    p + max(rows, cols)."""
    out, p = [], start
    for part in parts:
        if part[0] == "text":
            ids = p + np.arange(part[1])
            out.append(np.stack([ids, ids, ids], axis=1))
            p += part[1]
        else:
            rows, cols = part[1], part[2]
            rr, cc = np.divmod(np.arange(rows * cols), cols)
            out.append(np.stack([np.full(rows * cols, p), p + rr, p + cc], axis=1))
            p += max(rows, cols)
    return np.concatenate(out).astype(np.int64)


def head_weights(shape: Shape, seed: int) -> Dict[str, np.ndarray]:
    """Final norm weight [H] (1 + N(0, 0.02^2)) and output matrix [vocab, H] (N(0, 0.02^2)), float32."""
    w_norm = normal_f32([seed, 3000, 0], shape.H, 0.02) + np.float32(1.0)
    w_lm = normal_f32([seed, 3000, 1], shape.vocab * shape.H, 0.02).reshape(shape.vocab, shape.H)
    return {"w_norm_f": w_norm, "w_lm": w_lm}


def embedding_rows(wl: Workload) -> np.ndarray:
    """Input hidden rows [total_slots, H], float32, for every slot of every request.

    Text slots: rows of a 1024-row N(0, shape.text_scale^2) table (0.02 by default) at random ids.  Image slots: N(0, 1)
    (stand-in for the cached vision-encoder output of that image).
    """
    H = wl.shape.H
    rng = np.random.default_rng([wl.seed, 7])
    table = normal_f32([wl.seed, 8], 1024 * H, wl.shape.text_scale).reshape(1024, H)
    emb = np.empty((wl.total_slots, H), dtype=np.float32)
    for r_i, req in enumerate(wl.requests):
        for s_i, seg in enumerate(req.segments):
            lo = req.kv_start + seg.start
            if seg.is_image:
                emb[lo:lo + seg.length] = normal_f32([wl.seed, 9, r_i, s_i], seg.length * H).reshape(-1, H)
            else:
                emb[lo:lo + seg.length] = table[rng.integers(0, 1024, size=seg.length)]
    return emb


def profile_sample(shape: Shape, seed: int, t_cache_text: int, t_text: int, t_image: int, t_answer: int) -> dict:
    """One sample of the layer-wise sensitivity measurement: an image that was cached under a prompt
    (t_cache_text text rows | image) and is evaluated under another one (t_text text rows | image |
    t_answer answer rows).  Text rows: rows of a 1024-row N(0, text_scale^2) table at random ids
    (different ids for the two prompts); image rows N(0, 1), the same under both prompts.  1-D positions."""
    H = shape.H
    rng = np.random.default_rng([seed, 70])
    table = normal_f32([seed, 71], 1024 * H, shape.text_scale).reshape(1024, H)
    image = normal_f32([seed, 72], t_image * H).reshape(t_image, H)
    cache_emb = np.concatenate([table[rng.integers(0, 1024, size=t_cache_text)], image])
    emb = np.concatenate([table[rng.integers(0, 1024, size=t_text)], image, table[rng.integers(0, 1024, size=t_answer)]])
    cache_request = Request(_layout([("text", t_cache_text), ("image", t_image, t_cache_text, 0)]), 0)
    request = Request(_layout([("text", t_text), ("image", t_image, t_cache_text, 0), ("text", t_answer)]), 0)
    return {"cache_request": cache_request, "cache_emb": cache_emb, "request": request, "emb": emb,
            "answer_rows": np.arange(t_text + t_image, t_text + t_image + t_answer)}


def cached_kv(wl: Workload, layer: int):
    """Cached image K and V pools of one layer, float32 [cache_rows, Hkv, D], N(0, 1)."""
    sh = wl.shape
    n = wl.cache_rows * sh.Hkv * sh.D
    k = normal_f32([wl.seed, 2000 + layer, 0], n).reshape(wl.cache_rows, sh.Hkv, sh.D)
    v = normal_f32([wl.seed, 2000 + layer, 1], n).reshape(wl.cache_rows, sh.Hkv, sh.D)
    return k, v


def sensitivity_table(L: int, G: int, seed: int) -> np.ndarray:
    """Synthetic layer-sensitivity table, float64 [L, G+1]; column c is the score at rate c/500.

    Stand-in for the profiled logit-MSE scores of Sec. 4.1 Eq. 5 (they need trained weights and a
    proxy dataset).  Row i is w_i / (1 + c) with w_i = (L - i) + u_i, u ~ U[0,1): convex in c,
    early layers weighted more.
    """
    u = np.random.default_rng(seed).random(L)
    w = (L - np.arange(L)) + u
    return w[:, None] / (1.0 + np.arange(G + 1, dtype=np.float64))[None, :]
