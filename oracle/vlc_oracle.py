"""CPU oracle for VLCache's selective-recompute prefill (arxiv 2512.12977).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the HIP path is
checked against.  It may be imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py, and by nothing else; it shares no code with the
HIP library and never calls it.

What it computes (Sec. 4.1 "Basic Algorithm", Sec. 4.2, Fig. 4): a request reuses the
cached K/V of its image tokens at a new position.  In every decoder layer only the
text tokens and the first floor(r * T) tokens of each T-token image are run through
the layer; their fresh K/V overwrite the reused entries, reused keys are rotated to
the new position, and causal attention is evaluated for those query rows only, over
the whole blended key range.  Rates are non-increasing with depth (Sec. 4.1, last
paragraph), so the rows a layer needs are always among the rows the layer above
produced.  Per-layer rates come from a greedy allocation over a sensitivity table
(Sec. 4.1 "Dynamic Recomputation", Eq. 6-9).

The method is an approximation of full prefill by design, so there is no closed
form for its output; the functions below follow the algorithm's steps in the
paper's order.  All arithmetic is float64.  `store` is the rounding applied where
the GPU path keeps a tensor in its storage type (identity for the fp32 config,
bf16 round-to-nearest-even for the bf16 configs).

Readings of points the paper leaves open are marked "reading:" where they apply.

Pins (tests/test_oracle_*.py): rate 1.0 equals full prefill; exact-prefix reuse at
rate 0 equals full prefill; the same with every position shifted by a constant;
rope_shift(d) o rope_shift(-d) = id and composition with direct RoPE; brute-force
dense attention on tiny inputs; planner closed forms and exhaustive optimum; the first-token
head against a Hugging Face Qwen2 causal LM with the same weights, and closed forms.
Parity unpinned: agreement with the authors' own rate lists / prototype numerics
(their code and tables are not available); the sensitivity measurement (profile_prefill,
sensitivity_profile) is pinned by invariants only - the paper prints no value of S_i(r).
"""
from __future__ import annotations

import numpy as np

GRID = 500          # rates live on the grid k/500, k integer (step 0.002; Sec. 4.1 Eq. 9)
PLANNER_G = 150     # largest grid step the allocator may assign (rate 0.300; Eq. 9)


# ----------------------------------------------------------------------------------------------
# storage rounding
# ----------------------------------------------------------------------------------------------
def store_exact(x):
    """Storage rounding of the fp32 configuration: none (the oracle stays in float64)."""
    return np.asarray(x, dtype=np.float64)


def store_bf16(x):
    """Round float64 to the nearest bfloat16 value (ties to even); result kept as float64.

    bfloat16 has 8 significant bits.  Only the normal range is handled (all tensors on this
    path are O(1)); zeros pass through.
    """
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                      # x = m * 2**e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0), e - 8)


STORE = {"f32": store_exact, "bf16": store_bf16}


# ----------------------------------------------------------------------------------------------
# layer-rate allocation (Sec. 4.1, Eq. 6-9)
# ----------------------------------------------------------------------------------------------
def plan_layer_rates(sens, budget_steps, G=None):
    """Greedy allocation of per-layer grid steps k_i (rate r_i = k_i / 500).

    sens[i][c] is the sensitivity score of layer i at rate c/500 (column 0 = pure reuse).
    Minimises sum_i sens[i][k_i] approximately, subject to sum_i k_i <= budget_steps,
    k_0 >= k_1 >= ... >= k_{L-1} >= 0 and k_i <= G.

    reading: the paper only says "a simple greedy algorithm".  Taken as: start from all
    zeros; repeatedly raise by one step the layer whose next step lowers its score the
    most, among layers that stay within G and within the monotone constraint; the drop
    must be positive; equal drops go to the shallowest layer; stop when the budget is
    used or no layer qualifies.
    reading: Eq. 6 prints sum over l of S_i(r); taken as sum over i of S_i(r_i).
    reading: the grid is printed from 0.002 but Eq. 8 allows r_L >= 0 and Sec. 3.2 says some
    layers should recompute nothing, so step 0 is allowed.
    """
    sens = np.asarray(sens, dtype=np.float64)
    L = sens.shape[0]
    if G is None:
        G = sens.shape[1] - 1
    k = [0] * L
    used = 0
    while used < budget_steps:
        best, best_gain = -1, 0.0
        for i in range(L):
            if k[i] >= G:
                continue
            if i > 0 and k[i] + 1 > k[i - 1]:
                continue
            gain = sens[i][k[i]] - sens[i][k[i] + 1]
            if gain > best_gain:
                best, best_gain = i, gain
        if best < 0:
            break
        k[best] += 1
        used += 1
    return np.asarray(k, dtype=np.int32)


def plan_layer_rates_blocks(sens, budget_steps, G=None):
    """Greedy allocation as plan_layer_rates, with moves that raise a whole run of equal layers at once.

    reading: Sec. 3.2 observes that some layers gain nothing from recomputation, while Eq. 8 forces a
    deeper layer's rate below every shallower one's.  When the shallow layers' scores are flat (the first
    layer's always are: its cached keys/values do not depend on the prompt) the one-step greedy cannot
    raise any deeper layer and stops at zero.  The paper does not say how its greedy handles this; taken
    here as the smallest change that does: a move raises by one step the layers a..j, where a..j-1 are
    exactly the layers before j that sit at j's level (they have to rise with it, Eq. 8); it costs
    j-a+1 steps and gains the sum of the layers' score drops; among affordable moves with positive gain
    the largest gain per step wins (equal: the smallest j).  With a = j this is the one-step move.
    """
    sens = np.asarray(sens, dtype=np.float64)
    L = sens.shape[0]
    if G is None:
        G = sens.shape[1] - 1
    S = [[float(v) for v in row] for row in sens]
    k = [0] * L
    used = 0
    while used < budget_steps:
        best_j, best_a, best_gain, best_cost = -1, 0, 0.0, 1
        for j in range(L):
            if k[j] >= G:
                continue
            a = j
            while a > 0 and k[a - 1] == k[j]:
                a -= 1
            cost = j - a + 1
            if used + cost > budget_steps:
                continue
            gain = 0.0
            for i in range(a, j + 1):
                gain = gain + (S[i][k[i]] - S[i][k[i] + 1])
            if not gain > 0.0:
                continue
            # gain / cost > best_gain / best_cost, without dividing
            if best_j < 0 or gain * best_cost > best_gain * cost:
                best_j, best_a, best_gain, best_cost = j, a, gain, cost
        if best_j < 0:
            break
        for i in range(best_a, best_j + 1):
            k[i] += 1
        used += best_cost
    return np.asarray(k, dtype=np.int32)


def budget_steps_from_mean_rate(mean_rate_bp, L):
    """reading: Eq. 7 bounds the *sum* of rates while the tables quote a *mean* rate; the budget
    is given as a mean rate in basis points and converted to a total number of grid steps:
    bp/10000 * L * 500 = bp * L / 20, rounded down."""
    return (int(mean_rate_bp) * int(L)) // 20


# ----------------------------------------------------------------------------------------------
# token selection (Sec. 4.2: first floor(r*T) tokens of each image; Sec. 4.1: query tokens and
# selected tokens are concatenated)
# ----------------------------------------------------------------------------------------------
def leading_count(k, T):
    """floor(r * T) with r = k/500, in integer arithmetic."""
    return (int(k) * int(T)) // GRID


def select_slots(segments, counts):
    """Slots (relative to the request start, ascending) recomputed in one layer.

    counts[j] = number of leading tokens of the j-th *image* segment to recompute.
    reading: every non-image slot is recomputed in every layer, wherever it sits.
    """
    out, j = [], 0
    for seg in segments:
        if seg.is_image:
            out.extend(range(seg.start, seg.start + counts[j]))
            j += 1
        else:
            out.extend(range(seg.start, seg.start + seg.length))
    return np.asarray(out, dtype=np.int64)


def image_counts(segments, k=None, explicit=None):
    """Per-image leading-token counts for one layer from a grid step k or an explicit count."""
    res = []
    for seg in segments:
        if seg.is_image:
            res.append(min(seg.length, explicit) if explicit is not None else leading_count(k, seg.length))
    return res


def reused_slots(segments, counts):
    """(slot, cache_row, delta) of every image token that is NOT recomputed in this layer, where
    delta = new position - position the cached key was rotated at.  Positions are slot indices
    (plus the request's pos_start, which cancels in delta only if the cache used the same origin;
    the caller adds pos_start to `slot` when forming delta)."""
    slot, row, old = [], [], []
    j = 0
    for seg in segments:
        if not seg.is_image:
            continue
        for t in range(counts[j], seg.length):
            slot.append(seg.start + t)
            row.append(seg.cache_row + t)
            old.append(seg.old_pos + t)
        j += 1
    return (np.asarray(slot, dtype=np.int64), np.asarray(row, dtype=np.int64),
            np.asarray(old, dtype=np.int64))


# ----------------------------------------------------------------------------------------------
# rotary position embedding
# ----------------------------------------------------------------------------------------------
def rope_axes(D, section):
    """Which position axis (0 temporal, 1 height, 2 width) drives each of the D/2 rotation frequencies
    under 3-axis RoPE with `section` = (t, h, w) frequency counts.

    reading: the paper's main models are Qwen3-VL decoders (Sec. 5.1) and it does not restate their
    rotary layout; that family interleaves the axes over the frequency index i: height takes
    i = 1, 4, 7, ... below 3 * section[1], width i = 2, 5, 8, ... below 3 * section[2], the
    temporal axis everything else.  An empty section means ordinary 1-D RoPE (axis 0 everywhere).
    """
    ax = np.zeros(D // 2, dtype=np.int64)
    if section:
        i = np.arange(D // 2)
        ax[(i % 3 == 1) & (i < 3 * section[1])] = 1
        ax[(i % 3 == 2) & (i < 3 * section[2])] = 2
    return ax


def rope_angles(pos, D, base, section=()):
    """angle[t, i] = pos[t, axis(i)] * base**(-2 i / D), i in [0, D/2); pos [n] (one id for all axes) or [n, 3]."""
    i = np.arange(D // 2, dtype=np.float64)
    inv_freq = np.power(np.float64(base), -2.0 * i / D)
    pos = np.asarray(pos, dtype=np.float64)
    if pos.ndim == 1:
        return pos[:, None] * inv_freq[None, :]
    return pos[:, rope_axes(D, section)] * inv_freq[None, :]


def rope_rotate(x, pos, base, section=()):
    """Rotate x[t, head, :] by the angles of position pos[t] (may be negative).

    reading: the paper does not give the pairing; the Qwen-family convention is used: element i
    pairs with element i + D/2;  lo' = lo cos - hi sin,  hi' = hi cos + lo sin.
    Because rotations compose, calling this on keys that were already rotated at position q with
    pos = p - q leaves them rotated at p (Sec. 4.2 stores keys un-rotated, i.e. q = 0); with 3-axis
    positions that holds axis by axis, and a shift common to all axes is a 1-D pos.
    """
    x = np.asarray(x, dtype=np.float64)
    D = x.shape[-1]
    half = D // 2
    ang = rope_angles(pos, D, base, section)
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


# ----------------------------------------------------------------------------------------------
# decoder layer pieces
# ----------------------------------------------------------------------------------------------
def rmsnorm(x, w, eps):
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(w, dtype=np.float64)


def silu(x):
    return x / (1.0 + np.exp(-x))


def attention_rows(q, K, V, kv_len, scale):
    """o[i, h] = softmax(scale * q[i, h] . K[0:kv_len[i], h // g]) @ V[0:kv_len[i], h // g].

    q [n, Hq, D]; K, V [S, Hkv, D]; kv_len[i] = number of leading slots row i may see
    (its own slot + 1: causal in slot order).  Rows with kv_len 0 give zeros.
    Fig. 4: only the rows of recomputed tokens are evaluated, each over its whole key range.
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    n, Hq, D = q.shape
    S, Hkv, _ = K.shape
    g = Hq // Hkv
    kv_len = np.asarray(kv_len, dtype=np.int64)
    visible = np.arange(S)[None, :] < kv_len[:, None]           # [n, S]
    out = np.zeros((n, Hq, D), dtype=np.float64)
    for h in range(Hq):
        s = (q[:, h, :] @ K[:, h // g, :].T) * scale             # [n, S]
        s = np.where(visible, s, -np.inf)
        m = np.max(s, axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        p = np.exp(s - m)
        den = np.sum(p, axis=1, keepdims=True)
        p = np.where(den > 0, p / np.where(den > 0, den, 1.0), 0.0)
        out[:, h, :] = p @ V[:, h // g, :]
    return out


def linear(x, w, b=None):
    y = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T
    if b is not None:
        y = y + np.asarray(b, dtype=np.float64)
    return y


def route_top_k(logits, top_k):
    """Expert choice of a mixture-of-experts MLP: softmax over all experts, the top_k most probable
    (equal values: the lower expert index first), their probabilities renormalised to sum 1.
    logits [n, E] -> (idx [n, top_k] in order of decreasing probability, weight [n, top_k])."""
    logits = np.asarray(logits, dtype=np.float64)
    z = logits - np.max(logits, axis=1, keepdims=True)
    p = np.exp(z)
    p = p / np.sum(p, axis=1, keepdims=True)
    idx = np.argsort(-p, axis=1, kind="stable")[:, :top_k]          # stable: ties keep index order
    w = np.take_along_axis(p, idx, axis=1)
    return idx.astype(np.int64), w / np.sum(w, axis=1, keepdims=True)


def moe_mlp(shape, W, n2, store, forced=None):
    """Mixture-of-experts SwiGLU MLP of the normed rows n2 [n, H] (without the residual).

    reading (the paper's Qwen3-VL-30B-A3B model; it does not restate the block): router scores
    n2 . w_router^T, expert choice by route_top_k, every chosen expert e applies its own SwiGLU MLP
    (w_gate_up[e] rows: gate then up; w_down[e]) and the results are summed with the renormalised
    probabilities as weights.
    reading (storage rounding): router scores, probabilities and weights stay unrounded floats; the
    SwiGLU product and each expert's output row are tensors of the storage type; the weighted sum
    is formed in float.
    Returns dict: moe_idx [n, k], moe_w [n, k], act [n, k, I], y [n, k, H], mlp [n, H] (float sum).
    forced: optional moe_idx / moe_w / act / y to feed to the following step instead.
    """
    forced = forced or {}
    fed = lambda name, value: np.asarray(forced[name]) if name in forced else value
    n2 = np.asarray(n2, dtype=np.float64)
    n, k, I = n2.shape[0], shape.top_k, shape.I
    r = {}
    r["moe_idx"], r["moe_w"] = route_top_k(linear(n2, W["w_router"]), k)
    idx = fed("moe_idx", r["moe_idx"]).astype(np.int64)
    wts = np.asarray(fed("moe_w", r["moe_w"]), dtype=np.float64)
    act = np.zeros((n, k, I), dtype=np.float64)
    for e in np.unique(idx):
        rows, j = np.nonzero(idx == e)
        gu = linear(n2[rows], W["w_gate_up"][e])
        act[rows, j] = store(silu(gu[:, :I]) * gu[:, I:])
    r["act"] = act
    act = np.asarray(fed("act", act), dtype=np.float64)
    y = np.zeros((n, k, shape.H), dtype=np.float64)
    for e in np.unique(idx):
        rows, j = np.nonzero(idx == e)
        y[rows, j] = store(linear(act[rows, j], W["w_down"][e]))
    r["y"] = y
    y = np.asarray(fed("y", y), dtype=np.float64)
    r["mlp"] = np.einsum("nk,nkh->nh", wts, y)
    return r


STAGES = ("xn", "qkv", "q", "K", "V", "o", "h1", "n2", "act", "h2")


def layer_stages(shape, W, x, slots, pos, K, V, store, forced=None, kv_rows=None):
    """One decoder layer for the query rows `slots` of one request; returns every stage's result.

    x      [n, H]  hidden states of those rows (already gathered, storage-rounded)
    slots  [n]     their slot indices (ascending)
    pos    [n]     their position ids, or [n, 3] (temporal, height, width) under 3-axis RoPE
    K, V   [S, Hkv, D]  the request's keys/values for this layer with every slot that is NOT in
           `slots` already filled (reused image tokens, rotated to their new position); rows at
           `slots` are overwritten here with the fresh k, v  (the blend of Sec. 4.2).
    forced optional dict stage-name -> array: where present, the NEXT stage is fed this value
           instead of the one computed here (used by tests to check each stage of another
           implementation against this one on identical inputs).
    kv_rows optional indices into the row list: only these rows store their fresh k, v (default: all);
           the other rows are still computed and still attend, but the keys/values already in K, V at
           their slots stay (the layer-wise sensitivity measurement of Sec. 3.2 needs this).
    Returns a dict with the stages named in STAGES; K and V are the blended caches (updated in place).

    reading (decoder details, which the paper leaves to the Qwen family): pre-norm RMSNorm,
    fused q|k|v projection with optional bias, rotate-half RoPE on q and k, grouped-query
    attention scaled by 1/sqrt(D), output projection + residual, SwiGLU MLP + residual.
    reading (storage rounding of the bf16 path): the weights themselves (they are tensors of the
    storage type), normed activations, v after bias, q and k after
    RoPE (once: the projection result is rotated unrounded), attention output, both residual sums
    and the SwiGLU product are rounded to the storage type; gate and up projections are not
    rounded before the product.
    """
    Hq, Hkv, D = shape.Hq, shape.Hkv, shape.D
    n = x.shape[0]
    forced = forced or {}
    fed = lambda name, value: np.asarray(forced[name], dtype=np.float64) if name in forced else value
    r = {}
    x = np.asarray(x, dtype=np.float64)
    W = {name: (None if w is None else store(w)) for name, w in W.items()}
    r["xn"] = store(rmsnorm(x, W["w_ln1"], shape.eps))
    r["qkv"] = linear(fed("xn", r["xn"]), W["w_qkv"], W.get("b_qkv"))
    qkv = fed("qkv", r["qkv"])
    q = qkv[:, :Hq * D].reshape(n, Hq, D)
    k = qkv[:, Hq * D:(Hq + Hkv) * D].reshape(n, Hkv, D)
    if W.get("w_qnorm") is not None:
        # reading (Qwen3 family, the paper's main models): RMSNorm over the head dimension of every
        # q and k head, before the rotation; unrounded like the projection it follows
        q = rmsnorm(q, W["w_qnorm"], shape.eps)
        k = rmsnorm(k, W["w_knorm"], shape.eps)
    section = getattr(shape, "mrope_section", ())
    r["q"] = store(rope_rotate(q, pos, shape.rope_base, section))
    k = store(rope_rotate(k, pos, shape.rope_base, section))
    v = store(qkv[:, (Hq + Hkv) * D:].reshape(n, Hkv, D))
    if kv_rows is None:
        K[slots] = k
        V[slots] = v
    else:
        K[np.asarray(slots)[kv_rows]] = k[kv_rows]
        V[np.asarray(slots)[kv_rows]] = v[kv_rows]
    r["K"], r["V"] = K, V
    r["o"] = store(attention_rows(fed("q", r["q"]), fed("K", K), fed("V", V), np.asarray(slots) + 1,
                                  1.0 / np.sqrt(D)))
    r["h1"] = store(x + linear(fed("o", r["o"]).reshape(n, Hq * D), W["w_o"]))
    h1 = fed("h1", r["h1"])
    r["n2"] = store(rmsnorm(h1, W["w_ln2"], shape.eps))
    if W.get("w_router") is not None:
        m = moe_mlp(shape, W, fed("n2", r["n2"]), store, forced)
        r.update({name: m[name] for name in ("moe_idx", "moe_w", "act", "y")})
        r["h2"] = store(h1 + m["mlp"])
        return r
    gu = linear(fed("n2", r["n2"]), W["w_gate_up"])
    r["act"] = store(silu(gu[:, :shape.I]) * gu[:, shape.I:])
    r["h2"] = store(h1 + linear(fed("act", r["act"]), W["w_down"]))
    return r


def layer_forward(shape, W, x, slots, pos, K, V, store, kv_rows=None):
    """layer_stages without the intermediate results: (h_out [n, H], K, V)."""
    r = layer_stages(shape, W, x, slots, pos, K, V, store, kv_rows=kv_rows)
    return r["h2"], r["K"], r["V"]


def blended_kv_before_scatter(shape, request, counts, Kc, Vc, store):
    """K, V [S, Hkv, D] of one layer with the reused image tokens filled in: keys rotated by
    (new position - cached position), values copied; all other slots zero (they are overwritten
    by fresh k, v in layer_forward).  Sec. 4.2: reused tokens take their K/V from the cache and
    RoPE is applied for the new position."""
    S = request.S
    K = np.zeros((S, shape.Hkv, shape.D), dtype=np.float64)
    V = np.zeros((S, shape.Hkv, shape.D), dtype=np.float64)
    slot, row, old = reused_slots(request.segments, counts)
    if slot.size:
        if getattr(request, "pos3", None) is not None:
            # 3-axis ids: a reused image keeps its grid, so every axis of every token moves by the
            # shift of the image's first (temporal) id; `old` counts from that id token by token
            t_in_seg = np.concatenate([np.arange(c, seg.length) for seg, c in
                                       zip([g for g in request.segments if g.is_image], counts)])
            delta = np.asarray(request.pos3)[slot, 0] - (old - t_in_seg)
        else:
            delta = (request.pos_start + slot) - old
        K[slot] = store(rope_rotate(np.asarray(Kc, dtype=np.float64)[row], delta, shape.rope_base))
        V[slot] = np.asarray(Vc, dtype=np.float64)[row]
    return K, V


def selective_prefill(shape, weights, emb, request, counts_per_layer, cache, store):
    """Selective-recompute prefill of one request through all layers.

    weights[l]           dict of layer l (torch-Linear layout [out, in])
    emb [S, H]           input hidden rows of every slot of the request
    counts_per_layer[l]  per-image leading-token counts of layer l (non-increasing in l)
    cache[l] = (Kc, Vc)  cached image K/V pools of layer l
    Returns a list over layers of dicts {slots, h, K, V}: recomputed slots, their output hidden
    rows, and the blended K/V of that layer.
    """
    emb = store(emb)
    out = []
    prev_slots = np.arange(request.S, dtype=np.int64)
    prev_h = emb
    for l, W in enumerate(weights):
        counts = counts_per_layer[l]
        slots = select_slots(request.segments, counts)
        # rows of this layer are a subset of the rows the previous layer produced (Sec. 4.1)
        where = np.searchsorted(prev_slots, slots)
        if where.size and (where.max() >= prev_slots.size or np.any(prev_slots[where] != slots)):
            raise ValueError("layer %d recomputes a token the previous layer dropped" % l)
        x = prev_h[where]
        Kc, Vc = cache[l]
        K, V = blended_kv_before_scatter(shape, request, counts, store(Kc), store(Vc), store)
        h, K, V = layer_forward(shape, W, x, slots, positions_of(request, slots), K, V, store)
        out.append({"slots": slots, "h": h, "K": K, "V": V})
        prev_slots, prev_h = slots, h
    return out


def positions_of(request, slots):
    """Position ids of the given slots: [n], or [n, 3] when the request carries 3-axis ids."""
    if getattr(request, "pos3", None) is not None:
        return np.asarray(request.pos3, dtype=np.int64)[slots]
    return request.pos_start + np.asarray(slots, dtype=np.int64)


def full_prefill(shape, weights, emb, request, store):
    """Ordinary causal prefill of every slot (the cache-miss path of Sec. 4.1, and the
    'r = 1.0 (full-recompute)' column of the accuracy tables)."""
    S = request.S
    slots = np.arange(S, dtype=np.int64)
    h = store(emb)
    out = []
    for W in weights:
        K = np.zeros((S, shape.Hkv, shape.D), dtype=np.float64)
        V = np.zeros((S, shape.Hkv, shape.D), dtype=np.float64)
        h, K, V = layer_forward(shape, W, h, slots, positions_of(request, slots), K, V, store)
        out.append({"slots": slots, "h": h, "K": K, "V": V})
    return out


# ----------------------------------------------------------------------------------------------
# layer-wise sensitivity S_i(r) (Sec. 3.2 "Layer-wise Importance Difference", Sec. 4.1 Eq. 5)
# ----------------------------------------------------------------------------------------------
def profile_prefill(shape, weights, emb, request, layer_i, counts_i, cache, store):
    """The measurement pass behind Eq. 5: the image keys/values of a cache built under another prompt
    are used in ALL layers, and only in layer `layer_i` the leading counts_i[j] tokens of image j
    keep their freshly computed k, v.  Returns the last layer's hidden rows of every slot [S, H].

    reading: Sec. 3.2 injects the mismatched cache into all layers while recomputing some image
    tokens "in a single layer".  A token can only be recomputed in layer i if its hidden state
    reaches layer i, which the fast path's non-increasing rates guarantee but a single-layer
    recompute does not; so this measurement computes every slot in every layer (an ordinary forward
    pass) and overrides which keys/values the attention sees: cached ones for image tokens, except
    the chosen tokens in layer i.  Image rows still attend and still feed the next layer.
    """
    S = request.S
    slots = np.arange(S, dtype=np.int64)
    n_img = sum(1 for g in request.segments if g.is_image)
    h = store(emb)
    for l, W in enumerate(weights):
        counts = list(counts_i) if l == layer_i else [0] * n_img
        Kc, Vc = cache[l]
        K, V = blended_kv_before_scatter(shape, request, counts, store(Kc), store(Vc), store)
        reused, _, _ = reused_slots(request.segments, counts)
        keep = np.setdiff1d(slots, reused)
        h, K, V = layer_forward(shape, W, h, slots, positions_of(request, slots), K, V, store, kv_rows=keep)
    return h


def sensitivity_profile(shape, weights, head, samples, steps, store):
    """S[i, j] = mean over samples of MSE(z_orig, z_reuse(i, steps[j])) (Eq. 5), steps on the k/500 grid.

    Each sample is a dict:
      cache_request, cache_emb   the prompt the cache is built under (replacement text | image) and its rows
      request, emb               the evaluated prompt (text | image | answer); its image segments point into
                                 the cache (old_pos = position under the cache prompt, cache_row)
      answer_rows                slots whose output scores are compared (the decoding text)
    Phases (Sec. 3.2): (1) full prefill of the cache prompt, its image K/V per layer are the cache;
    (2) full prefill of the evaluated prompt gives z_orig; (3) for every layer i and step k the pass
    of profile_prefill gives z_reuse(i, k).  MSE = mean over answer rows and vocabulary of the squared
    score difference.
    """
    L = len(weights)
    out = np.zeros((L, len(steps)), dtype=np.float64)
    for smp in samples:
        creq = smp["cache_request"]
        full_c = full_prefill(shape, weights, smp["cache_emb"], creq, store)
        img = np.concatenate([g.start + np.arange(g.length) for g in creq.segments if g.is_image])
        cache = [(full_c[l]["K"][img], full_c[l]["V"][img]) for l in range(L)]
        req = smp["request"]
        rows = np.asarray(smp["answer_rows"], dtype=np.int64)
        z_orig = first_token_logits(shape, head, full_prefill(shape, weights, smp["emb"], req, store)[-1]["h"][rows], store)
        for i in range(L):
            for j, k in enumerate(steps):
                counts = image_counts(req.segments, k=int(k))
                h = profile_prefill(shape, weights, smp["emb"], req, i, counts, cache, store)
                z = first_token_logits(shape, head, h[rows], store)
                out[i, j] += np.mean((z - z_orig) ** 2)
    return out / max(len(samples), 1)


# ----------------------------------------------------------------------------------------------
# first output token (what the paper's time-to-first-token ends with; Sec. 5.1 "TTFT", Tables 2-5)
# ----------------------------------------------------------------------------------------------
def first_token_logits(shape, Wh, h_last, store):
    """Output scores of the rows h_last [m, H] of the last layer (one row per request: its last slot).

    reading: the paper measures time to the first token but does not describe the output stage;
    the Qwen decoders it evaluates end with a final RMSNorm (weight Wh["w_norm_f"]) followed by the
    output matrix Wh["w_lm"] [vocab, H] without bias, and that is what is computed here.  The normed
    row is rounded to the storage type, the scores are not.
    """
    w_norm = store(Wh["w_norm_f"])
    w_lm = store(Wh["w_lm"])
    xn = store(rmsnorm(store(h_last), w_norm, shape.eps))
    return linear(xn, w_lm)


def first_token(logits):
    """Greedy choice: index of the largest score of every row; of equal scores the lowest index.

    reading: the first token is taken greedily (the paper reports latency, not a sampling rule).
    """
    return np.argmax(np.asarray(logits, dtype=np.float64), axis=-1).astype(np.int64)
