// vlc_layer_forward: one decoder layer of the selective-recompute prefill, composed from the
// library's kernels on one stream (Sec. 4.1 "Basic Algorithm", Sec. 4.2).
#include <cmath>

#include "vlc_internal.h"

using vlc::fail;

namespace {

inline int64_t align256(int64_t b) { return (b + 255) & ~(int64_t)255; }

struct Workspace {
  int64_t xn, qkv32, q, attn, h1, n2, act, splitk, splitk_bytes, att, att_bytes, total;   // byte offsets
  // mixture-of-experts only (-1 otherwise)
  int64_t moe_idx, moe_w, moe_pos, moe_y, moe_logits, moe_offset, moe_rank, moe_count, moe_tiles, moe_ntiles, moe_row;
};

Workspace layout(const vlc_layer_shape& s, int64_t n) {
  const int64_t es = vlc::elem_size(s.dtype);
  const int64_t nqkv = (int64_t)(s.Hq + 2 * s.Hkv) * s.D;
  Workspace w;
  int64_t at = 0;
  w.xn = at;   at += align256(n * s.H * es);          // input-normed activations
  w.qkv32 = at; at += align256(n * nqkv * 4);         // fused q|k|v rows, unrounded float
  w.q = at;    at += align256(n * (int64_t)s.Hq * s.D * es);   // rotated queries
  w.attn = at; at += align256(n * (int64_t)s.Hq * s.D * es);
  w.h1 = at;   at += align256(n * s.H * es);          // hidden after the attention residual
  w.n2 = at;   at += align256(n * s.H * es);          // post-attention-normed activations
  const int64_t pairs = s.n_experts > 0 ? n * s.top_k : n;
  w.act = at;  at += align256(pairs * (int64_t)s.I * es); // SwiGLU product (per (row, expert) pair with experts)
  w.moe_idx = w.moe_w = w.moe_pos = w.moe_y = w.moe_logits = w.moe_offset = -1;
  w.moe_rank = w.moe_count = w.moe_tiles = w.moe_ntiles = w.moe_row = -1;
  if (s.n_experts > 0) {
    const int64_t E = s.n_experts;
    w.moe_idx = at;    at += align256(pairs * 4);
    w.moe_w = at;      at += align256(pairs * 4);
    w.moe_pos = at;    at += align256(pairs * 4);
    w.moe_y = at;      at += align256(pairs * (int64_t)s.H * es);
    w.moe_logits = at; at += align256(n * E * 4);
    w.moe_offset = at; at += align256((E + 1) * 4);
    w.moe_rank = at;   at += align256(pairs * 4);
    w.moe_count = at;  at += align256(E * 4);
    w.moe_tiles = at;  at += align256((pairs / 64 + E + 1) * (int64_t)sizeof(vlc::GroupTile));   // 64: smallest tile
    w.moe_ntiles = at; at += 256;
    w.moe_row = at;    at += align256(pairs * 4);
  }
  w.splitk = at;                                      // float partials of split-K GEMMs and of tail tiles
  w.splitk_bytes = s.dtype == VLC_BF16 ? vlc::gemm_splitk_ws_bytes(n, nqkv) : 0;
  at += align256(w.splitk_bytes);
  w.att = at;                                         // partials of key-split attention (few rows only)
  w.att_bytes = vlc::attention_ws_bytes(n, s.Hq, s.Hkv, s.D, s.dtype);
  at += align256(w.att_bytes);
  w.total = at;
  return w;
}

int check_shape(const vlc_layer_shape* s, const char* who) {
  if (!s) return fail(VLC_ERR_NULL, "%s: shape is NULL", who);
  if (s->dtype != VLC_F32 && s->dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "%s: dtype=%d", who, s->dtype);
  if (s->H <= 0 || s->Hq <= 0 || s->Hkv <= 0 || s->I <= 0 || s->Hq % s->Hkv)
    return fail(VLC_ERR_SHAPE, "%s: H=%d Hq=%d Hkv=%d I=%d", who, s->H, s->Hq, s->Hkv, s->I);
  if (s->D != 64 && s->D != 128) return fail(VLC_ERR_SHAPE, "%s: D=%d (64 or 128)", who, s->D);
  if (s->dtype == VLC_BF16 && s->D != 128) return fail(VLC_ERR_SHAPE, "%s: bf16 needs D=128", who);
  if (s->H % 64 || s->I % 64 || (s->Hq * s->D) % 64)
    return fail(VLC_ERR_SHAPE, "%s: H, I and Hq*D must be multiples of 64", who);
  if (!(s->rope_base > 0.0) || !(s->eps >= 0.f)) return fail(VLC_ERR_SHAPE, "%s: rope_base/eps", who);
  if (s->mrope_t < 0 || s->mrope_h < 0 || s->mrope_w < 0 ||
      ((s->mrope_t | s->mrope_h | s->mrope_w) != 0 && s->mrope_t + s->mrope_h + s->mrope_w != s->D / 2))
    return fail(VLC_ERR_SHAPE, "%s: 3-axis RoPE sections %d+%d+%d must add up to D/2 = %d", who, s->mrope_t,
                s->mrope_h, s->mrope_w, s->D / 2);
  if (s->n_experts < 0 || s->top_k < 0 || (s->n_experts > 0 && (s->n_experts > 256 || s->top_k < 1 || s->top_k > 16 ||
                                                               s->top_k > s->n_experts)))
    return fail(VLC_ERR_SHAPE, "%s: n_experts=%d (0..256), top_k=%d (1..16, <= n_experts)", who, s->n_experts, s->top_k);
  if (s->dtype == VLC_BF16 && s->n_experts % 4)   // the router scores leave the MFMA GEMM four columns per lane
    return fail(VLC_ERR_SHAPE, "%s: n_experts=%d must be a multiple of 4 in bf16", who, s->n_experts);
  return VLC_OK;
}

}  // namespace

extern "C" int64_t vlc_layer_workspace_bytes(const vlc_layer_shape* shape, int64_t n_rows_max) {
  if (check_shape(shape, "vlc_layer_workspace_bytes")) return 0;
  if (n_rows_max < 0) {
    fail(VLC_ERR_SHAPE, "vlc_layer_workspace_bytes: n_rows_max=%lld", (long long)n_rows_max);
    return 0;
  }
  // The row buffers grow with n; the attention scratch area exists only for small n.  A workspace sized
  // here must serve every call with n <= n_rows_max: take the row buffers at n_rows_max and, for each
  // scratch area, the largest size any smaller n can ask for.
  const vlc_layer_shape& s = *shape;
  const int64_t rows_only = layout(s, n_rows_max).splitk;             // scratch areas come last
  const int64_t g = s.Hq / s.Hkv;
  const int64_t rows_per_tile = g <= 128 ? 128 / g : 1;
  int64_t n_att = ((512 + s.Hkv - 1) / s.Hkv - 1) * rows_per_tile;    // largest n whose attention may split
  if (n_att > n_rows_max) n_att = n_rows_max;
  const int64_t splitk_max = layout(s, n_rows_max).splitk_bytes;      // the same for every row count > 0
  const int64_t att_max = n_att > 0 ? layout(s, n_att).att_bytes : 0;
  return rows_only + align256(splitk_max) + align256(att_max);
}

extern "C" int vlc_layer_workspace_layout(const vlc_layer_shape* shape, int64_t n_rows, int64_t* offsets) {
  int rc = check_shape(shape, "vlc_layer_workspace_layout");
  if (rc) return rc;
  if (!offsets) return fail(VLC_ERR_NULL, "vlc_layer_workspace_layout: offsets is NULL");
  if (n_rows < 0) return fail(VLC_ERR_SHAPE, "vlc_layer_workspace_layout: n_rows=%lld", (long long)n_rows);
  const Workspace w = layout(*shape, n_rows);
  const int64_t o[VLC_WS_FIELDS] = {w.xn,      w.qkv32, w.q,       w.attn,  w.h1,         w.n2,        w.act,
                                    w.moe_idx, w.moe_w, w.moe_pos, w.moe_y, w.moe_logits, w.moe_offset};
  for (int i = 0; i < VLC_WS_FIELDS; ++i) offsets[i] = o[i];
  return VLC_OK;
}

static int layer_forward_impl(const vlc_layer_shape* shape, const vlc_layer_weights* w,
                              const vlc_layer_plan* p, const void* h_in, void* h_out, void* k_cache,
                              void* v_cache, void* workspace, int64_t workspace_bytes, void* stream,
                              void* const* ev, int xn_ready = 0, const void* next_w_ln1 = nullptr,
                              const int32_t* next_row = nullptr) {
  const char* who = "vlc_layer_forward";
  // optional stage timing: ev[i] is recorded before stage i, ev[VLC_LAYER_STAGES] after the last
#define VLC_MARK(i)                                                                     \
  do {                                                                                  \
    if (ev && ev[i]) VLC_CHECK_HIP(hipEventRecord((hipEvent_t)ev[i], (hipStream_t)stream)); \
  } while (0)
  int rc = check_shape(shape, who);
  if (rc) return rc;
  if (!w || !p) return fail(VLC_ERR_NULL, "%s: weights or plan is NULL", who);
  if (p->n < 0 || p->n_in < 0 || p->n_reuse < 0 || p->kv_rows < 0)
    return fail(VLC_ERR_SHAPE, "%s: negative count in plan", who);
  if (p->n > p->n_in) return fail(VLC_ERR_INFEASIBLE, "%s: layer recomputes %lld rows but only %lld were kept above",
                                  who, (long long)p->n, (long long)p->n_in);
  if (!k_cache || !v_cache) return fail(VLC_ERR_NULL, "%s: k_cache/v_cache is NULL", who);
  if (p->n_reuse > 0 && (!p->reuse_src || !p->reuse_dst || !p->reuse_delta || !p->k_pool || !p->v_pool))
    return fail(VLC_ERR_NULL, "%s: reuse list or pool is NULL", who);
  const vlc_layer_shape& s = *shape;
  hipStream_t st = (hipStream_t)stream;
  const bool mrope = s.mrope_t > 0 || s.mrope_h > 0 || s.mrope_w > 0;
  // the reused keys move by one shift common to all axes, so their rotation needs no axis table
  const vlc::RopeFreq freq = vlc::make_rope_freq(s.rope_base, s.D, s.mrope_h, s.mrope_w);

  VLC_MARK(0);
  // Reused image tokens: keys rotated by the position delta, values copied (independent of the rows).
  if (p->n_reuse > 0) {
    rc = vlc::launch_rope_shift(p->k_pool, p->v_pool, k_cache, v_cache, p->reuse_src, p->reuse_dst,
                                p->reuse_delta, p->n_reuse, s.Hkv, s.D, freq, s.dtype, st);
    if (rc) return rc;
  }
  const int64_t n = p->n;
  if (n == 0) {
    for (int i = 1; i <= VLC_LAYER_STAGES; ++i) VLC_MARK(i);
    return VLC_OK;
  }
  if (!w->w_ln1 || !w->w_qkv || !w->w_o || !w->w_ln2 || !w->w_gate_up || !w->w_down)
    return fail(VLC_ERR_NULL, "%s: a weight pointer is NULL", who);
  if (!p->map || !p->slot || !(mrope ? (const void*)p->pos3 : (const void*)p->pos) || !p->row_kv_start ||
      !p->row_kv_len || !h_in || !h_out)
    return fail(VLC_ERR_NULL, "%s: NULL pointer in plan / hidden states", who);
  if (s.n_experts > 0 && !w->w_router) return fail(VLC_ERR_NULL, "%s: w_router is NULL", who);
  if ((w->w_qnorm == nullptr) != (w->w_knorm == nullptr))
    return fail(VLC_ERR_NULL, "%s: w_qnorm and w_knorm come together", who);
  if (h_in == h_out) return fail(VLC_ERR_SHAPE, "%s: h_out must not alias h_in", who);
  const Workspace ws = layout(s, n);
  if (!workspace || workspace_bytes < ws.total)
    return fail(VLC_ERR_WORKSPACE, "%s: workspace of %lld bytes, %lld needed", who, (long long)workspace_bytes,
                (long long)ws.total);
  if ((uintptr_t)workspace & 255) return fail(VLC_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned", who);
  char* base = static_cast<char*>(workspace);
  void* xn = base + ws.xn;
  float* qkv32 = reinterpret_cast<float*>(base + ws.qkv32);
  void* qrot = base + ws.q;
  void* attn = base + ws.attn;
  void* h1 = base + ws.h1;
  void* n2 = base + ws.n2;
  void* act = base + ws.act;
  void* skw = ws.splitk_bytes ? base + ws.splitk : nullptr;
  const int64_t H = s.H, nqkv = (int64_t)(s.Hq + 2 * s.Hkv) * s.D, hqd = (int64_t)s.Hq * s.D, I = s.I;

  // x = h_in[map] is never materialised: the norm reads through the map, and so does the residual.
  // (a chained call finds the normed rows in the workspace: the layer above wrote them with its last kernel)
  VLC_MARK(1);
  if (!xn_ready) {
    rc = vlc::launch_rmsnorm(h_in, p->map, w->w_ln1, xn, n, s.H, s.eps, s.dtype, st);
    if (rc) return rc;
  }
  VLC_MARK(2);
  int qkv_splits = 0;   // > 0: the projection is still split-K partials, summed by the next kernel
  rc = vlc::launch_gemm(xn, H, w->w_qkv, qkv32, nqkv, n, nqkv, H, vlc::EPI_BIAS_F32, w->b_qkv, nullptr, 0,
                        nullptr, s.dtype, skw, ws.splitk_bytes, st, &qkv_splits);
  if (rc) return rc;
  // RoPE at the new positions; fresh k, v overwrite their slots (after the reused tokens were placed).
  VLC_MARK(3);
  rc = vlc::launch_rope_qk_scatter(qkv32, p->pos, p->slot, n, s.Hq, s.Hkv, s.D, freq, qrot, k_cache, v_cache,
                                   s.dtype, st, static_cast<const float*>(skw), qkv_splits > 0 ? qkv_splits : 1,
                                   w->b_qkv, mrope ? p->pos3 : nullptr, w->w_qnorm, w->w_knorm, s.eps);
  if (rc) return rc;
  VLC_MARK(4);
  rc = vlc::launch_attention(qrot, hqd, k_cache, v_cache, p->row_kv_start, p->row_kv_len, n, s.Hq, s.Hkv, s.D,
                             1.0f / sqrtf((float)s.D), attn, s.dtype, ws.att_bytes ? base + ws.att : nullptr,
                             ws.att_bytes, p->kv_rows, st);
  if (rc) return rc;
  VLC_MARK(5);
  int o_splits = 0;
  rc = vlc::launch_gemm(attn, hqd, w->w_o, h1, H, n, H, hqd, vlc::EPI_RESIDUAL, nullptr, h_in, H, p->map,
                        s.dtype, skw, ws.splitk_bytes, st, &o_splits);
  if (rc) return rc;
  VLC_MARK(6);
  if (o_splits > 0)   // split-K partials: sum + residual -> h1 and the norm of h1 in one kernel
    rc = vlc::launch_sum_residual_rmsnorm(static_cast<const float*>(skw), o_splits, h_in, p->map, w->w_ln2, h1,
                                          n2, n, s.H, s.eps, st);
  else
    rc = vlc::launch_rmsnorm(h1, nullptr, w->w_ln2, n2, n, s.H, s.eps, s.dtype, st);
  if (rc) return rc;
  VLC_MARK(7);
  if (s.n_experts > 0) {
    // router scores (float), expert choice and grouping, then the experts' gate|up GEMMs with SwiGLU over the
    // (row, expert) pairs in grouped order (rows of n2 fetched through the position -> row list)
    const int E = s.n_experts, K = s.top_k;
    const int64_t pairs = n * K;
    float* logits = reinterpret_cast<float*>(base + ws.moe_logits);
    vlc::MoeScratch ms;
    ms.idx = reinterpret_cast<int32_t*>(base + ws.moe_idx);
    ms.wts = reinterpret_cast<float*>(base + ws.moe_w);
    ms.rank = reinterpret_cast<int32_t*>(base + ws.moe_rank);
    ms.count = reinterpret_cast<int32_t*>(base + ws.moe_count);
    ms.offset = reinterpret_cast<int32_t*>(base + ws.moe_offset);
    ms.tiles = reinterpret_cast<vlc::GroupTile*>(base + ws.moe_tiles);
    ms.n_tiles = reinterpret_cast<int32_t*>(base + ws.moe_ntiles);
    ms.pair_row = reinterpret_cast<int32_t*>(base + ws.moe_row);
    ms.pair_pos = reinterpret_cast<int32_t*>(base + ws.moe_pos);
    void* y = base + ws.moe_y;
    const int tile_rows = vlc::gemm_group_tile_rows(pairs, E, s.dtype);
    int r_splits = 0;    // > 0: the scores are still split-K partials, summed by the choice kernel
    rc = vlc::launch_gemm(n2, H, w->w_router, logits, E, n, E, H,
                          s.dtype == VLC_BF16 ? vlc::EPI_BIAS_F32 : vlc::EPI_BIAS, nullptr, nullptr, 0, nullptr,
                          s.dtype, skw, ws.splitk_bytes, st, &r_splits);
    if (rc) return rc;
    rc = vlc::launch_moe_route(r_splits > 0 ? static_cast<const float*>(skw) : logits, r_splits > 0 ? r_splits : 1,
                               n * E, r_splits > 0 ? logits : nullptr, n, E, K, tile_rows, ms, st);
    if (rc) return rc;
    rc = vlc::launch_gemm_grouped(n2, H, ms.pair_row, w->w_gate_up, 2 * I * H, act, I, pairs, E, I, H,
                                  vlc::EPI_SWIGLU, ms.tiles, ms.n_tiles, tile_rows, s.dtype, st, n);
    if (rc) return rc;
    VLC_MARK(8);
    rc = vlc::launch_gemm_grouped(act, I, nullptr, w->w_down, H * I, y, H, pairs, E, H, I, vlc::EPI_BIAS, ms.tiles,
                                  ms.n_tiles, tile_rows, s.dtype, st, pairs);
    if (rc) return rc;
    if (next_w_ln1)   // chained: the weighted sum and the input norm of the layer below in one kernel
      rc = vlc::launch_moe_combine_norm(h1, y, ms.wts, ms.pair_pos, n, K, s.H, h_out, next_w_ln1, xn, next_row,
                                        s.eps, s.dtype, st);
    else
      rc = vlc::launch_moe_combine(h1, y, ms.wts, ms.pair_pos, n, K, s.H, h_out, s.dtype, st);
    if (rc) return rc;
    VLC_MARK(9);
    return VLC_OK;
  }
  rc = vlc::launch_gemm(n2, H, w->w_gate_up, act, I, n, I, H, vlc::EPI_SWIGLU, nullptr, nullptr, 0, nullptr,
                        s.dtype, skw, ws.splitk_bytes, st);
  if (rc) return rc;
  VLC_MARK(8);
  // Chained: the input norm of the layer below is taken here, where the rows of h_out are at hand - with a
  // split k range in the kernel that sums the partials, so h_out is not read back and one launch goes.
  int down_splits = 0;
  rc = vlc::launch_gemm(act, I, w->w_down, h_out, H, n, H, I, vlc::EPI_RESIDUAL, nullptr, h1, H, nullptr,
                        s.dtype, skw, ws.splitk_bytes, st, next_w_ln1 ? &down_splits : nullptr);
  if (rc) return rc;
  if (next_w_ln1) {
    if (down_splits > 0)
      rc = vlc::launch_sum_residual_rmsnorm(static_cast<const float*>(skw), down_splits, h1, nullptr, next_w_ln1,
                                            h_out, xn, n, s.H, s.eps, st, next_row);
    else
      rc = vlc::launch_rmsnorm(h_out, nullptr, next_w_ln1, xn, n, s.H, s.eps, s.dtype, st, next_row);
    if (rc) return rc;
  }
  VLC_MARK(9);
  return VLC_OK;
#undef VLC_MARK
}

extern "C" int vlc_layer_forward(const vlc_layer_shape* shape, const vlc_layer_weights* w,
                                 const vlc_layer_plan* p, const void* h_in, void* h_out, void* k_cache,
                                 void* v_cache, void* workspace, int64_t workspace_bytes, void* stream) {
  return layer_forward_impl(shape, w, p, h_in, h_out, k_cache, v_cache, workspace, workspace_bytes, stream,
                            nullptr);
}

extern "C" int vlc_layer_forward_timed(const vlc_layer_shape* shape, const vlc_layer_weights* w,
                                       const vlc_layer_plan* p, const void* h_in, void* h_out, void* k_cache,
                                       void* v_cache, void* workspace, int64_t workspace_bytes, void* stream,
                                       void* const* stage_events) {
  if (!stage_events) return fail(VLC_ERR_NULL, "vlc_layer_forward_timed: stage_events is NULL");
  return layer_forward_impl(shape, w, p, h_in, h_out, k_cache, v_cache, workspace, workspace_bytes, stream,
                            stage_events);
}

extern "C" int vlc_layer_forward_chained(const vlc_layer_shape* shape, const vlc_layer_weights* w,
                                         const vlc_layer_plan* p, const void* h_in, void* h_out, void* k_cache,
                                         void* v_cache, void* workspace, int64_t workspace_bytes, void* stream,
                                         int input_norm_ready, const void* next_w_ln1, const int32_t* next_row,
                                         void* const* stage_events) {
  if (input_norm_ready != 0 && input_norm_ready != 1)
    return fail(VLC_ERR_SHAPE, "vlc_layer_forward_chained: input_norm_ready=%d (0 or 1)", input_norm_ready);
  return layer_forward_impl(shape, w, p, h_in, h_out, k_cache, v_cache, workspace, workspace_bytes, stream,
                            stage_events, input_norm_ready, next_w_ln1, next_w_ln1 ? next_row : nullptr);
}

// ---------------------------------------------------------------------------------------------
// first output token: final RMSNorm of one row per request, output matrix, greedy choice
// ---------------------------------------------------------------------------------------------
extern "C" int64_t vlc_first_token_workspace_bytes(int H, int64_t n_req, int dtype) {
  if (H <= 0 || n_req < 0 || (dtype != VLC_F32 && dtype != VLC_BF16)) {
    fail(VLC_ERR_SHAPE, "vlc_first_token_workspace_bytes: H=%d n_req=%lld dtype=%d", H, (long long)n_req, dtype);
    return 0;
  }
  return align256(n_req * (int64_t)H * (dtype == VLC_BF16 ? 2 : 4)) +   // the normed rows
         align256(vlc::argmax_ws_bytes(n_req));                           // partial choices
}

extern "C" int vlc_first_token(const void* h, const int32_t* rows, int64_t n_req, int H, int64_t vocab,
                               float eps, const void* w_norm, const void* w_out, float* logits,
                               int32_t* token, void* workspace, int64_t workspace_bytes, int dtype,
                               void* stream) {
  const char* who = "vlc_first_token";
  if (dtype != VLC_F32 && dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "%s: dtype=%d", who, dtype);
  if (n_req < 0 || H <= 0 || H % 64 || vocab <= 0 || vocab % 4 || !(eps >= 0.f))
    return fail(VLC_ERR_SHAPE, "%s: n_req=%lld H=%d vocab=%lld (H multiple of 64, vocab multiple of 4)", who,
                (long long)n_req, H, (long long)vocab);
  if (n_req == 0) return VLC_OK;
  if (!h || !rows || !w_norm || !w_out || !logits || !token) return fail(VLC_ERR_NULL, "%s: NULL pointer", who);
  const int64_t need = vlc_first_token_workspace_bytes(H, n_req, dtype);
  if (!workspace || workspace_bytes < need)
    return fail(VLC_ERR_WORKSPACE, "%s: workspace of %lld bytes, %lld needed", who, (long long)workspace_bytes,
                (long long)need);
  if ((uintptr_t)workspace & 255) return fail(VLC_ERR_WORKSPACE, "%s: workspace must be 256-byte aligned", who);
  hipStream_t st = (hipStream_t)stream;
  int rc = vlc::launch_rmsnorm(h, rows, w_norm, workspace, n_req, H, eps, dtype, st);
  if (rc) return rc;
  // The output matrix is streamed once (vocab * H elements) by the GEMM: 128-row MFMA tiles whose few real rows are
  // the requests - HBM-bound whatever the count (a kernel that kept the rows in LDS and formed the products with
  // dot instructions was slower from two requests on: every 16 bytes of the matrix cost a 16-byte LDS read per row).
  rc = vlc::launch_gemm(workspace, H, w_out, logits, vocab, n_req, vocab, H, vlc::EPI_BIAS_F32, nullptr, nullptr, 0,
                        nullptr, dtype, nullptr, 0, st);
  if (rc) return rc;
  char* part = static_cast<char*>(workspace) + align256(n_req * (int64_t)H * (dtype == VLC_BF16 ? 2 : 4));
  return vlc::launch_argmax_rows(logits, n_req, vocab, token, part, st);
}
