/*
 * vlcache.h - C ABI of the selective-recompute prefill library for MI355X (gfx950).
 *
 * The library implements the per-layer hot path of VLCache (arxiv 2512.12977): a cached
 * image's vision-token K/V is reused at a new, non-prefix position and only the text tokens
 * plus a leading fraction of each image's tokens are recomputed in every decoder layer
 * (Sec. 4.1 "Basic Algorithm", Sec. 4.2, Fig. 4).
 *
 * Conventions
 *   - Every function returns VLC_OK (0) or a VLC_ERR_* code; vlc_last_error() gives the text of
 *     the calling thread's last failure.  Nothing throws across this boundary.
 *   - The caller owns all memory.  The library never allocates or frees device memory; scratch
 *     space is a caller-provided workspace sized by vlc_layer_workspace_bytes().
 *   - "host" pointers are read/written by the CPU inside the call.  "device" pointers are only
 *     handed to kernels.  Device functions enqueue work on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and return without synchronising.
 *   - Tensors are dense, row-major.  dtype is VLC_F32 or VLC_BF16 and applies to every tensor
 *     of a call (weights included).  Index arrays are int32.
 *   - K/V storage is token-major: [rows, Hkv, D] per layer.  Linear weights use the
 *     [out_features, in_features] layout.
 *   - Device functions launch kernels and nothing else (no allocation, no synchronisation, no memset
 *     node), so their calls can be recorded into a HIP graph.  The first launch of a kernel variant
 *     on a device sets one attribute of that kernel (its dynamic LDS size, once per device and
 *     kernel, thread-safe): run the calls once eagerly, as a warm-up, before capturing them.
 *   - A call with zero rows is a no-op that returns VLC_OK.
 *   - Contents of device index arrays are the caller's contract (in range; scatter targets
 *     unique); the host-side builders below produce arrays that satisfy it.
 */
#ifndef VLCACHE_H_
#define VLCACHE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  VLC_OK = 0,
  VLC_ERR_NULL = 1,       /* a required pointer is NULL */
  VLC_ERR_SHAPE = 2,      /* a size is negative, zero where it must not be, or unsupported */
  VLC_ERR_DTYPE = 3,      /* dtype is not VLC_F32 / VLC_BF16 */
  VLC_ERR_INDEX = 4,      /* a host-side index / segment description is inconsistent */
  VLC_ERR_WORKSPACE = 5,  /* workspace too small or misaligned */
  VLC_ERR_HIP = 6,        /* a HIP runtime call failed (text in vlc_last_error) */
  VLC_ERR_INFEASIBLE = 7  /* the requested plan violates the method's constraints */
};

enum { VLC_F32 = 0, VLC_BF16 = 1 };

/* Rates live on the grid k/500 (step 0.002, Sec. 4.1 Eq. 9). */
#define VLC_RATE_GRID 500
/* Largest grid step the allocator assigns (rate 0.300, Sec. 4.1 Eq. 9). */
#define VLC_PLANNER_MAX_STEP 150

const char* vlc_last_error(void);
int vlc_version(void);

/* ------------------------------------------------------------------------------------------
 * Host-side planning
 * ---------------------------------------------------------------------------------------- */

/*
 * Layer-aware budget allocation (Sec. 4.1 "Dynamic Recomputation", Eq. 6-9): choose grid
 * steps k[0..L) (rate k/500) that approximately minimise sum_i sens[i][k_i] subject to
 * sum_i k_i <= budget_steps, k_0 >= k_1 >= ... >= k_{L-1} >= 0 and k_i <= G.
 * Greedy: from all zeros, repeatedly add one step to the layer whose score drops the most,
 * among layers that stay <= G and keep the sequence non-increasing; the drop must be > 0;
 * equal drops go to the lowest layer index; stops when the budget is spent or no layer
 * qualifies.  The result is unique.
 * Limitation: from all zeros only layer 0 can move under Eq. 8, so a table whose first layer's scores do not
 * fall (measured tables: layer 0's cached keys/values do not depend on the prompt, Sec. 3.2) yields the
 * all-zero plan with VLC_OK and the budget unspent; use vlc_plan_layer_rates_blocks for such tables.
 *   sens   host, [L][G+1] doubles, column c = score of that layer at rate c/500
 *   k_out  host, [L] int32, written
 * Errors: NULL pointers, L <= 0, G <= 0 or G > VLC_RATE_GRID, budget_steps < 0.
 */
int vlc_plan_layer_rates(int L, int G, const double* sens, int64_t budget_steps, int32_t* k_out);

/*
 * The same problem (Eq. 6-9) with moves that raise a whole run of equal layers.  Sec. 3.2 notes that
 * some layers gain nothing from recomputation, yet Eq. 8 keeps every deeper layer at or below them: with
 * flat scores in the shallow layers (the first layer's always are - its cached keys/values do not depend
 * on the prompt) the one-step greedy above stops at zero.  Here a move raises layers a..j by one step,
 * a..j-1 being exactly the layers before j at j's level; it costs j-a+1 steps and gains the sum of their
 * score drops (summed in layer order).  Among affordable moves with positive gain the largest gain per
 * step wins (compared as gain * other_cost > other_gain * cost; equal: the smallest j).  Arguments,
 * errors and uniqueness as vlc_plan_layer_rates.
 */
int vlc_plan_layer_rates_blocks(int L, int G, const double* sens, int64_t budget_steps, int32_t* k_out);

/*
 * One run of consecutive slots of a request inside the packed K/V of a batch.
 *   start      first packed slot of the run
 *   length     number of tokens
 *   is_image   non-zero: vision tokens whose K/V are available in the cache pool
 *   pos        position id of the run's first token in the new request
 *   old_pos    position id the cached key of the run's first token was rotated at (0 for keys
 *              stored before RoPE, Sec. 4.2)
 *   cache_row  row of the run's first token in the cache pool
 *   kv_start   first packed slot of the request this run belongs to
 * Runs must be given in ascending slot order, must not overlap, and the runs of one request
 * must be adjacent.
 */
typedef struct {
  int32_t start, length, is_image, pos, old_pos, cache_row, kv_start;
} vlc_segment;

/*
 * Token selection for every layer (Sec. 4.2: the first floor(r*T) tokens of each T-token
 * image are recomputed; Sec. 4.1: they are concatenated with the text tokens; rates must not
 * increase with depth so that each layer's rows exist in the layer above).
 *   k          host [L], grid step of each layer, 0..500; count = (k*T) / 500 (integer floor)
 *   count_override host [L] or NULL: if given, layer l recomputes min(T, count_override[l])
 *              leading tokens of every image instead (k is then ignored and may be NULL)
 *   cap        row capacity of each per-layer output array
 * Outputs (host, int32, [L][cap] unless noted; only the first n_rows[l] entries are written):
 *   n_rows [L] number of recomputed rows
 *   slot       packed slot of each recomputed row, ascending
 *   map        index of that row in the previous layer's row list (layer 0: the packed slot
 *              itself, i.e. the row of the input embedding matrix)
 *   pos        position id of the row
 *   kv_start   first packed slot of the row's request
 *   kv_len     number of leading slots of its request the row attends to (slot-kv_start+1)
 * Any output pointer except n_rows may be NULL to skip it.
 * Errors: VLC_ERR_INDEX for malformed segments, VLC_ERR_INFEASIBLE if a layer would recompute
 * more tokens of some image than the layer above, VLC_ERR_SHAPE if cap is too small.
 */
int vlc_plan_token_indices(int n_seg, const vlc_segment* seg, int L, const int32_t* k,
                           const int32_t* count_override, int64_t cap, int32_t* n_rows,
                           int32_t* slot, int32_t* map, int32_t* pos, int32_t* kv_start,
                           int32_t* kv_len);

/*
 * Where each row of a layer goes in the layer below (Sec. 4.1, last paragraph / Eq. 8: rates do not increase
 * with depth, so the rows of layer l+1 are a subset of those of layer l): next_row[l][i] = index of row i of
 * layer l among the rows of layer l+1, or -1 if layer l+1 drops it - the inverse of that layer's `map`
 * (next_row[l][map[l+1][j]] == j).  The last layer's entries are all -1.  This is the list
 * vlc_layer_forward_chained takes.  Output host int32 [L][cap], the first n_rows[l] entries of each layer
 * written; k / count_override / cap rules and errors as vlc_plan_token_indices.
 */
int vlc_plan_next_rows(int n_seg, const vlc_segment* seg, int L, const int32_t* k,
                       const int32_t* count_override, int64_t cap, int32_t* next_row);

/*
 * Budget of the allocator from a mean recomputation rate (Eq. 7 bounds the sum of the layers' rates; Sec. 5.1
 * quotes mean rates): a mean of mean_rate_bp / 10000 over L layers is mean_rate_bp * L / 20 steps of the
 * 0.002 grid, rounded down.  steps: host, written.  Errors: NULL, mean_rate_bp outside 0..10000, L <= 0.
 */
int vlc_plan_budget_steps(int mean_rate_bp, int L, int64_t* steps);

/*
 * The complementary list: image tokens that are reused (not recomputed) in each layer, with the
 * cache-pool row they come from, the packed slot they go to, and the position delta
 * (new position - old_pos) their cached key must be rotated by (Sec. 4.2).
 * Outputs host int32 [L][cap], first n_reuse[l] entries written; same k / count_override rules.
 */
int vlc_plan_reuse_rows(int n_seg, const vlc_segment* seg, int L, const int32_t* k,
                        const int32_t* count_override, int64_t cap, int32_t* n_reuse,
                        int32_t* src_row, int32_t* dst_slot, int32_t* delta);

/* ------------------------------------------------------------------------------------------
 * Device kernels of the hot path (all pointers below are DEVICE pointers unless noted)
 * ---------------------------------------------------------------------------------------- */

/*
 * Row gather: dst[i, :] = src[idx[i], :], i in [0, n)  (Sec. 4.2: the computation mask indexes
 * the input hidden states and only the selected rows go on).
 *   src [src_rows, row_elems], dst [n, row_elems]; row_elems * elem size must be a multiple of 16.
 */
int vlc_gather_rows(const void* src, int64_t src_rows, int64_t row_elems, const int32_t* idx,
                    int64_t n, void* dst, int dtype, void* stream);

/*
 * Re-rotate reused keys to their new position and place reused K/V into the request's K/V
 * (Sec. 4.2: K/V are stored position-free and RoPE is applied for the new position; with keys
 * stored already rotated at old_pos the same rotation by delta = new - old applies, because
 * rotations compose).
 *   k_dst[dst_row[t]] = R(delta[t]) * k_src[src_row[t]]     t in [0, n_tok)
 *   v_dst[dst_row[t]] = v_src[src_row[t]]                   (skipped if v_src or v_dst is NULL)
 * R(d) rotates the pair (x[i], x[i + D/2]) of every head by the angle d * rope_base^(-2i/D):
 *   lo' = lo cos - hi sin, hi' = hi cos + lo sin.  delta may be negative.
 * k_src/v_src [src_rows, Hkv, D], k_dst/v_dst [dst_rows, Hkv, D].  In-place use
 * (k_dst == k_src with dst_row[t] == src_row[t]) is allowed; any other overlap is not.
 * Angles are formed in double precision and reduced before the float sine/cosine.
 * D must be 64 or 128.
 */
int vlc_rope_shift_kv(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                      const int32_t* src_row, const int32_t* dst_row, const int32_t* delta,
                      int64_t n_tok, int Hkv, int D, double rope_base, int dtype, void* stream);

/*
 * The same for several independent jobs in one launch - the reused keys of all layers of a prompt (Sec. 4.2):
 * the cached K/V of every layer and the position shifts are known before the first layer runs and depend
 * on nothing the layers compute, so the per-layer calls can be replaced by one call ahead of the layer
 * loop; the layers are then run with n_reuse = 0.
 *   jobs: DEVICE array [n_jobs] of vlc_shift_job records, 8-byte aligned (all its pointers device, same meaning,
 *         layouts and aliasing rules as the arguments of vlc_rope_shift_kv; v_src/v_dst NULL: keys only).
 *         Jobs must not write rows another job reads or writes.  The table must stay valid until the
 *         kernel has run.
 *   max_n_tok: host-side upper bound of every job's n_tok (sizes the grid; a job with a larger n_tok
 *         is processed only up to max_n_tok tokens).  Jobs with n_tok = 0 are skipped.
 * The library cannot check a device table: row indices and pointers in it are the caller's responsibility.
 */
typedef struct {
  const void* k_src;
  const void* v_src;
  void* k_dst;
  void* v_dst;
  const int32_t* src_row;
  const int32_t* dst_row;
  const int32_t* delta;
  int64_t n_tok;
} vlc_shift_job;
int vlc_rope_shift_kv_layers(const vlc_shift_job* jobs, int n_jobs, int64_t max_n_tok, int Hkv, int D,
                             double rope_base, int dtype, void* stream);

/*
 * KV blend (Sec. 4.2 "fine-grained KV cache reuse"): fresh K/V rows of the recomputed tokens
 * overwrite their slots.  k_cache[dst_row[i]] = k_new[i], v_cache[dst_row[i]] = v_new[i].
 *   k_new, v_new [n, Hkv, D]; k_cache, v_cache [cache_rows, Hkv, D]; dst_row entries unique.
 */
int vlc_scatter_kv(const void* k_new, const void* v_new, const int32_t* dst_row, int64_t n,
                   void* k_cache, void* v_cache, int64_t cache_rows, int Hkv, int D, int dtype,
                   void* stream);

/*
 * Attention for the recomputed query rows only, against the whole blended K/V (Fig. 4):
 *   out[i, h] = softmax_j( scale * q[i, h] . K[s_i + j, h / g] ) @ V[s_i + j, h / g],
 *   j in [0, row_kv_len[i]),  s_i = row_kv_start[i],  g = Hq / Hkv.
 * Rows with row_kv_len 0 produce zeros.  Rows of one request (equal row_kv_start) must be
 * adjacent; lengths need not be sorted.
 *   q, out [n, Hq, D]; k_cache, v_cache [*, Hkv, D].  D must be 64 or 128 (bf16: 128 only).
 * bf16: scores and softmax in float, probabilities rounded to bf16 before the PV product.
 */
int vlc_sparse_q_attention(const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* row_kv_start, const int32_t* row_kv_len, int64_t n,
                           int Hq, int Hkv, int D, float scale, void* out, int dtype,
                           void* stream);

/* ------------------------------------------------------------------------------------------
 * One decoder layer of the selective-recompute prefill
 * ---------------------------------------------------------------------------------------- */
typedef struct {
  int32_t H, Hq, Hkv, D, I;   /* hidden, query heads, kv heads, head dim, MLP width */
  int32_t dtype;              /* VLC_F32 | VLC_BF16 */
  float eps;                  /* RMSNorm epsilon */
  double rope_base;
  /* 3-axis RoPE (Qwen3-VL family, the paper's main models, Sec. 5.1): numbers of rotation
   * frequencies driven by the temporal / height / width position id, interleaved over the frequency
   * index i: height takes i = 1, 4, 7, ... below 3*mrope_h, width i = 2, 5, 8, ... below 3*mrope_w,
   * the temporal id the rest.  All three 0: ordinary 1-D RoPE (plan->pos).  Otherwise the ids of
   * the recomputed rows come from plan->pos3. */
  int32_t mrope_t, mrope_h, mrope_w;
  /* Mixture-of-experts MLP (the Qwen3-VL-30B-A3B model of Sec. 5.1): n_experts > 0 replaces the MLP
   * by n_experts SwiGLU experts of width I each, of which every row uses top_k (1 <= top_k <= 16,
   * n_experts <= 256, in bf16 a multiple of 4): router scores row . w_router^T, the top_k largest (equal scores: lower index
   * first), weights = softmax over all experts renormalised over the chosen ones; the experts'
   * output rows are rounded to the storage type and summed in float.  0: one dense MLP. */
  int32_t n_experts, top_k;
} vlc_layer_shape;

typedef struct {              /* device pointers; b_qkv may be NULL (no bias) */
  const void* w_ln1;          /* [H] */
  const void* w_qkv;          /* [(Hq+2Hkv)*D, H], rows: q heads, k heads, v heads */
  const void* b_qkv;          /* [(Hq+2Hkv)*D] or NULL */
  const void* w_o;            /* [H, Hq*D] */
  const void* w_ln2;          /* [H] */
  const void* w_gate_up;      /* [2I, H], rows: gate then up */
  const void* w_down;         /* [H, I] */
  const void* w_qnorm;        /* [D] or NULL: RMSNorm weight applied to every q head before RoPE (Qwen3 family) */
  const void* w_knorm;        /* [D] or NULL: the same for every k head; both or neither */
  const void* w_router;       /* [n_experts, H] when n_experts > 0 (then w_gate_up is [n_experts, 2I, H] and
                                 w_down [n_experts, H, I]), else ignored */
} vlc_layer_weights;

typedef struct {
  int64_t n_in;                 /* rows of h_in (the previous layer's output rows) */
  int64_t n;                    /* rows recomputed by this layer */
  const int32_t* map;           /* device [n]: row of h_in each recomputed row comes from */
  const int32_t* slot;          /* device [n]: packed K/V slot of each row (scatter target); a negative entry:
                                   the row is computed and attends, but its fresh k, v are not stored - what the
                                   cache holds at its slot stays (used by the sensitivity measurement, Sec. 3.2) */
  const int32_t* pos;           /* device [n]: position id of each row */
  const int32_t* row_kv_start;  /* device [n] */
  const int32_t* row_kv_len;    /* device [n] */
  int64_t kv_rows;              /* rows of k_cache / v_cache */
  int64_t n_reuse;              /* reused image tokens to place before attention (may be 0) */
  const int32_t* reuse_src;     /* device [n_reuse]: row in k_pool / v_pool */
  const int32_t* reuse_dst;     /* device [n_reuse]: packed slot in k_cache / v_cache */
  const int32_t* reuse_delta;   /* device [n_reuse]: new position - cached position */
  const void* k_pool;           /* device [pool_rows, Hkv, D] cached image keys of this layer */
  const void* v_pool;           /* device [pool_rows, Hkv, D] */
  int64_t pool_rows;
  /* device [n, 3] (temporal, height, width ids of the recomputed rows) when the shape has 3-axis
   * RoPE, else NULL (pos is then not read).  A reused image keeps its grid, so all three ids of all
   * its tokens move by one amount: reuse_delta stays one number per reused token. */
  const int32_t* pos3;
} vlc_layer_plan;

/* Bytes of workspace vlc_layer_forward needs for up to n_rows_max recomputed rows (0 on error). */
int64_t vlc_layer_workspace_bytes(const vlc_layer_shape* shape, int64_t n_rows_max);

/*
 * Where the intermediate results of the last vlc_layer_forward call with n_rows recomputed rows
 * live inside its workspace (byte offsets; for tests and profilers, which check each stage of the
 * layer in place).  offsets (host, [VLC_WS_FIELDS]): input-normed rows [n,H]; q|k|v projection
 * before RoPE as float [n,(Hq+2Hkv)D]; rotated queries [n,Hq,D]; attention output [n,Hq,D];
 * hidden after the attention residual [n,H]; post-attention-normed rows [n,H]; SwiGLU product
 * [n,I].  All but the second have the layer's storage type.  With experts the seventh is
 * [n*top_k, I] in grouped order and six more follow: chosen experts [n,top_k] int32, their weights
 * [n,top_k] float, position of every (row, choice) pair in the grouped order [n,top_k] int32, the
 * experts' output rows [n*top_k, H] (storage type, grouped order), router scores [n, n_experts]
 * float, first pair of every expert [n_experts + 1] int32.  Without experts these six are -1.
 */
#define VLC_WS_FIELDS 13
int vlc_layer_workspace_layout(const vlc_layer_shape* shape, int64_t n_rows, int64_t* offsets);

/*
 * One layer (Sec. 4.1 "Basic Algorithm" / Sec. 4.2; decoder details follow the Qwen family the
 * paper evaluates): for the n recomputed rows
 *   x  = h_in[map]                       gather of the retained rows
 *   q,k,v = RMSNorm(x) Wqkv^T + b ;  optional per-head RMSNorm of q, k ;  RoPE(q), RoPE(k) at pos (or pos3)
 *   K/V: reused image tokens placed (keys rotated by reuse_delta), then K[slot]=k, V[slot]=v
 *   a  = attention of the n rows over K/V[row_kv_start : row_kv_start + row_kv_len)
 *   h1 = x + a Wo^T ;  h_out = h1 + (silu(n2 Wg^T) * (n2 Wu^T)) Wd^T,  n2 = RMSNorm(h1)
 *        (with experts: h_out = h1 + sum over the row's top_k experts of weight * that expert's MLP)
 * h_in [n_in, H], h_out [n, H] (must not alias h_in), k_cache/v_cache [kv_rows, Hkv, D] updated
 * in place.  Storage rounding for VLC_BF16: normed activations, v after bias, q and k after
 * RoPE (rounded once: the projection is rotated as float), attention output, both residual sums
 * and the SwiGLU product are bf16; accumulation, softmax, RoPE and norms are computed in float.  workspace must be 256-byte aligned.
 * Supported: D in {64,128} for VLC_F32, D == 128 for VLC_BF16; H, I, Hq*D multiples of 64.
 */
int vlc_layer_forward(const vlc_layer_shape* shape, const vlc_layer_weights* weights,
                      const vlc_layer_plan* plan, const void* h_in, void* h_out, void* k_cache,
                      void* v_cache, void* workspace, int64_t workspace_bytes, void* stream);

/*
 * vlc_layer_forward with per-stage timing marks, for benchmarks: stage_events (host array of
 * VLC_LAYER_STAGES + 1 hipEvent_t handles created by the caller) - event i is recorded on `stream`
 * before stage i starts, the last one after the final stage; a NULL entry records nothing (each
 * recorded event costs a few microseconds of stream time, so a caller interested in one stage
 * passes only the two events around it).  Stages, in launch order:
 *   0 reused K/V placement (RoPE shift)   1 input RMSNorm (reads h_in through map)
 *   2 q|k|v projection                    3 RoPE of q,k + scatter of fresh k,v
 *   4 attention of the recomputed rows    5 output projection + residual
 *   6 post-attention RMSNorm              7 gate|up projection + SwiGLU     8 down projection + residual
 * Everything else is identical to vlc_layer_forward.
 */
#define VLC_LAYER_STAGES 9
int vlc_layer_forward_timed(const vlc_layer_shape* shape, const vlc_layer_weights* weights,
                            const vlc_layer_plan* plan, const void* h_in, void* h_out, void* k_cache,
                            void* v_cache, void* workspace, int64_t workspace_bytes, void* stream,
                            void* const* stage_events);

/*
 * vlc_layer_forward for consecutive layers of one prefill (Sec. 4.1, last paragraph / Eq. 8: rates do not
 * increase with depth, which makes the rows of a layer a subset of those of the layer above): the input RMSNorm of the layer below is produced by this
 * layer's last kernel - the one that sums the down projection's partial products when its k range is
 * split - instead of a kernel of its own at the head of the next call.  Results equal vlc_layer_forward's
 * bit for bit.
 *   next_w_ln1 (device [H], or NULL): input-norm weight of the layer below.  Non-NULL: after h_out, the
 *     rows RMSNorm(h_out) * next_w_ln1 that the layer below recomputes are left in the workspace (its first
 *     field, see vlc_layer_workspace_layout), in that layer's row order.  The layer below must run next on
 *     the same workspace and stream, with a plan whose n_in equals this plan's n, and input_norm_ready = 1.
 *   next_row (device [n] int32, or NULL; read only with next_w_ln1): for every row of this layer its index
 *     among the rows of the layer below, negative if that layer drops it - the inverse of that layer's
 *     `map`: next_row[map_below[j]] == j for all j < n_below.  NULL: the layer below keeps every row
 *     (n_below == n, map_below[i] == i).
 *   input_norm_ready (0 or 1): 1 = the workspace already holds this layer's input-normed rows, left by the
 *     call for the layer above as described; h_in is then read only for the residual.
 *   stage_events: NULL, or as in vlc_layer_forward_timed (stage 1 is empty when input_norm_ready is 1,
 *     stage 8 includes the norm when next_w_ln1 is given).
 * With next_w_ln1 == NULL and input_norm_ready == 0 this is vlc_layer_forward(_timed).  n == 0: nothing is
 * written, also not the normed rows.
 */
int vlc_layer_forward_chained(const vlc_layer_shape* shape, const vlc_layer_weights* weights,
                              const vlc_layer_plan* plan, const void* h_in, void* h_out, void* k_cache,
                              void* v_cache, void* workspace, int64_t workspace_bytes, void* stream,
                              int input_norm_ready, const void* next_w_ln1, const int32_t* next_row,
                              void* const* stage_events);

/*
 * First output token of each request - where the paper's time-to-first-token ends (Sec. 5.1; Tables
 * 2-5 report TTFT).  The paper does not describe the output stage; as in the Qwen decoders it
 * evaluates, row rows[r] of the last layer's output h [n, H] (the request's last slot, a text token
 * and therefore always recomputed) goes through the final RMSNorm (weight w_norm [H], eps) and the
 * output matrix w_out [vocab, H] (row-major, no bias):
 *   logits[r, v] = sum_c RMSNorm(h[rows[r]])[c] * w_out[v, c]     float, not rounded
 *   token[r]     = index of the largest logits[r, :], the lowest index among equal ones
 * The normed row is rounded to `dtype` before the product (storage contract of the layer).
 * All pointers are device memory: h, w_norm, w_out of `dtype`; rows int32 [n_req] with values in
 * [0, n) (not checked); logits float [n_req, vocab]; token int32 [n_req]; workspace of at least
 * vlc_first_token_workspace_bytes(H, n_req, dtype) bytes, 256-byte aligned, caller-owned like every
 * buffer.  Requirements: H a multiple of 64, vocab a multiple of 4, n_req >= 0 (0: no-op).
 * Errors: VLC_ERR_NULL, VLC_ERR_SHAPE, VLC_ERR_DTYPE, VLC_ERR_WORKSPACE, VLC_ERR_HIP (launch failure).
 * Enqueues four kernels on `stream` and returns without synchronising.
 */
int64_t vlc_first_token_workspace_bytes(int H, int64_t n_req, int dtype);
int vlc_first_token(const void* h, const int32_t* rows, int64_t n_req, int H, int64_t vocab, float eps,
                    const void* w_norm, const void* w_out, float* logits, int32_t* token, void* workspace,
                    int64_t workspace_bytes, int dtype, void* stream);

/*
 * vlc_first_token for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as vlc_first_token without the
 * workspace pair: the scratch (normed rows + partial choices) is a device array built into the library,
 * vlc_first_token_noalloc_max_bytes() = 1 MiB per GPU, which every GPU the entry point is called on holds until
 * the process ends.  The call allocates and frees nothing and enqueues the same four kernels on `stream`.
 * Limit: vlc_first_token_workspace_bytes(H, n_req, dtype) must not exceed that size (bf16: 128 requests at
 * H = 3584, 60 at H = 8192), else VLC_ERR_WORKSPACE and nothing is enqueued.  All calls on one GPU share the
 * array: calls that may overlap on one GPU (different streams, several threads) race on it and must be ordered
 * by the caller; nothing in it needs clearing between calls.
 */
int64_t vlc_first_token_noalloc_max_bytes(void);
int vlc_first_token_noalloc(const void* h, const int32_t* rows, int64_t n_req, int H, int64_t vocab, float eps,
                            const void* w_norm, const void* w_out, float* logits, int32_t* token, int dtype,
                            void* stream);

/*
 * Mean squared difference of two float arrays, the error measure of the layer-wise sensitivity
 * score S_i(r) = E MSE(z_orig, z_reuse) (Sec. 4.1, Eq. 5): out[0] = sum_i (a[i] - b[i])^2 / n,
 * accumulated in double.  a, b: device float [n]; out: device double [1]; workspace: device, at
 * least vlc_mean_squared_error_workspace_bytes() bytes, 8-byte aligned, caller-owned.
 * Errors: VLC_ERR_SHAPE (n <= 0), VLC_ERR_NULL, VLC_ERR_WORKSPACE, VLC_ERR_HIP.  Enqueues two kernels.
 */
int64_t vlc_mean_squared_error_workspace_bytes(void);
int vlc_mean_squared_error(const float* a, const float* b, int64_t n, double* out, void* workspace,
                           int64_t workspace_bytes, void* stream);

/*
 * Measurement aid, no part of the method: one launch of a register-only loop of v_mfma_f32_32x32x16_bf16 on every
 * CU (one workgroup per CU, waves_per_simd wavefronts per SIMD, iters x 8 MFMAs per wavefront on operands read once
 * from `operands`), against which bench.py sets the rates of the GEMM and attention kernels: with operands of random
 * bits it shows what the matrix pipe delivers at the clock the chip sustains under a real kernel's power draw.
 *   operands: device, >= 131072 bytes of bf16 data, 16-byte aligned; out: device float [>= CUs * 256 * waves_per_simd]
 *   (written, content meaningless); flops: host, receives the flops of the launch.  Enqueues one kernel.
 * Errors: VLC_ERR_NULL, VLC_ERR_SHAPE (iters <= 0, waves_per_simd not 1 or 2, buffers too small), VLC_ERR_HIP.
 */
int vlc_probe_mfma_bf16(const void* operands, int64_t operand_bytes, float* out, int64_t out_elems, int iters,
                        int waves_per_simd, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VLCACHE_H_ */
