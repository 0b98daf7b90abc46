// Internal helpers shared by the library's translation units (not part of the C ABI).
#ifndef VLC_INTERNAL_H_
#define VLC_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "vlcache.h"

namespace vlc {

// Records the message for vlc_last_error() and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

inline int elem_size(int dtype) { return dtype == VLC_BF16 ? 2 : 4; }

#define VLC_CHECK_HIP(expr)                                                              \
  do {                                                                                   \
    hipError_t e_ = (expr);                                                              \
    if (e_ != hipSuccess)                                                                \
      return ::vlc::fail(VLC_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));    \
  } while (0)

#define VLC_CHECK_LAUNCH(name)                                                           \
  do {                                                                                   \
    hipError_t e_ = hipGetLastError();                                                   \
    if (e_ != hipSuccess)                                                                \
      return ::vlc::fail(VLC_ERR_HIP, "launch of %s failed: %s", name,                   \
                         hipGetErrorString(e_));                                         \
  } while (0)

// Raises a kernel's dynamic-LDS limit to `bytes`, once per (device, kernel): thread-safe, keyed by the current
// device (the attribute belongs to the kernel's code object on that device).  Returns VLC_OK or VLC_ERR_HIP.
int ensure_dynamic_lds(const void* kernel, int bytes);

// RoPE inverse frequencies theta_i = base^(-2i/D), i < D/2, in double; passed to kernels by value.
// axis[i]: which position id (0 temporal, 1 height, 2 width) drives frequency i (all 0: 1-D RoPE).
struct RopeFreq {
  double inv_freq[64];
  unsigned char axis[64];
};
RopeFreq make_rope_freq(double base, int D, int mrope_h = 0, int mrope_w = 0);

// ---- internal launchers (enqueue only; arguments already validated by the callers) ----------

// dst[i,:] = src[idx[i],:] in 16-byte chunks; row_bytes % 16 == 0.  idx may be NULL (identity).
int launch_gather_rows(const void* src, int64_t row_bytes, const int32_t* idx, int64_t n, void* dst,
                       hipStream_t st);

// y[ymap ? ymap[i] : i, :] = rmsnorm(x[map ? map[i] : i, :]) * w; rows with ymap[i] < 0 are skipped
int launch_rmsnorm(const void* x, const int32_t* map, const void* w, void* y, int64_t n, int H,
                   float eps, int dtype, hipStream_t st, const int32_t* ymap = nullptr);

// bf16 path, after a GEMM that left `splits` float partial matrices [splits][n][H]:
// h = round(sum of partials + resid[rmap ? rmap[i] : i]) (stored), y[ymap ? ymap[i] : i] = RMSNorm(h) * w
// (no norm for rows with ymap[i] < 0).
int launch_sum_residual_rmsnorm(const float* partials, int splits, const void* resid, const int32_t* rmap,
                                const void* w, void* h, void* y, int64_t n, int H, float eps,
                                hipStream_t st, const int32_t* ymap = nullptr);

// out[r] = index of the largest x[r, :] (lowest index among equals); x float [rows, cols], cols % 4 == 0;
// ws: argmax_ws_bytes(rows) bytes of scratch (8-byte aligned)
int launch_argmax_rows(const float* x, int64_t rows, int64_t cols, int32_t* out, void* ws, hipStream_t st);
int64_t argmax_ws_bytes(int64_t rows);

int launch_rope_shift(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                      const int32_t* src_row, const int32_t* dst_row, const int32_t* delta,
                      int64_t n_tok, int Hkv, int D, const RopeFreq& f, int dtype, hipStream_t st);

// The same for n_jobs independent jobs (device table) in one launch; max_n_tok bounds every job's n_tok.
int launch_rope_shift_jobs(const vlc_shift_job* jobs, int n_jobs, int64_t max_n_tok, int Hkv, int D,
                           const RopeFreq& f, int dtype, hipStream_t st);

// Strided scatter of K/V rows: cache[dst_row[i]] = src[i * src_stride_elems ...]
int launch_scatter_kv(const void* k_new, const void* v_new, int64_t src_stride_elems,
                      const int32_t* dst_row, int64_t n, void* k_cache, void* v_cache, int Hkv, int D,
                      int dtype, hipStream_t st);

// From the unrounded float rows qkv32 [n, (Hq+2Hkv)*D]: q rotated at pos[i] -> q_out [n, Hq*D];
// k rotated -> k_cache[slot[i]]; v -> v_cache[slot[i]].  Outputs have the storage type `dtype`
// and are rounded once, after the rotation.
// splits > 1 (bf16 path): the projection is still `splits` float partial matrices [splits][n][(Hq+2Hkv)D]
// at `partials`; they are summed in split order, the bias (may be NULL) added, and the sum is
// also written to qkv32.  Otherwise qkv32 is the finished projection and is only read.
// pos3 (optional, [n, 3]): per-axis position ids, selected per frequency by f.axis; else pos [n].
// w_qnorm / w_knorm (optional, [D]): RMSNorm over each q / k head (eps) before the rotation.
int launch_rope_qk_scatter(const float* qkv32, const int32_t* pos, const int32_t* slot, int64_t n, int Hq,
                           int Hkv, int D, const RopeFreq& f, void* q_out, void* k_cache, void* v_cache,
                           int dtype, hipStream_t st, const float* partials = nullptr, int splits = 1,
                           const void* bias = nullptr, const int32_t* pos3 = nullptr,
                           const void* w_qnorm = nullptr, const void* w_knorm = nullptr, float eps = 0.f);

// q rows have a row stride of q_stride elements (dense q: Hq*D).  ws: optional float scratch of
// attention_ws_bytes() that allows splitting the key range when there are few query rows.
int launch_attention(const void* q, int64_t q_stride, const void* k_cache, const void* v_cache,
                     const int32_t* row_kv_start, const int32_t* row_kv_len, int64_t n, int Hq, int Hkv,
                     int D, float scale, void* out, int dtype, void* ws, int64_t ws_bytes, int64_t max_kv_len,
                     hipStream_t st);   // max_kv_len: upper bound of row_kv_len if known, else 0
int64_t attention_ws_bytes(int64_t n, int Hq, int Hkv, int D, int dtype);

enum Epilogue {
  EPI_BIAS = 0,      // C = A W^T + bias[n]               (bias may be NULL)
  EPI_RESIDUAL = 1,  // C = A W^T + resid[rmap ? rmap[m] : m, n]
  EPI_SWIGLU = 2,    // W = [gate(I rows); up(I rows)], C[m, j] = silu(A Wg^T)[m,j] * (A Wu^T)[m,j], N = I
  EPI_BIAS_F32 = 3   // as EPI_BIAS but C is a float matrix whatever the input type (no rounding)
};
// C[M,N] = epilogue(A[M,K] (row stride lda) * W[N(or 2N),K]^T); C row stride ldc.
// splitk_ws: optional float scratch for split-K partials (used when the output has few tiles);
// gemm_splitk_ws_bytes gives a size that lets every GEMM of a layer with n rows split freely.
// deferred (optional): if the k range was split, the epilogue kernel is NOT run, *deferred is the
// number of float partial matrices [splits][M][N] left at splitk_ws and the caller's next kernel
// must sum them and apply the epilogue; *deferred = 0 means C is complete.
int launch_gemm(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                int64_t K, int epilogue, const void* bias, const void* resid, int64_t ldr,
                const int32_t* rmap, int dtype, void* splitk_ws, int64_t splitk_ws_bytes, hipStream_t st,
                int* deferred = nullptr);
int64_t gemm_splitk_ws_bytes(int64_t n_rows, int64_t max_n);

// Grouped GEMM (mixture-of-experts): C[m, :] = epilogue(A[amap ? amap[m] : m, :] * W[g]^T) for the rows m
// of group g; the rows of a group are contiguous in C.  `tiles` (device) lists (group, first row, end row)
// with at most tile_rows rows each, *n_tiles (device) says how many entries count; both are written by
// launch_moe_plan.  rows: total number of rows over all groups; a_rows: rows of A (bound of the amap values, or
// = rows without a map); w_stride: elements between two groups' matrices.  Epilogues: EPI_BIAS without a bias (plain product) and EPI_SWIGLU.
struct GroupTile {
  int32_t expert, m0, m_end, pad;
};
int gemm_group_tile_rows(int64_t rows, int n_groups, int dtype);
int launch_gemm_grouped(const void* A, int64_t lda, const int32_t* amap, const void* W, int64_t w_stride, void* C,
                        int64_t ldc, int64_t rows, int n_groups, int64_t N, int64_t K, int epilogue,
                        const GroupTile* tiles, const int32_t* n_tiles, int tile_rows, int dtype, hipStream_t st,
                        int64_t a_rows);

// Mixture-of-experts routing.  All pointers device.  launch_moe_route: from router scores [n, E] (float)
// writes the chosen experts idx [n, K], weights wts [n, K], the grouped order (offset [E + 1]: first pair
// of every expert; pair_pos [n, K]: position of a pair; pair_row [n * K]: row of the pair at a position)
// and the tile table of the grouped GEMMs (tiles [n * K / tile_rows + E], n_tiles [1]).  rank [n, K] and
// count [E] are scratch.  launch_moe_combine: out[r] = h1[r] + sum_k wts[r, k] * y[pair_pos[r, k]].
struct MoeScratch {
  int32_t* idx;
  float* wts;
  int32_t* rank;
  int32_t* count;
  int32_t* offset;
  GroupTile* tiles;
  int32_t* n_tiles;
  int32_t* pair_row;
  int32_t* pair_pos;
};
// logits: `splits` partial matrices [n, E] to sum, split_stride floats apart; sum_out (optional): where the summed
// scores are left
int launch_moe_route(const float* logits, int splits, int64_t split_stride, float* sum_out, int64_t n,
                     int n_experts, int top_k, int tile_rows, const MoeScratch& s, hipStream_t st);
int launch_moe_combine(const void* h1, const void* y, const float* wts, const int32_t* pair_pos, int64_t n,
                       int top_k, int H, void* out, int dtype, hipStream_t st);
// launch_moe_combine, then normed[ymap ? ymap[i] : i] = RMSNorm(out[i]) * norm_w in the same kernel
// (rows with ymap[i] < 0 get no norm); the same bits as launch_moe_combine + launch_rmsnorm
int launch_moe_combine_norm(const void* h1, const void* y, const float* wts, const int32_t* pair_pos, int64_t n,
                            int top_k, int H, void* out, const void* norm_w, void* normed, const int32_t* ymap,
                            float eps, int dtype, hipStream_t st);

}  // namespace vlc
#endif
