// Mixture-of-experts MLP (the Qwen3-VL-30B-A3B-shaped layer of the paper's evaluation, Sec. 5.1):
// expert choice per recomputed row, grouping of the (row, expert) pairs by expert for the grouped
// GEMMs, and the weighted sum of the experts' outputs with the residual.
//
//   route   : per row, the top_k largest router scores (equal scores: lower expert index first),
//             weights exp(z_k - z_max) / sum over the chosen ones (the softmax denominator over
//             all experts cancels in the renormalised weights); each pair takes a rank inside its
//             expert from an atomic counter (the order inside an expert does not change any result:
//             every pair is computed on its own)
//   plan    : exclusive scan of the expert counts -> first pair of every expert, and the table of
//             row tiles (expert, first row, end row) the grouped GEMMs walk
//   fill    : pair position = first pair of its expert + rank; the inverse list position -> row
//   combine : h_out[row] = h1[row] + sum_k w[row, k] * y[position(row, k)]   (float sum, one rounding)
#include <hip/hip_runtime.h>

#include <cfloat>
#include <climits>

#include "vlc_internal.h"

namespace vlc {
namespace {

constexpr int kMaxExperts = 256;   // four scores per lane
constexpr int kMaxTopK = 16;
constexpr int64_t kSmallPlanPairs = 65536;   // up to here one workgroup groups the pairs

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

__device__ __forceinline__ void better(float& bv, int& be, float v, int e) {
  if (v > bv || (v == bv && e < be)) {
    bv = v;
    be = e;
  }
}

// one wavefront per row
// logits: `splits` float partial matrices [n, E] (split_stride floats apart) whose sum are the scores
// (1: the scores themselves).  count == NULL: no ranks are taken (the single-workgroup plan does that).
__global__ __launch_bounds__(256) void moe_route_kernel(const float* __restrict__ logits, int splits,
                                                        int64_t split_stride, float* __restrict__ sum_out,
                                                        int64_t n, int E, int K,
                                                        int32_t* __restrict__ idx, float* __restrict__ wts,
                                                        int32_t* __restrict__ rank, int32_t* __restrict__ count) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= n) return;
  float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    float z = -INFINITY;
    if (e < E) {
      z = logits[row * E + e];
      for (int s = 1; s < splits; ++s) z += logits[s * split_stride + row * E + e];   // in split order
      if (sum_out) sum_out[row * E + e] = z;             // the scores the choice is taken from, for inspection
    }
    if (e < E && !(z >= -FLT_MAX)) z = -FLT_MAX;        // NaN or -inf scores rank last but stay selectable
    v[j] = z;
  }
  float my_v = 0.f, top_v = 0.f;
  int my_e = 0;
  for (int k = 0; k < K; ++k) {
    float bv = -INFINITY;
    int be = INT_MAX;
#pragma unroll
    for (int j = 0; j < 4; ++j) better(bv, be, v[j], lane + 64 * j);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) better(bv, be, __shfl_xor(bv, o), __shfl_xor(be, o));
    if (k == 0) top_v = bv;
    if (lane == k) {
      my_v = bv;
      my_e = be;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (lane + 64 * j == be) v[j] = -INFINITY;         // taken
  }
  float ex = lane < K ? expf(my_v - top_v) : 0.f;
  float sum = ex;
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o);   // K <= 16: lanes 0..15
  if (lane < K) {
    const int e = my_e < E ? my_e : E - 1;
    idx[row * K + lane] = e;
    wts[row * K + lane] = ex / sum;
    if (count) rank[row * K + lane] = atomicAdd(&count[e], 1);
  }
}

// Few pairs: counting, scan, tile table, positions and the inverse list in ONE workgroup (LDS atomics),
// instead of the zero / plan / fill kernels around the counting in moe_route_kernel.
__global__ __launch_bounds__(1024) void moe_plan_small_kernel(const int32_t* __restrict__ idx, int64_t pairs, int K,
                                                              int E, int tile_rows, int32_t* __restrict__ offset,
                                                              GroupTile* __restrict__ tiles,
                                                              int32_t* __restrict__ n_tiles,
                                                              int32_t* __restrict__ pair_row,
                                                              int32_t* __restrict__ pair_pos) {
  __shared__ int cnt[256], sc[256], stl[256], cur[256];
  const int t = threadIdx.x;
  if (t < 256) cnt[t] = 0;
  __syncthreads();
  for (int64_t i = t; i < pairs; i += 1024) atomicAdd(&cnt[idx[i]], 1);
  __syncthreads();
  const int c = t < 256 ? cnt[t] : 0;
  const int nt = (c + tile_rows - 1) / tile_rows;
  if (t < 256) {
    sc[t] = c;
    stl[t] = nt;
  }
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {      // inclusive scans over the 256 expert slots
    int a = 0, b = 0;
    if (t < 256 && t >= o) {
      a = sc[t - o];
      b = stl[t - o];
    }
    __syncthreads();
    if (t < 256) {
      sc[t] += a;
      stl[t] += b;
    }
    __syncthreads();
  }
  if (t < 256) {
    const int off = sc[t] - c, toff = stl[t] - nt;
    cur[t] = off;
    if (t < E) {
      offset[t] = off;
      for (int k = 0; k < nt; ++k) {
        GroupTile g;
        g.expert = t;
        g.m0 = off + k * tile_rows;
        g.m_end = off + c;
        g.pad = 0;
        tiles[toff + k] = g;
      }
    }
    if (t == 255) {
      offset[E] = sc[255];
      *n_tiles = stl[255];
    }
  }
  __syncthreads();
  for (int64_t i = t; i < pairs; i += 1024) {
    const int pos = atomicAdd(&cur[idx[i]], 1);
    pair_pos[i] = pos;
    pair_row[pos] = (int32_t)(i / K);
  }
}

// one workgroup of 256 threads, thread e owns expert e
__global__ __launch_bounds__(256) void moe_plan_kernel(const int32_t* __restrict__ count, int E, int tile_rows,
                                                       int32_t* __restrict__ offset, GroupTile* __restrict__ tiles,
                                                       int32_t* __restrict__ n_tiles) {
  __shared__ int sc[256], stl[256];
  const int e = threadIdx.x;
  const int cnt = e < E ? count[e] : 0;
  const int nt = (cnt + tile_rows - 1) / tile_rows;
  sc[e] = cnt;
  stl[e] = nt;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {      // inclusive scans
    const int a = e >= o ? sc[e - o] : 0, b = e >= o ? stl[e - o] : 0;
    __syncthreads();
    sc[e] += a;
    stl[e] += b;
    __syncthreads();
  }
  const int off = sc[e] - cnt, toff = stl[e] - nt;
  if (e < E) {
    offset[e] = off;
    for (int t = 0; t < nt; ++t) {
      GroupTile g;
      g.expert = e;
      g.m0 = off + t * tile_rows;
      g.m_end = off + cnt;
      g.pad = 0;
      tiles[toff + t] = g;
    }
  }
  if (e == 255) {
    offset[E] = sc[255];
    *n_tiles = stl[255];
  }
}

__global__ __launch_bounds__(256) void moe_fill_kernel(const int32_t* __restrict__ idx, const int32_t* __restrict__ rank,
                                                       const int32_t* __restrict__ offset, int64_t pairs, int K,
                                                       int32_t* __restrict__ pair_row, int32_t* __restrict__ pair_pos) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= pairs) return;
  const int pos = offset[idx[i]] + rank[i];
  pair_pos[i] = pos;
  pair_row[pos] = (int32_t)(i / K);
}

__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const uint16_t* p) { return __uint_as_float(((uint32_t)*p) << 16); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(uint16_t* p, float v) {
  uint32_t u = __float_as_uint(v);
  u += 0x7fffu + ((u >> 16) & 1u);
  *p = (uint16_t)(u >> 16);
}

// one workgroup per row; a thread owns 16-byte chunks of the row
template <typename T>
__global__ __launch_bounds__(256) void moe_combine_kernel(const T* __restrict__ h1, const T* __restrict__ y,
                                                          const float* __restrict__ wts,
                                                          const int32_t* __restrict__ pair_pos, int K, int H,
                                                          T* __restrict__ out) {
  constexpr int VEC = 16 / sizeof(T);
  const int64_t row = blockIdx.x;
  __shared__ float w[kMaxTopK];
  __shared__ int pos[kMaxTopK];
  if (threadIdx.x < K) {
    w[threadIdx.x] = wts[row * K + threadIdx.x];
    pos[threadIdx.x] = pair_pos[row * K + threadIdx.x];
  }
  __syncthreads();
  for (int c = threadIdx.x * VEC; c < H; c += 256 * VEC) {
    float acc[VEC];
    uint4 raw = *reinterpret_cast<const uint4*>(h1 + row * H + c);
    const T* hp = reinterpret_cast<const T*>(&raw);
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    for (int k = 0; k < K; ++k) {
      const uint4 yr = *reinterpret_cast<const uint4*>(y + (int64_t)pos[k] * H + c);
      const T* yp = reinterpret_cast<const T*>(&yr);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w[k], ld_elem(yp + i), acc[i]);
    }
    uint4 o;
    T* op = reinterpret_cast<T*>(&o);
#pragma unroll
    for (int i = 0; i < VEC; ++i) st_elem(op + i, ld_elem(hp + i) + acc[i]);
    *reinterpret_cast<uint4*>(out + row * H + c) = o;
  }
}

// moe_combine_kernel followed by the RMSNorm of the row it has just written (the input norm of the layer below,
// weight nw): thread t owns chunks t, t + 256, ... as the stand-alone norm kernel does, and the sums are taken
// in the same order on the stored (rounded) values, so both routes give the same bits.  The normed row goes to
// yn[ymap ? ymap[row] : row]; a negative entry: no norm for this row.
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void moe_combine_norm_kernel(const T* __restrict__ h1, const T* __restrict__ y,
                                                               const float* __restrict__ wts,
                                                               const int32_t* __restrict__ pair_pos, int K, int H,
                                                               T* __restrict__ out, const T* __restrict__ nw,
                                                               T* __restrict__ yn, const int32_t* __restrict__ ymap,
                                                               float inv_h, float eps) {
  constexpr int VEC = 16 / sizeof(T);
  const int64_t row = blockIdx.x;
  __shared__ float w[kMaxTopK];
  __shared__ int pos[kMaxTopK];
  __shared__ float red[4];
  if (threadIdx.x < K) {
    w[threadIdx.x] = wts[row * K + threadIdx.x];
    pos[threadIdx.x] = pair_pos[row * K + threadIdx.x];
  }
  __syncthreads();
  float v[MAXC][VEC];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = (threadIdx.x + j * 256) * VEC;
    if (c < H) {
      float acc[VEC];
      uint4 raw = *reinterpret_cast<const uint4*>(h1 + row * H + c);
      const T* hp = reinterpret_cast<const T*>(&raw);
#pragma unroll
      for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
      for (int k = 0; k < K; ++k) {
        const uint4 yr = *reinterpret_cast<const uint4*>(y + (int64_t)pos[k] * H + c);
        const T* yp = reinterpret_cast<const T*>(&yr);
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = fmaf(w[k], ld_elem(yp + i), acc[i]);
      }
      uint4 o;
      T* op = reinterpret_cast<T*>(&o);
#pragma unroll
      for (int i = 0; i < VEC; ++i) st_elem(op + i, ld_elem(hp + i) + acc[i]);
      *reinterpret_cast<uint4*>(out + row * H + c) = o;
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        v[j][i] = ld_elem(op + i);
        ss += v[j][i] * v[j][i];
      }
    }
  }
  const int64_t yrow = ymap ? (int64_t)ymap[row] : row;
  if (yrow < 0) return;                    // the same for the whole workgroup
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) tot += red[i];
  const float r = 1.0f / sqrtf(tot * inv_h + eps);
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = (threadIdx.x + j * 256) * VEC;
    if (c < H) {
      const uint4 wr = *reinterpret_cast<const uint4*>(nw + c);
      const T* wp = reinterpret_cast<const T*>(&wr);
      uint4 o;
      T* op = reinterpret_cast<T*>(&o);
#pragma unroll
      for (int i = 0; i < VEC; ++i) st_elem(op + i, v[j][i] * r * ld_elem(wp + i));
      *reinterpret_cast<uint4*>(yn + yrow * H + c) = o;
    }
  }
}

}  // namespace

int launch_moe_route(const float* logits, int splits, int64_t split_stride, float* sum_out, int64_t n,
                     int n_experts, int top_k, int tile_rows, const MoeScratch& s, hipStream_t st) {
  if (n <= 0) return VLC_OK;
  if (splits < 1) return fail(VLC_ERR_SHAPE, "moe: splits=%d", splits);
  if (n_experts < 1 || n_experts > kMaxExperts || top_k < 1 || top_k > kMaxTopK || top_k > n_experts)
    return fail(VLC_ERR_SHAPE, "moe: n_experts=%d (<= %d), top_k=%d (<= %d, <= n_experts)", n_experts, kMaxExperts,
                top_k, kMaxTopK);
  if (n * top_k > INT32_MAX) return fail(VLC_ERR_SHAPE, "moe: too many (row, expert) pairs");
  const int64_t pairs = n * top_k;
  if (pairs <= kSmallPlanPairs) {
    hipLaunchKernelGGL(moe_route_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, logits, splits,
                       split_stride, sum_out, n, n_experts, top_k, s.idx, s.wts, (int32_t*)nullptr,
                       (int32_t*)nullptr);
    VLC_CHECK_LAUNCH("moe_route");
    hipLaunchKernelGGL(moe_plan_small_kernel, dim3(1), dim3(1024), 0, st, (const int32_t*)s.idx, pairs, top_k,
                       n_experts, tile_rows, s.offset, s.tiles, s.n_tiles, s.pair_row, s.pair_pos);
    VLC_CHECK_LAUNCH("moe_plan_small");
    return VLC_OK;
  }
  hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(256), 0, st, s.count, n_experts);
  VLC_CHECK_LAUNCH("moe_zero");
  hipLaunchKernelGGL(moe_route_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, logits, splits, split_stride,
                     sum_out, n, n_experts, top_k, s.idx, s.wts, s.rank, s.count);
  VLC_CHECK_LAUNCH("moe_route");
  hipLaunchKernelGGL(moe_plan_kernel, dim3(1), dim3(256), 0, st, (const int32_t*)s.count, n_experts, tile_rows,
                     s.offset, s.tiles, s.n_tiles);
  VLC_CHECK_LAUNCH("moe_plan");
  hipLaunchKernelGGL(moe_fill_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st,
                     (const int32_t*)s.idx, (const int32_t*)s.rank, (const int32_t*)s.offset, pairs, top_k,
                     s.pair_row, s.pair_pos);
  VLC_CHECK_LAUNCH("moe_fill");
  return VLC_OK;
}

int launch_moe_combine(const void* h1, const void* y, const float* wts, const int32_t* pair_pos, int64_t n,
                       int top_k, int H, void* out, int dtype, hipStream_t st) {
  if (n <= 0) return VLC_OK;
  if (top_k < 1 || top_k > kMaxTopK) return fail(VLC_ERR_SHAPE, "moe combine: top_k=%d", top_k);
  if (dtype == VLC_BF16) {
    if (H % 8) return fail(VLC_ERR_SHAPE, "moe combine: H=%d must be a multiple of 8", H);
    hipLaunchKernelGGL(moe_combine_kernel<uint16_t>, dim3((unsigned)n), dim3(256), 0, st, (const uint16_t*)h1,
                       (const uint16_t*)y, wts, pair_pos, top_k, H, (uint16_t*)out);
  } else if (dtype == VLC_F32) {
    if (H % 4) return fail(VLC_ERR_SHAPE, "moe combine: H=%d must be a multiple of 4", H);
    hipLaunchKernelGGL(moe_combine_kernel<float>, dim3((unsigned)n), dim3(256), 0, st, (const float*)h1,
                       (const float*)y, wts, pair_pos, top_k, H, (float*)out);
  } else {
    return fail(VLC_ERR_DTYPE, "moe combine: dtype=%d", dtype);
  }
  VLC_CHECK_LAUNCH("moe_combine");
  return VLC_OK;
}

int launch_moe_combine_norm(const void* h1, const void* y, const float* wts, const int32_t* pair_pos, int64_t n,
                            int top_k, int H, void* out, const void* norm_w, void* normed, const int32_t* ymap,
                            float eps, int dtype, hipStream_t st) {
  if (n <= 0) return VLC_OK;
  if (top_k < 1 || top_k > kMaxTopK) return fail(VLC_ERR_SHAPE, "moe combine: top_k=%d", top_k);
  if (dtype != VLC_BF16 && dtype != VLC_F32) return fail(VLC_ERR_DTYPE, "moe combine: dtype=%d", dtype);
  const int vec = dtype == VLC_BF16 ? 8 : 4;
  if (H % vec) return fail(VLC_ERR_SHAPE, "moe combine: H=%d must be a multiple of %d", H, vec);
  const int chunks = H / vec;
  const float inv_h = 1.0f / (float)H;
#define VLC_LAUNCH_MCN(T, MAXC)                                                                              \
  hipLaunchKernelGGL((moe_combine_norm_kernel<T, MAXC>), dim3((unsigned)n), dim3(256), 0, st, (const T*)h1,  \
                     (const T*)y, wts, pair_pos, top_k, H, (T*)out, (const T*)norm_w, (T*)normed, ymap, inv_h, eps)
  if (chunks <= 256 * 2) {
    if (dtype == VLC_BF16) VLC_LAUNCH_MCN(uint16_t, 2); else VLC_LAUNCH_MCN(float, 2);
  } else if (chunks <= 256 * 8) {
    if (dtype == VLC_BF16) VLC_LAUNCH_MCN(uint16_t, 8); else VLC_LAUNCH_MCN(float, 8);
  } else {   // very wide rows: the two kernels one after the other
    const int rc = launch_moe_combine(h1, y, wts, pair_pos, n, top_k, H, out, dtype, st);
    return rc ? rc : launch_rmsnorm(out, nullptr, norm_w, normed, n, H, eps, dtype, st, ymap);
  }
#undef VLC_LAUNCH_MCN
  VLC_CHECK_LAUNCH("moe_combine_norm");
  return VLC_OK;
}

}  // namespace vlc
