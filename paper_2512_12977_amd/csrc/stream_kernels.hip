// HBM-bound kernels of the selective-recompute path: row gather, KV scatter, key re-rotation
// (RoPE shift), RoPE + scatter of fresh q/k/v rows, RMSNorm.  All move 16-byte chunks per lane
// so that a wavefront touches whole 128-byte lines of each row.
#include <hip/hip_runtime.h>

#include "vlc_internal.h"

namespace vlc {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {   // round to nearest, ties to even
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// A 16-byte chunk viewed as VEC elements of T, converted to/from float.
__device__ __forceinline__ float elem_to_float(float v) { return v; }
__device__ __forceinline__ float elem_to_float(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }   // bf16

template <typename T> struct Chunk;
template <> struct Chunk<float> {
  static constexpr int VEC = 4;
  __device__ static void unpack(const uint4& r, float* f) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
    f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  }
  __device__ static uint4 pack(const float* f) {
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                      __float_as_uint(f[3]));
  }
};
template <> struct Chunk<uint16_t> {   // bf16
  static constexpr int VEC = 8;
  __device__ static void unpack(const uint4& r, float* f) {
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static uint4 pack(const float* f) {
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
  }
};

// sin/cos of delta * inv_freq.  The angle is formed and reduced to [-pi, pi] in double (positions
// reach tens of thousands of radians, beyond what a float angle resolves), then evaluated in float.
// FAST (bf16 storage, 8 significant bits): the hardware sine/cosine, which take the angle in
// revolutions; otherwise the library routines on the reduced angle.
template <bool FAST>
__device__ __forceinline__ void rope_sincos(double inv_freq, int delta, float* s, float* c) {
  double rev = (double)delta * inv_freq * 0.15915494309189535;   // angle / 2pi
  rev -= rint(rev);
  if (FAST) {
    *s = __builtin_amdgcn_sinf((float)rev);
    *c = __builtin_amdgcn_cosf((float)rev);
  } else {
    const float r = (float)(rev * 6.283185307179586);
    *s = sinf(r);
    *c = cosf(r);
  }
}

// ---------------------------------------------------------------------------------------------
// gather / scatter of whole rows in 16-byte chunks
// ---------------------------------------------------------------------------------------------
// dst chunk (i, c) = src chunk (src_idx ? src_idx[i] : i, c) written at row (dst_idx ? dst_idx[i] : i).
// Row strides are given in chunks.  Plain cached accesses (non-temporal ones measured half the rate
// here).  blockIdx.y selects one of up to two
// (src, dst) pairs that share the index arrays (K and V of a scatter go in one launch).
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kCopyThreads = 256;

// One 16-byte chunk per thread.  (Several chunks per thread are slower: a 1 GiB copy runs at 5.8 TB/s with four,
// at 6.35 TB/s with one, at half that with eight - short-lived threads keep more loads in flight.)
__global__ __launch_bounds__(kCopyThreads) void copy_rows_kernel(const u32x4* __restrict__ src0,
                                                                 const u32x4* __restrict__ src1,
                                                                 u32x4* __restrict__ dst0, u32x4* __restrict__ dst1,
                                                                 int64_t src_stride,
                                                                 const int32_t* __restrict__ src_idx,
                                                                 int64_t dst_stride,
                                                                 const int32_t* __restrict__ dst_idx, uint32_t total,
                                                                 uint32_t chunks_per_row) {
  const u32x4* __restrict__ src = blockIdx.y ? src1 : src0;
  u32x4* __restrict__ dst = blockIdx.y ? dst1 : dst0;
  const uint32_t id = blockIdx.x * (uint32_t)kCopyThreads + threadIdx.x;
  if (id >= total) return;
  const uint32_t row = id / chunks_per_row;
  const uint32_t c = id - row * chunks_per_row;
  const int64_t srow = src_idx ? (int64_t)src_idx[row] : (int64_t)row;
  const int64_t drow = dst_idx ? (int64_t)dst_idx[row] : (int64_t)row;
  dst[drow * dst_stride + c] = src[srow * src_stride + c];
}

// One or two row copies (same row count, strides and index arrays) in a single launch.
int copy_rows(const void* src0, const void* src1, int64_t src_stride_bytes, const int32_t* src_idx, void* dst0,
              void* dst1, int64_t dst_stride_bytes, const int32_t* dst_idx, int64_t n, int64_t row_bytes,
              hipStream_t st, const char* name) {
  const int64_t cpr = row_bytes / 16;
  if (n <= 0 || cpr <= 0) return VLC_OK;
  // keep flat chunk ids within 31 bits: slice the row range if needed
  const int64_t rows_per_launch = ((int64_t)1 << 30) / cpr > 0 ? ((int64_t)1 << 30) / cpr : 1;
  for (int64_t r0 = 0; r0 < n; r0 += rows_per_launch) {
    const int64_t rows = (n - r0 < rows_per_launch) ? n - r0 : rows_per_launch;
    const uint32_t total = (uint32_t)(rows * cpr);
    const uint32_t blocks = (total + kCopyThreads - 1) / kCopyThreads;
    const int64_t so = src_idx ? 0 : r0 * src_stride_bytes, dof = dst_idx ? 0 : r0 * dst_stride_bytes;
    const u32x4* s0 = reinterpret_cast<const u32x4*>(static_cast<const char*>(src0) + so);
    u32x4* d0 = reinterpret_cast<u32x4*>(static_cast<char*>(dst0) + dof);
    const u32x4* s1 = src1 ? reinterpret_cast<const u32x4*>(static_cast<const char*>(src1) + so) : nullptr;
    u32x4* d1 = dst1 ? reinterpret_cast<u32x4*>(static_cast<char*>(dst1) + dof) : nullptr;
    hipLaunchKernelGGL(copy_rows_kernel, dim3(blocks, src1 ? 2 : 1), dim3(kCopyThreads), 0, st, s0, s1, d0, d1,
                       src_stride_bytes / 16, src_idx ? src_idx + r0 : nullptr, dst_stride_bytes / 16,
                       dst_idx ? dst_idx + r0 : nullptr, total, (uint32_t)cpr);
    VLC_CHECK_LAUNCH(name);
  }
  return VLC_OK;
}

// ---------------------------------------------------------------------------------------------
// RoPE shift of reused keys + copy of reused values (Sec. 4.2)
// ---------------------------------------------------------------------------------------------
// One thread owns VEC rotation pairs of one head of one token: a 16-byte chunk of the low half and the matching
// chunk of the high half of the key, and the same two chunks of the value.  Consecutive lanes cover consecutive
// chunks, then the heads of a token, then tokens, so a wavefront touches whole 128-byte lines.  (Threads that walk
// over all heads of a token, to compute each sine/cosine once, are 3-5 % slower: the kernel is bound by memory
// parallelism, and four short-lived threads keep more loads in flight than one long one.)
template <typename T, int D>
__device__ __forceinline__ void rope_shift_thread(
    int64_t gid, const uint4* k_src, const uint4* v_src, uint4* k_dst, uint4* v_dst,   // may alias (in-place use)
    const int32_t* __restrict__ src_row, const int32_t* __restrict__ dst_row,
    const int32_t* __restrict__ delta, int64_t n_tok, int Hkv, const RopeFreq& freq) {
  constexpr int VEC = Chunk<T>::VEC;
  constexpr int CH = (D / 2) / VEC;                  // chunks per half head
  constexpr int HEAD_CHUNKS = 2 * CH;                // chunks per head
  const int64_t t = gid / CH;
  const int c = (int)(gid - t * CH);
  const int64_t tok = t / Hkv;
  const int h = (int)(t - tok * Hkv);
  if (tok >= n_tok) return;
  const int64_t srow = src_row[tok], drow = dst_row[tok];
  const int d = delta[tok];
  const int64_t row_chunks = (int64_t)Hkv * HEAD_CHUNKS;
  const int64_t so = srow * row_chunks + h * HEAD_CHUNKS + c, dof = drow * row_chunks + h * HEAD_CHUNKS + c;
  const bool do_v = v_src != nullptr && v_dst != nullptr;
  const uint4 lo_r = k_src[so];
  const uint4 hi_r = k_src[so + CH];
  uint4 v_lo, v_hi;
  if (do_v) {
    v_lo = v_src[so];
    v_hi = v_src[so + CH];
  }
  float sn[VEC], cs[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) rope_sincos<sizeof(T) == 2>(freq.inv_freq[c * VEC + i], d, &sn[i], &cs[i]);
  float lo[VEC], hi[VEC], olo[VEC], ohi[VEC];
  Chunk<T>::unpack(lo_r, lo);
  Chunk<T>::unpack(hi_r, hi);
#pragma unroll
  for (int i = 0; i < VEC; ++i) {
    olo[i] = lo[i] * cs[i] - hi[i] * sn[i];
    ohi[i] = hi[i] * cs[i] + lo[i] * sn[i];
  }
  k_dst[dof] = Chunk<T>::pack(olo);
  k_dst[dof + CH] = Chunk<T>::pack(ohi);
  if (do_v) {
    v_dst[dof] = v_lo;
    v_dst[dof + CH] = v_hi;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void rope_shift_kernel(
    const uint4* k_src, const uint4* v_src, uint4* k_dst, uint4* v_dst,
    const int32_t* __restrict__ src_row, const int32_t* __restrict__ dst_row,
    const int32_t* __restrict__ delta, int64_t n_tok, int Hkv, RopeFreq freq) {
  rope_shift_thread<T, D>((int64_t)blockIdx.x * kThreads + threadIdx.x, k_src, v_src, k_dst, v_dst, src_row, dst_row,
                          delta, n_tok, Hkv, freq);
}

// The same for a table of jobs (one per layer): blockIdx.y picks the job, blocks beyond its token count leave.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void rope_shift_jobs_kernel(const vlc_shift_job* __restrict__ jobs, int Hkv,
                                                                   RopeFreq freq) {
  const vlc_shift_job j = jobs[blockIdx.y];
  rope_shift_thread<T, D>((int64_t)blockIdx.x * kThreads + threadIdx.x, (const uint4*)j.k_src, (const uint4*)j.v_src,
                          (uint4*)j.k_dst, (uint4*)j.v_dst, j.src_row, j.dst_row, j.delta, j.n_tok, Hkv, freq);
}

constexpr int kMaxSplits = 8;   // the GEMM never splits the k range into more parts

// One thread owns VEC rotation pairs of one head of one row of the fused q|k|v matrix (unrounded float; several
// heads per thread, to reuse each sine/cosine, measured 9 % slower at 18944 rows: memory parallelism counts, the
// arithmetic does not).  Head index < Hq: query, rotated, written to q_out.  < Hq+Hkv: key,
// rotated and written to its cache slot (the blend).  Otherwise: value, written to its cache slot.
// Outputs are rounded to the storage type once, after the rotation.
// SUM: the projection was left as `splits` float partial matrices (split_stride elements apart,
// split-K); they are added here in split order, then the bias, and the sum is also stored to
// qkv_sum so the unrounded projection stays available to the caller.
// pos3 (optional): per-axis position ids [n, 3]; frequency i then takes the id of axis freq.axis[i].
// w_qn / w_kn (optional, [D]): RMSNorm over every q / k head before the rotation (a head's D values
// are spread over CH consecutive lanes, which exchange their partial sums of squares).
template <typename T, int D, bool SUM>
__global__ __launch_bounds__(kThreads) void rope_qk_scatter_kernel(
    const float* __restrict__ qkv, int splits, int64_t split_stride, const uint16_t* __restrict__ bias,
    float* __restrict__ qkv_sum, const int32_t* __restrict__ pos, const int32_t* __restrict__ pos3,
    const T* __restrict__ w_qn, const T* __restrict__ w_kn, float eps, const int32_t* __restrict__ slot,
    int64_t n, int Hq, int Hkv, RopeFreq freq, uint4* __restrict__ q_out,
    uint4* __restrict__ k_cache, uint4* __restrict__ v_cache) {
  constexpr int VEC = Chunk<T>::VEC;
  constexpr int CH = (D / 2) / VEC;
  constexpr int HEAD_CHUNKS = 2 * CH;
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  const int c = (int)(gid % CH);
  const int64_t t = gid / CH;
  const int heads = Hq + 2 * Hkv;
  const int h = (int)(t % heads);
  const int64_t row = t / heads;
  if (row >= n) return;
  float sn[VEC], cs[VEC];
  if (pos3) {
    const int p3[3] = {pos3[3 * row], pos3[3 * row + 1], pos3[3 * row + 2]};
#pragma unroll
    for (int i = 0; i < VEC; ++i)
      rope_sincos<sizeof(T) == 2>(freq.inv_freq[c * VEC + i], p3[freq.axis[c * VEC + i]], &sn[i], &cs[i]);
  } else {
    const int p = pos[row];
#pragma unroll
    for (int i = 0; i < VEC; ++i) rope_sincos<sizeof(T) == 2>(freq.inv_freq[c * VEC + i], p, &sn[i], &cs[i]);
  }
  const float* r = qkv + row * ((int64_t)heads * D) + c * VEC;
  uint4* qo = q_out + row * ((int64_t)Hq * HEAD_CHUNKS) + c;
  const int row_slot = slot[row];
  const bool keep_kv = row_slot >= 0;      // a negative slot: the row is computed, its k and v are not stored
  const int64_t dst = (int64_t)(keep_kv ? row_slot : 0) * ((int64_t)Hkv * HEAD_CHUNKS) + c;
  {
    float lo[VEC], hi[VEC];
#pragma unroll
    for (int i = 0; i < VEC; i += 4) {
      float4 a = *reinterpret_cast<const float4*>(r + (int64_t)h * D + i);
      float4 b = *reinterpret_cast<const float4*>(r + (int64_t)h * D + D / 2 + i);
      if constexpr (SUM) {
        float4 pa[kMaxSplits], pb[kMaxSplits];   // independent loads first, then the sum in split order
#pragma unroll
        for (int k = 1; k < kMaxSplits; ++k)
          if (k < splits) {
            pa[k] = *reinterpret_cast<const float4*>(r + k * split_stride + (int64_t)h * D + i);
            pb[k] = *reinterpret_cast<const float4*>(r + k * split_stride + (int64_t)h * D + D / 2 + i);
          }
#pragma unroll
        for (int k = 1; k < kMaxSplits; ++k)
          if (k < splits) {
            a.x += pa[k].x; a.y += pa[k].y; a.z += pa[k].z; a.w += pa[k].w;
            b.x += pb[k].x; b.y += pb[k].y; b.z += pb[k].z; b.w += pb[k].w;
          }
        if (bias) {
          const uint2 ba = *reinterpret_cast<const uint2*>(bias + h * D + c * VEC + i);
          const uint2 bb = *reinterpret_cast<const uint2*>(bias + h * D + D / 2 + c * VEC + i);
          a.x += __uint_as_float(ba.x << 16); a.y += __uint_as_float(ba.x & 0xffff0000u);
          a.z += __uint_as_float(ba.y << 16); a.w += __uint_as_float(ba.y & 0xffff0000u);
          b.x += __uint_as_float(bb.x << 16); b.y += __uint_as_float(bb.x & 0xffff0000u);
          b.z += __uint_as_float(bb.y << 16); b.w += __uint_as_float(bb.y & 0xffff0000u);
        }
        float* so = qkv_sum + row * ((int64_t)heads * D) + c * VEC + (int64_t)h * D;
        *reinterpret_cast<float4*>(so + i) = a;
        *reinterpret_cast<float4*>(so + D / 2 + i) = b;
      }
      lo[i] = a.x; lo[i + 1] = a.y; lo[i + 2] = a.z; lo[i + 3] = a.w;
      hi[i] = b.x; hi[i + 1] = b.y; hi[i + 2] = b.z; hi[i + 3] = b.w;
    }
    if (h >= Hq + Hkv) {
      if (keep_kv) {
        v_cache[dst + (h - Hq - Hkv) * HEAD_CHUNKS] = Chunk<T>::pack(lo);
        v_cache[dst + (h - Hq - Hkv) * HEAD_CHUNKS + CH] = Chunk<T>::pack(hi);
      }
      return;
    }
    if (w_qn) {   // RMSNorm over the head, float; every lane of the head's CH-lane group is here
      float ss = 0.f;
#pragma unroll
      for (int i = 0; i < VEC; ++i) ss += lo[i] * lo[i] + hi[i] * hi[i];
#pragma unroll
      for (int o = 1; o < CH; o <<= 1) ss += __shfl_xor(ss, o);
      const float rn = 1.0f / sqrtf(ss * (1.0f / (float)D) + eps);
      const T* wn = (h < Hq ? w_qn : w_kn) + c * VEC;
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        lo[i] = lo[i] * rn * elem_to_float(wn[i]);
        hi[i] = hi[i] * rn * elem_to_float(wn[D / 2 + i]);
      }
    }
    float olo[VEC], ohi[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
      olo[i] = lo[i] * cs[i] - hi[i] * sn[i];
      ohi[i] = hi[i] * cs[i] + lo[i] * sn[i];
    }
    const uint4 plo = Chunk<T>::pack(olo), phi = Chunk<T>::pack(ohi);
    if (h < Hq) {
      qo[h * HEAD_CHUNKS] = plo;
      qo[h * HEAD_CHUNKS + CH] = phi;
    } else {
      if (keep_kv) {
        k_cache[dst + (h - Hq) * HEAD_CHUNKS] = plo;
        k_cache[dst + (h - Hq) * HEAD_CHUNKS + CH] = phi;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// RMSNorm with optional row gather: y[i] = x[map[i]] * rsqrt(mean(x^2) + eps) * w.  With a destination list
// the result of row i goes to y[ymap[i]], and a row whose entry is negative is skipped.
// ---------------------------------------------------------------------------------------------
template <typename T, int MAXC>
__global__ __launch_bounds__(kThreads) void rmsnorm_kernel(const uint4* __restrict__ x,
                                                           const int32_t* __restrict__ map,
                                                           const uint4* __restrict__ w,
                                                           uint4* __restrict__ y, int chunks, float inv_h,
                                                           float eps, const int32_t* __restrict__ ymap) {
  constexpr int VEC = Chunk<T>::VEC;
  const int64_t row = blockIdx.x;
  const int64_t yrow = ymap ? (int64_t)ymap[row] : row;
  if (yrow < 0) return;                    // the same for the whole workgroup
  const int64_t srow = map ? (int64_t)map[row] : row;
  const uint4* xr = x + srow * chunks;
  float v[MAXC][VEC];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    if (c < chunks) {
      Chunk<T>::unpack(xr[c], v[j]);
#pragma unroll
      for (int i = 0; i < VEC; ++i) ss += v[j][i] * v[j][i];
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < kThreads / 64; ++i) tot += part[i];
  const float r = 1.0f / sqrtf(tot * inv_h + eps);
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    if (c < chunks) {
      float wv[VEC], o[VEC];
      Chunk<T>::unpack(w[c], wv);
#pragma unroll
      for (int i = 0; i < VEC; ++i) o[i] = v[j][i] * r * wv[i];
      y[yrow * chunks + c] = Chunk<T>::pack(o);
    }
  }
}

// Split-K partial sums [splits][n][H] (float) of a projection + residual -> h (rounded to bf16 and
// stored), then RMSNorm of the rounded h -> y.  One workgroup per row; same summation order as the
// stand-alone split-K epilogue (partials in split order, then the residual).
template <int MAXC>
__global__ __launch_bounds__(kThreads) void sum_residual_rmsnorm_kernel(
    const float* __restrict__ part, int splits, int64_t split_stride, const uint4* __restrict__ resid,
    const int32_t* __restrict__ rmap, const uint4* __restrict__ w, uint4* __restrict__ h,
    uint4* __restrict__ y, int chunks, float inv_h, float eps, const int32_t* __restrict__ ymap) {
  using CB = Chunk<uint16_t>;
  const int64_t row = blockIdx.x;
  const int64_t rrow = rmap ? (int64_t)rmap[row] : row;
  const int64_t yrow = ymap ? (int64_t)ymap[row] : row;    // < 0: h is written, the norm is not wanted
  float v[MAXC][8];
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    if (c < chunks) {
      const float* p0 = part + row * ((int64_t)chunks * 8) + c * 8;
      float4 pa[kMaxSplits], pb[kMaxSplits];
#pragma unroll
      for (int k = 0; k < kMaxSplits; ++k)
        if (k < splits) {
          pa[k] = *reinterpret_cast<const float4*>(p0 + k * split_stride);
          pb[k] = *reinterpret_cast<const float4*>(p0 + k * split_stride + 4);
        }
      float rs[8];
      CB::unpack(resid[rrow * chunks + c], rs);
      float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
#pragma unroll
      for (int k = 0; k < kMaxSplits; ++k)
        if (k < splits) {
          a.x += pa[k].x; a.y += pa[k].y; a.z += pa[k].z; a.w += pa[k].w;
          b.x += pb[k].x; b.y += pb[k].y; b.z += pb[k].z; b.w += pb[k].w;
        }
      float o[8] = {a.x + rs[0], a.y + rs[1], a.z + rs[2], a.w + rs[3],
                    b.x + rs[4], b.y + rs[5], b.z + rs[6], b.w + rs[7]};
      const uint4 packed = CB::pack(o);
      h[row * chunks + c] = packed;
      CB::unpack(packed, v[j]);            // the norm sees the stored (rounded) values
#pragma unroll
      for (int i = 0; i < 8; ++i) ss += v[j][i] * v[j][i];
    }
  }
  if (yrow < 0) return;                    // the same for the whole workgroup
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o);
  __shared__ float red[kThreads / 64];
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < kThreads / 64; ++i) tot += red[i];
  const float r = 1.0f / sqrtf(tot * inv_h + eps);
#pragma unroll
  for (int j = 0; j < MAXC; ++j) {
    const int c = threadIdx.x + j * kThreads;
    if (c < chunks) {
      float wv[8], o[8];
      CB::unpack(w[c], wv);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] = v[j][i] * r * wv[i];
      y[yrow * chunks + c] = CB::pack(o);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Greedy choice: index of the largest score of a row, the lowest index among equal scores; NaNs
// never win.  Two passes: kArgmaxSlices workgroups per row each scan a slice of the columns (16
// bytes per lane) and leave their best (value, index); one workgroup per row then picks among those.
// ---------------------------------------------------------------------------------------------
constexpr int kArgmaxSlices = 64;

__device__ __forceinline__ void take_better(float v, int64_t c, float& best, int64_t& bi) {
  if (v > best || (v == best && c < bi)) { best = v; bi = c; }
}

// best of the whole workgroup in sv[0] / si[0]
__device__ __forceinline__ void block_best(float best, int64_t bi, float* sv, int64_t* si) {
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int o = kThreads / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) take_better(sv[threadIdx.x + o], si[threadIdx.x + o], sv[threadIdx.x], si[threadIdx.x]);
    __syncthreads();
  }
}

__global__ __launch_bounds__(kThreads) void argmax_slices_kernel(const float* __restrict__ x, int64_t cols,
                                                                 float* __restrict__ part_v,
                                                                 int64_t* __restrict__ part_i) {
  const int64_t row = blockIdx.y;
  const int64_t quads = cols / 4;                      // cols is a multiple of 4
  const int64_t per = (quads + kArgmaxSlices - 1) / kArgmaxSlices;
  const int64_t q0 = blockIdx.x * per, q1 = min(quads, q0 + per);
  const float4* r = reinterpret_cast<const float4*>(x + row * cols);
  float best = -INFINITY;
  int64_t bi = cols;                                   // "none yet": larger than every real index
  for (int64_t q = q0 + threadIdx.x; q < q1; q += kThreads) {
    const float4 v = r[q];
    take_better(v.x, 4 * q, best, bi);
    take_better(v.y, 4 * q + 1, best, bi);
    take_better(v.z, 4 * q + 2, best, bi);
    take_better(v.w, 4 * q + 3, best, bi);
  }
  __shared__ float sv[kThreads];
  __shared__ int64_t si[kThreads];
  block_best(best, bi, sv, si);
  if (threadIdx.x == 0) {
    part_v[row * kArgmaxSlices + blockIdx.x] = sv[0];
    part_i[row * kArgmaxSlices + blockIdx.x] = si[0];
  }
}

__global__ __launch_bounds__(kThreads) void argmax_pick_kernel(const float* __restrict__ part_v,
                                                               const int64_t* __restrict__ part_i, int64_t cols,
                                                               int32_t* __restrict__ out) {
  const int64_t row = blockIdx.x;
  float best = -INFINITY;
  int64_t bi = cols;
  if (threadIdx.x < kArgmaxSlices)
    take_better(part_v[row * kArgmaxSlices + threadIdx.x], part_i[row * kArgmaxSlices + threadIdx.x], best, bi);
  __shared__ float sv[kThreads];
  __shared__ int64_t si[kThreads];
  block_best(best, bi, sv, si);
  if (threadIdx.x == 0) out[row] = si[0] < cols ? (int32_t)si[0] : 0;   // all NaN / -inf: index 0
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
int launch_gather_rows(const void* src, int64_t row_bytes, const int32_t* idx, int64_t n, void* dst,
                       hipStream_t st) {
  return copy_rows(src, nullptr, row_bytes, idx, dst, nullptr, row_bytes, nullptr, n, row_bytes, st, "gather_rows");
}

int launch_scatter_kv(const void* k_new, const void* v_new, int64_t src_stride_elems,
                      const int32_t* dst_row, int64_t n, void* k_cache, void* v_cache, int Hkv, int D,
                      int dtype, hipStream_t st) {
  const int64_t es = elem_size(dtype);
  const int64_t row_bytes = (int64_t)Hkv * D * es;
  return copy_rows(k_new, v_new, src_stride_elems * es, nullptr, k_cache, v_cache, row_bytes, dst_row, n,
                   row_bytes, st, "scatter_kv");
}

int launch_rope_shift(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                      const int32_t* src_row, const int32_t* dst_row, const int32_t* delta,
                      int64_t n_tok, int Hkv, int D, const RopeFreq& f, int dtype, hipStream_t st) {
  if (n_tok <= 0) return VLC_OK;
  const int vec = dtype == VLC_BF16 ? 8 : 4;
  const int64_t threads = n_tok * Hkv * ((D / 2) / vec);
  const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads));
#define VLC_LAUNCH_SHIFT(T, DD)                                                                       \
  hipLaunchKernelGGL((rope_shift_kernel<T, DD>), grid, dim3(kThreads), 0, st, (const uint4*)k_src,    \
                     (const uint4*)v_src, (uint4*)k_dst, (uint4*)v_dst, src_row, dst_row, delta,      \
                     n_tok, Hkv, f)
  if (dtype == VLC_BF16 && D == 128) VLC_LAUNCH_SHIFT(uint16_t, 128);
  else if (dtype == VLC_BF16 && D == 64) VLC_LAUNCH_SHIFT(uint16_t, 64);
  else if (dtype == VLC_F32 && D == 128) VLC_LAUNCH_SHIFT(float, 128);
  else if (dtype == VLC_F32 && D == 64) VLC_LAUNCH_SHIFT(float, 64);
  else return fail(VLC_ERR_SHAPE, "rope shift: unsupported D=%d", D);
#undef VLC_LAUNCH_SHIFT
  VLC_CHECK_LAUNCH("rope_shift_kv");
  return VLC_OK;
}

int launch_rope_shift_jobs(const vlc_shift_job* jobs, int n_jobs, int64_t max_n_tok, int Hkv, int D,
                           const RopeFreq& f, int dtype, hipStream_t st) {
  if (n_jobs <= 0 || max_n_tok <= 0) return VLC_OK;
  const int vec = dtype == VLC_BF16 ? 8 : 4;
  const int64_t threads = max_n_tok * Hkv * ((D / 2) / vec);
  const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads), (unsigned)n_jobs);
#define VLC_LAUNCH_SHIFT(T, DD) \
  hipLaunchKernelGGL((rope_shift_jobs_kernel<T, DD>), grid, dim3(kThreads), 0, st, jobs, Hkv, f)
  if (dtype == VLC_BF16 && D == 128) VLC_LAUNCH_SHIFT(uint16_t, 128);
  else if (dtype == VLC_BF16 && D == 64) VLC_LAUNCH_SHIFT(uint16_t, 64);
  else if (dtype == VLC_F32 && D == 128) VLC_LAUNCH_SHIFT(float, 128);
  else if (dtype == VLC_F32 && D == 64) VLC_LAUNCH_SHIFT(float, 64);
  else return fail(VLC_ERR_SHAPE, "rope shift: unsupported D=%d", D);
#undef VLC_LAUNCH_SHIFT
  VLC_CHECK_LAUNCH("rope_shift_kv_layers");
  return VLC_OK;
}

int launch_rope_qk_scatter(const float* qkv32, const int32_t* pos, const int32_t* slot, int64_t n, int Hq,
                           int Hkv, int D, const RopeFreq& f, void* q_out, void* k_cache, void* v_cache,
                           int dtype, hipStream_t st, const float* partials, int splits, const void* bias,
                           const int32_t* pos3, const void* w_qnorm, const void* w_knorm, float eps) {
  if (n <= 0) return VLC_OK;
  if ((w_qnorm == nullptr) != (w_knorm == nullptr))
    return fail(VLC_ERR_NULL, "rope+scatter: q and k norm weights come together");
  if (splits > 1 && (dtype != VLC_BF16 || !partials))
    return fail(VLC_ERR_SHAPE, "rope+scatter: split partials are a bf16-path input");
  const int64_t split_stride = n * (int64_t)(Hq + 2 * Hkv) * D;
  const int vec = dtype == VLC_BF16 ? 8 : 4;
  const int heads = Hq + 2 * Hkv;
  const int64_t threads = n * heads * ((D / 2) / vec);
  const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads));
#define VLC_LAUNCH_RQS(T, DD, SUM)                                                                    \
  hipLaunchKernelGGL((rope_qk_scatter_kernel<T, DD, SUM>), grid, dim3(kThreads), 0, st,               \
                     SUM ? partials : qkv32, splits, split_stride, (const uint16_t*)bias,             \
                     const_cast<float*>(qkv32), pos, pos3, (const T*)w_qnorm, (const T*)w_knorm, eps, \
                     slot, n, Hq, Hkv, f, (uint4*)q_out, (uint4*)k_cache, (uint4*)v_cache)
  if (splits > 1 && D == 128) VLC_LAUNCH_RQS(uint16_t, 128, true);
  else if (splits > 1 && D == 64) VLC_LAUNCH_RQS(uint16_t, 64, true);
  else if (dtype == VLC_BF16 && D == 128) VLC_LAUNCH_RQS(uint16_t, 128, false);
  else if (dtype == VLC_BF16 && D == 64) VLC_LAUNCH_RQS(uint16_t, 64, false);
  else if (dtype == VLC_F32 && D == 128) VLC_LAUNCH_RQS(float, 128, false);
  else if (dtype == VLC_F32 && D == 64) VLC_LAUNCH_RQS(float, 64, false);
  else return fail(VLC_ERR_SHAPE, "rope+scatter: unsupported D=%d", D);
#undef VLC_LAUNCH_RQS
  VLC_CHECK_LAUNCH("rope_qk_scatter");
  return VLC_OK;
}

int launch_rmsnorm(const void* x, const int32_t* map, const void* w, void* y, int64_t n, int H,
                   float eps, int dtype, hipStream_t st, const int32_t* ymap) {
  if (n <= 0) return VLC_OK;
  const int vec = dtype == VLC_BF16 ? 8 : 4;
  if (H % vec) return fail(VLC_ERR_SHAPE, "rmsnorm: H=%d not a multiple of %d", H, vec);
  const int chunks = H / vec;
  const dim3 grid((unsigned)n);
  const float inv_h = 1.0f / (float)H;
#define VLC_LAUNCH_RMS(T, MAXC)                                                                       \
  hipLaunchKernelGGL((rmsnorm_kernel<T, MAXC>), grid, dim3(kThreads), 0, st, (const uint4*)x, map,    \
                     (const uint4*)w, (uint4*)y, chunks, inv_h, eps, ymap)
  if (chunks <= kThreads * 2) {
    if (dtype == VLC_BF16) VLC_LAUNCH_RMS(uint16_t, 2); else VLC_LAUNCH_RMS(float, 2);
  } else if (chunks <= kThreads * 4) {
    if (dtype == VLC_BF16) VLC_LAUNCH_RMS(uint16_t, 4); else VLC_LAUNCH_RMS(float, 4);
  } else if (chunks <= kThreads * 8) {
    if (dtype == VLC_BF16) VLC_LAUNCH_RMS(uint16_t, 8); else VLC_LAUNCH_RMS(float, 8);
  } else {
    return fail(VLC_ERR_SHAPE, "rmsnorm: H=%d too large", H);
  }
#undef VLC_LAUNCH_RMS
  VLC_CHECK_LAUNCH("rmsnorm");
  return VLC_OK;
}

int launch_sum_residual_rmsnorm(const float* partials, int splits, const void* resid, const int32_t* rmap,
                                const void* w, void* h, void* y, int64_t n, int H, float eps,
                                hipStream_t st, const int32_t* ymap) {
  if (n <= 0) return VLC_OK;
  if (H % 8) return fail(VLC_ERR_SHAPE, "sum+residual+rmsnorm: H=%d not a multiple of 8", H);
  if (splits < 1 || splits > kMaxSplits) return fail(VLC_ERR_SHAPE, "sum+residual+rmsnorm: %d splits", splits);
  const int chunks = H / 8;
  const dim3 grid((unsigned)n);
  const float inv_h = 1.0f / (float)H;
  const int64_t split_stride = n * (int64_t)H;
#define VLC_LAUNCH_SRN(MAXC)                                                                          \
  hipLaunchKernelGGL((sum_residual_rmsnorm_kernel<MAXC>), grid, dim3(kThreads), 0, st, partials,      \
                     splits, split_stride, (const uint4*)resid, rmap, (const uint4*)w, (uint4*)h,     \
                     (uint4*)y, chunks, inv_h, eps, ymap)
  if (chunks <= kThreads * 2) VLC_LAUNCH_SRN(2);
  else if (chunks <= kThreads * 4) VLC_LAUNCH_SRN(4);
  else if (chunks <= kThreads * 8) VLC_LAUNCH_SRN(8);
  else return fail(VLC_ERR_SHAPE, "sum+residual+rmsnorm: H=%d too large", H);
#undef VLC_LAUNCH_SRN
  VLC_CHECK_LAUNCH("sum_residual_rmsnorm");
  return VLC_OK;
}

int64_t argmax_ws_bytes(int64_t rows) { return rows * kArgmaxSlices * 16; }

int launch_argmax_rows(const float* x, int64_t rows, int64_t cols, int32_t* out, void* ws, hipStream_t st) {
  if (rows <= 0) return VLC_OK;
  if (cols <= 0 || cols > INT32_MAX || cols % 4 || rows > 65535)
    return fail(VLC_ERR_SHAPE, "argmax: rows=%lld cols=%lld (cols a multiple of 4)", (long long)rows, (long long)cols);
  float* part_v = static_cast<float*>(ws);
  int64_t* part_i = reinterpret_cast<int64_t*>(static_cast<char*>(ws) + rows * kArgmaxSlices * 8);   // 8-byte aligned
  hipLaunchKernelGGL(argmax_slices_kernel, dim3(kArgmaxSlices, (unsigned)rows), dim3(kThreads), 0, st, x, cols,
                     part_v, part_i);
  VLC_CHECK_LAUNCH("argmax_slices");
  hipLaunchKernelGGL(argmax_pick_kernel, dim3((unsigned)rows), dim3(kThreads), 0, st, part_v, part_i, cols, out);
  VLC_CHECK_LAUNCH("argmax_pick");
  return VLC_OK;
}

// Mean squared difference of two float arrays: per-workgroup partial sums in double, then one workgroup.
namespace {
constexpr int kMseBlocks = 1024;
__global__ __launch_bounds__(256) void sqdiff_partial_kernel(const float* __restrict__ a, const float* __restrict__ b,
                                                             int64_t n, double* __restrict__ part) {
  double s = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const double d = (double)a[i] - (double)b[i];
    s += d * d;
  }
  __shared__ double sh[256];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) part[blockIdx.x] = sh[0];
}
__global__ __launch_bounds__(256) void sqdiff_final_kernel(const double* __restrict__ part, int blocks, int64_t n,
                                                           double* __restrict__ out) {
  double s = 0.0;
  for (int i = threadIdx.x; i < blocks; i += 256) s += part[i];
  __shared__ double sh[256];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = sh[0] / (double)n;
}
}  // namespace

}  // namespace vlc

extern "C" int64_t vlc_mean_squared_error_workspace_bytes(void) { return vlc::kMseBlocks * 8; }

extern "C" int vlc_mean_squared_error(const float* a, const float* b, int64_t n, double* out, void* workspace,
                                      int64_t workspace_bytes, void* stream) {
  if (n <= 0) return vlc::fail(VLC_ERR_SHAPE, "vlc_mean_squared_error: n=%lld", (long long)n);
  if (!a || !b || !out || !workspace) return vlc::fail(VLC_ERR_NULL, "vlc_mean_squared_error: NULL pointer");
  if (workspace_bytes < vlc::kMseBlocks * 8 || ((uintptr_t)workspace & 7))
    return vlc::fail(VLC_ERR_WORKSPACE, "vlc_mean_squared_error: workspace of %lld bytes, %d needed (8-byte aligned)",
                     (long long)workspace_bytes, vlc::kMseBlocks * 8);
  const int blocks = (int)((n + 255) / 256 < vlc::kMseBlocks ? (n + 255) / 256 : vlc::kMseBlocks);
  hipLaunchKernelGGL(vlc::sqdiff_partial_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, a, b, n,
                     static_cast<double*>(workspace));
  VLC_CHECK_LAUNCH("sqdiff_partial");
  hipLaunchKernelGGL(vlc::sqdiff_final_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const double*>(workspace), blocks, n, out);
  VLC_CHECK_LAUNCH("sqdiff_final");
  return VLC_OK;
}

// ---------------------------------------------------------------------------------------------
// C ABI entry points of the streaming kernels
// ---------------------------------------------------------------------------------------------
using vlc::fail;

extern "C" int vlc_gather_rows(const void* src, int64_t src_rows, int64_t row_elems, const int32_t* idx,
                               int64_t n, void* dst, int dtype, void* stream) {
  if (dtype != VLC_F32 && dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "vlc_gather_rows: dtype=%d", dtype);
  if (n < 0 || src_rows < 0 || row_elems <= 0)
    return fail(VLC_ERR_SHAPE, "vlc_gather_rows: n=%lld src_rows=%lld row_elems=%lld", (long long)n,
                (long long)src_rows, (long long)row_elems);
  if (n == 0) return VLC_OK;
  if (!src || !idx || !dst) return fail(VLC_ERR_NULL, "vlc_gather_rows: NULL pointer");
  const int64_t row_bytes = row_elems * vlc::elem_size(dtype);
  if (row_bytes % 16) return fail(VLC_ERR_SHAPE, "vlc_gather_rows: row of %lld bytes is not a multiple of 16",
                                  (long long)row_bytes);
  if (((uintptr_t)src | (uintptr_t)dst) & 15) return fail(VLC_ERR_SHAPE, "vlc_gather_rows: pointers must be 16-byte aligned");
  return vlc::launch_gather_rows(src, row_bytes, idx, n, dst, (hipStream_t)stream);
}

static int check_kv(const char* who, int Hkv, int D, int dtype) {
  if (dtype != VLC_F32 && dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "%s: dtype=%d", who, dtype);
  if (Hkv <= 0 || (D != 64 && D != 128)) return fail(VLC_ERR_SHAPE, "%s: Hkv=%d D=%d unsupported", who, Hkv, D);
  return VLC_OK;
}

extern "C" int vlc_rope_shift_kv(const void* k_src, const void* v_src, void* k_dst, void* v_dst,
                                 const int32_t* src_row, const int32_t* dst_row, const int32_t* delta,
                                 int64_t n_tok, int Hkv, int D, double rope_base, int dtype, void* stream) {
  int rc = check_kv("vlc_rope_shift_kv", Hkv, D, dtype);
  if (rc) return rc;
  if (n_tok < 0) return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv: n_tok=%lld", (long long)n_tok);
  if (!(rope_base > 0.0)) return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv: rope_base must be positive");
  if (n_tok == 0) return VLC_OK;
  if (!k_src || !k_dst || !src_row || !dst_row || !delta)
    return fail(VLC_ERR_NULL, "vlc_rope_shift_kv: NULL pointer");
  if (((uintptr_t)k_src | (uintptr_t)k_dst | (uintptr_t)v_src | (uintptr_t)v_dst) & 15)
    return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv: pointers must be 16-byte aligned");
  return vlc::launch_rope_shift(k_src, v_src, k_dst, v_dst, src_row, dst_row, delta, n_tok, Hkv, D,
                                vlc::make_rope_freq(rope_base, D), dtype, (hipStream_t)stream);
}

extern "C" int vlc_rope_shift_kv_layers(const vlc_shift_job* jobs, int n_jobs, int64_t max_n_tok, int Hkv, int D,
                                       double rope_base, int dtype, void* stream) {
  int rc = check_kv("vlc_rope_shift_kv_layers", Hkv, D, dtype);
  if (rc) return rc;
  if (n_jobs < 0 || n_jobs > 65535)
    return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv_layers: n_jobs=%d (0 ... 65535)", n_jobs);
  if (max_n_tok < 0 || max_n_tok > ((int64_t)1 << 31))
    return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv_layers: max_n_tok=%lld", (long long)max_n_tok);
  if (!(rope_base > 0.0)) return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv_layers: rope_base must be positive");
  if (n_jobs == 0 || max_n_tok == 0) return VLC_OK;
  if (!jobs) return fail(VLC_ERR_NULL, "vlc_rope_shift_kv_layers: jobs is NULL");
  if ((uintptr_t)jobs & 7) return fail(VLC_ERR_SHAPE, "vlc_rope_shift_kv_layers: jobs must be 8-byte aligned");
  return vlc::launch_rope_shift_jobs(jobs, n_jobs, max_n_tok, Hkv, D, vlc::make_rope_freq(rope_base, D), dtype,
                                     (hipStream_t)stream);
}

extern "C" int vlc_scatter_kv(const void* k_new, const void* v_new, const int32_t* dst_row, int64_t n,
                              void* k_cache, void* v_cache, int64_t cache_rows, int Hkv, int D, int dtype,
                              void* stream) {
  int rc = check_kv("vlc_scatter_kv", Hkv, D, dtype);
  if (rc) return rc;
  if (n < 0 || cache_rows < 0) return fail(VLC_ERR_SHAPE, "vlc_scatter_kv: n=%lld cache_rows=%lld", (long long)n, (long long)cache_rows);
  if (n == 0) return VLC_OK;
  if (!k_new || !v_new || !dst_row || !k_cache || !v_cache) return fail(VLC_ERR_NULL, "vlc_scatter_kv: NULL pointer");
  if (n > cache_rows) return fail(VLC_ERR_INDEX, "vlc_scatter_kv: %lld unique rows cannot fit a cache of %lld rows", (long long)n, (long long)cache_rows);
  if (((uintptr_t)k_new | (uintptr_t)v_new | (uintptr_t)k_cache | (uintptr_t)v_cache) & 15)
    return fail(VLC_ERR_SHAPE, "vlc_scatter_kv: pointers must be 16-byte aligned");
  return vlc::launch_scatter_kv(k_new, v_new, (int64_t)Hkv * D, dst_row, n, k_cache, v_cache, Hkv, D, dtype,
                                (hipStream_t)stream);
}
