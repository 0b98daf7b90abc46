// GEMMs of the recomputed rows: C[M,N] = epilogue(A[M,K] * W[N,K]^T), both operands K-contiguous.
//   bf16: MFMA (v_mfma_f32_32x32x16_bf16), LDS-tiled, float accumulation.
//   f32 : plain SIMT tile kernel (the small fp32 configuration).
// Epilogues: + bias, + residual (optionally gathered through a row map), SwiGLU of a gate|up pair.
#include <hip/hip_runtime.h>

#include "vlc_internal.h"

namespace vlc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // a 16-byte chunk (native vector: stays in registers)

__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {   // round to nearest, ties to even
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + __expf(-x)); }

// ---------------------------------------------------------------------------------------------
// tile id -> (tile_m, tile_n).  Workgroups are dealt round-robin to the 8 XCDs, each with its own
// L2; the remap hands every XCD one contiguous range of tile ids, and inside a range tiles are
// walked in groups of GROUP_M row-tiles so that concurrently resident tiles share A and W panels.
// ---------------------------------------------------------------------------------------------
constexpr int kXcds = 8;
constexpr int kGroupM = 8;

__device__ __forceinline__ void tile_coords(int pid, int total, int tiles_m, int tiles_n, int* tm, int* tn) {
  const int per = total / kXcds;
  int vid = pid;
  if (pid < per * kXcds) vid = (pid % kXcds) * per + pid / kXcds;
  const int in_group = kGroupM * tiles_n;
  const int group = vid / in_group;
  const int first_m = group * kGroupM;
  const int gm = min(tiles_m - first_m, kGroupM);
  const int r = vid - group * in_group;
  *tm = first_m + r % gm;
  *tn = r / gm;
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ---------------------------------------------------------------------------------------------
// Workgroup: 256 threads = 4 wavefronts in a 2 x 2 grid; wavefront tile (BM/2) x (BN/2) made of
// 32x32 MFMA tiles.  The MFMA "A" operand is the W fragment and the "B" operand the activation
// fragment, so an accumulator tile is indexed [n][m]: lane l holds, for m = l % 32, the outputs
// n = 8*(j/4) + 4*(l/32) + j%4 (j = register index): four consecutive n per lane, i.e. 8
// contiguous bytes of a C row.
//
// LDS holds [rows][64] bf16 tiles (128 B per row = 8 chunks of 16 B); the chunk index is XOR-ed
// with a function of the row so that the 16-byte fragment reads of consecutive rows fall into
// different banks.
constexpr int BK = 64;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row & 7) ^ ((row >> 3) & 1)); }

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(
    const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ W, uint16_t* __restrict__ C,
    int64_t ldc, int M, int N, int K, const uint16_t* __restrict__ bias, const uint16_t* __restrict__ resid,
    int64_t ldr, const int32_t* __restrict__ rmap, int tiles_m, int tiles_n) {
  constexpr int WM = BM / 2, WN = BN / 2;        // wavefront tile
  constexpr int MT = WM / 32, NT = WN / 32;      // MFMA tiles per wavefront
  constexpr int A_ITERS = BM / 32, W_ITERS = BN / 32;   // 16-byte chunks per thread per k-tile
  // columns of C covered by this tile: SwiGLU consumes a gate and an up row per output column
  constexpr int CN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* ldsA = reinterpret_cast<u32x4*>(smem);                     // [2][BM][8] chunks
  u32x4* ldsW = reinterpret_cast<u32x4*>(smem) + 2 * BM * 8;        // [2][BN][8] chunks

  int tm, tn;
  tile_coords(blockIdx.x, gridDim.x, tiles_m, tiles_n, &tm, &tn);
  const int m0 = tm * BM, n0 = tn * CN;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, x = lane >> 5;

  // ---- global -> register staging: thread handles chunk (tid % 8) of rows tid/8 + 32*i ----------
  const int ld_row = tid >> 3, ld_chunk = tid & 7;
  const u32x4* a_src[A_ITERS];
  const u32x4* w_src[W_ITERS];
#pragma unroll
  for (int i = 0; i < A_ITERS; ++i) {
    int r = m0 + ld_row + 32 * i;
    r = r < M ? r : M - 1;                                  // ragged tail: re-read the last row
    a_src[i] = reinterpret_cast<const u32x4*>(A + (int64_t)r * lda) + ld_chunk;
  }
#pragma unroll
  for (int i = 0; i < W_ITERS; ++i) {
    const int lr = ld_row + 32 * i;                          // row inside the LDS W tile
    int r;
    if (EPI == EPI_SWIGLU) r = lr < BN / 2 ? n0 + lr : N + n0 + (lr - BN / 2);   // gate rows | up rows
    else r = n0 + lr;
    const int limit = (EPI == EPI_SWIGLU) ? 2 * N : N;
    r = r < limit ? r : limit - 1;
    w_src[i] = reinterpret_cast<const u32x4*>(W + (int64_t)r * K) + ld_chunk;
  }
  u32x4 a_reg[A_ITERS], w_reg[W_ITERS];

#define VLC_LOAD_GLOBAL(kt_)                                                                 \
  _Pragma("unroll") for (int i = 0; i < A_ITERS; ++i) a_reg[i] = a_src[i][(kt_) * (BK / 8)]; \
  _Pragma("unroll") for (int i = 0; i < W_ITERS; ++i) w_reg[i] = w_src[i][(kt_) * (BK / 8)];
#define VLC_STORE_LDS(buf_)                                                                 \
  _Pragma("unroll") for (int i = 0; i < A_ITERS; ++i) {                                     \
    const int r_ = ld_row + 32 * i;                                                         \
    ldsA[((buf_) * BM + r_) * 8 + swz(r_, ld_chunk)] = a_reg[i];                            \
  }                                                                                         \
  _Pragma("unroll") for (int i = 0; i < W_ITERS; ++i) {                                     \
    const int r_ = ld_row + 32 * i;                                                         \
    ldsW[((buf_) * BN + r_) * 8 + swz(r_, ld_chunk)] = w_reg[i];                            \
  }

  // LDS row of MFMA tile nt of this wavefront inside the W tile
  int w_row[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if constexpr (EPI == EPI_SWIGLU)
      w_row[nt] = nt < NT / 2 ? wn * (WN / 2) + nt * 32 : BN / 2 + wn * (WN / 2) + (nt - NT / 2) * 32;
    else
      w_row[nt] = wn * WN + nt * 32;
  }

  f32x16 acc[NT][MT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int KT = K / BK;
  VLC_LOAD_GLOBAL(0)
  VLC_STORE_LDS(0)
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < KT) { VLC_LOAD_GLOBAL(kt + 1) }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 wf[NT], af[MT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int r = w_row[nt] + l32;
        const u32x4 v = ldsW[(buf * BN + r) * 8 + swz(r, 2 * ks + x)];
        wf[nt] = __builtin_bit_cast(bf16x8, v);
      }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int r = wm * WM + mt * 32 + l32;
        const u32x4 v = ldsA[(buf * BM + r) * 8 + swz(r, 2 * ks + x)];
        af[mt] = __builtin_bit_cast(bf16x8, v);
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nt], af[mt], acc[nt][mt], 0, 0, 0);
    }
    if (kt + 1 < KT) { VLC_STORE_LDS(buf ^ 1) }
    __syncthreads();
  }
#undef VLC_LOAD_GLOBAL
#undef VLC_STORE_LDS

  // ---- epilogue ---------------------------------------------------------------------------------
  constexpr int ONT = (EPI == EPI_SWIGLU) ? NT / 2 : NT;   // output tiles along n per wavefront
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m0 + wm * WM + mt * 32 + l32;
    if (m >= M) continue;
    int64_t rrow = 0;
    if constexpr (EPI == EPI_RESIDUAL) rrow = rmap ? (int64_t)rmap[m] : (int64_t)m;
#pragma unroll
    for (int nt = 0; nt < ONT; ++nt) {
      const int nbase = n0 + ((EPI == EPI_SWIGLU) ? wn * (WN / 2) : wn * WN) + nt * 32 + 4 * x;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nbase + 8 * q;
        if (n >= N) continue;                                  // N is a multiple of 4
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[nt][mt][4 * q + e];
        if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_F32) {
          if (bias) {
            const uint2 b = *reinterpret_cast<const uint2*>(bias + n);
            v[0] += __uint_as_float(b.x << 16); v[1] += __uint_as_float(b.x & 0xffff0000u);
            v[2] += __uint_as_float(b.y << 16); v[3] += __uint_as_float(b.y & 0xffff0000u);
          }
        } else if constexpr (EPI == EPI_RESIDUAL) {
          const uint2 b = *reinterpret_cast<const uint2*>(resid + rrow * ldr + n);
          v[0] += __uint_as_float(b.x << 16); v[1] += __uint_as_float(b.x & 0xffff0000u);
          v[2] += __uint_as_float(b.y << 16); v[3] += __uint_as_float(b.y & 0xffff0000u);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = silu_f(v[e]) * acc[nt + NT / 2][mt][4 * q + e];
        }
        if constexpr (EPI == EPI_BIAS_F32) {   // unrounded float output (C is a float matrix)
          float4 o = make_float4(v[0], v[1], v[2], v[3]);
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + (int64_t)m * ldc + n) = o;
        } else {
          uint2 o;
          o.x = f32_to_bf16(v[0]) | (f32_to_bf16(v[1]) << 16);
          o.y = f32_to_bf16(v[2]) | (f32_to_bf16(v[3]) << 16);
          *reinterpret_cast<uint2*>(C + (int64_t)m * ldc + n) = o;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// f32 SIMT kernel: 64 x 64 tile, 256 threads, 4 x 4 outputs per thread, k-tile 16
// ---------------------------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t lda,
                                                       const float* __restrict__ W, float* __restrict__ C,
                                                       int64_t ldc, int M, int N, int K,
                                                       const float* __restrict__ bias,
                                                       const float* __restrict__ resid, int64_t ldr,
                                                       const int32_t* __restrict__ rmap) {
  constexpr int T = 64, KB = 16;
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  __shared__ float As[KB][T + 1];
  __shared__ float Ws[NW][KB][T + 1];
  const int m0 = blockIdx.y * T, n0 = blockIdx.x * T;
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[NW][4][4] = {};
  for (int k0 = 0; k0 < K; k0 += KB) {
    for (int e = threadIdx.x; e < T * KB; e += 256) {
      const int r = e / KB, kk = e % KB;
      const int m = m0 + r, n = n0 + r, k = k0 + kk;
      As[kk][r] = (m < M && k < K) ? A[(int64_t)m * lda + k] : 0.f;
      Ws[0][kk][r] = (n < N && k < K) ? W[(int64_t)n * K + k] : 0.f;
      if (EPI == EPI_SWIGLU) Ws[NW - 1][kk][r] = (n < N && k < K) ? W[(int64_t)(N + n) * K + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KB; ++kk) {
      float a[4], w[NW][4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int s = 0; s < NW; ++s)
#pragma unroll
        for (int j = 0; j < 4; ++j) w[s][j] = Ws[s][kk][tx * 4 + j];
#pragma unroll
      for (int s = 0; s < NW; ++s)
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[s][i][j] = fmaf(a[i], w[s][j], acc[s][i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[0][i][j];
      if (EPI == EPI_BIAS) {
        if (bias) v += bias[n];
      } else if (EPI == EPI_RESIDUAL) {
        const int64_t rr = rmap ? (int64_t)rmap[m] : (int64_t)m;
        v += resid[rr * ldr + n];
      } else {
        v = v / (1.0f + expf(-v)) * acc[NW - 1][i][j];
      }
      C[(int64_t)m * ldc + n] = v;
    }
  }
}

template <int BM, int BN, int EPI>
int launch_bf16(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                int64_t K, const void* bias, const void* resid, int64_t ldr, const int32_t* rmap,
                hipStream_t st) {
  constexpr int CN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + CN - 1) / CN);
  const size_t lds = (size_t)2 * (BM + BN) * BK * 2;
  auto kern = gemm_bf16_kernel<BM, BN, EPI>;
  static bool attr_set = false;    // raising the dynamic LDS limit is per kernel, once per process
  if (!attr_set) {
    VLC_CHECK_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), lds, st, (const uint16_t*)A, lda,
                     (const uint16_t*)W, (uint16_t*)C, ldc, (int)M, (int)N, (int)K, (const uint16_t*)bias,
                     (const uint16_t*)resid, ldr, rmap, tiles_m, tiles_n);
  VLC_CHECK_LAUNCH("gemm_bf16");
  return VLC_OK;
}

template <int EPI>
int dispatch_bf16(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                  int64_t K, const void* bias, const void* resid, int64_t ldr, const int32_t* rmap,
                  hipStream_t st) {
  // Few rows: 128-row tiles waste less of the ragged tail and put more workgroups on the chip.
  if (M <= 1024) return launch_bf16<128, 256, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
  return launch_bf16<256, 256, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
}

template <int EPI>
int launch_f32(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
               int64_t K, const void* bias, const void* resid, int64_t ldr, const int32_t* rmap,
               hipStream_t st) {
  const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
  hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, st, (const float*)A, lda, (const float*)W,
                     (float*)C, ldc, (int)M, (int)N, (int)K, (const float*)bias, (const float*)resid, ldr,
                     rmap);
  VLC_CHECK_LAUNCH("gemm_f32");
  return VLC_OK;
}

}  // namespace

int launch_gemm(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                int64_t K, int epilogue, const void* bias, const void* resid, int64_t ldr,
                const int32_t* rmap, int dtype, hipStream_t st) {
  if (M <= 0 || N <= 0) return VLC_OK;
  if (K <= 0) return fail(VLC_ERR_SHAPE, "gemm: K=%lld", (long long)K);
  if (M > INT32_MAX || N > INT32_MAX / 2 || K > INT32_MAX)
    return fail(VLC_ERR_SHAPE, "gemm: dimension exceeds 32-bit tile indexing");
  if (dtype == VLC_BF16) {
    if (K % BK) return fail(VLC_ERR_SHAPE, "gemm(bf16): K=%lld must be a multiple of %d", (long long)K, BK);
    if (N % 4 || lda % 8 || ldc % 4 || (epilogue == EPI_RESIDUAL && ldr % 4))
      return fail(VLC_ERR_SHAPE, "gemm(bf16): N, lda, ldc, ldr must keep 8-byte (A: 16-byte) alignment");
    switch (epilogue) {
      case EPI_BIAS: return dispatch_bf16<EPI_BIAS>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
      case EPI_BIAS_F32: return dispatch_bf16<EPI_BIAS_F32>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
      case EPI_RESIDUAL: return dispatch_bf16<EPI_RESIDUAL>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
      case EPI_SWIGLU: return dispatch_bf16<EPI_SWIGLU>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
    }
  } else if (dtype == VLC_F32) {
    switch (epilogue) {
      case EPI_BIAS:
      case EPI_BIAS_F32: return launch_f32<EPI_BIAS>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
      case EPI_RESIDUAL: return launch_f32<EPI_RESIDUAL>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
      case EPI_SWIGLU: return launch_f32<EPI_SWIGLU>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, st);
    }
  }
  return fail(VLC_ERR_DTYPE, "gemm: dtype=%d epilogue=%d", dtype, epilogue);
}

}  // namespace vlc
