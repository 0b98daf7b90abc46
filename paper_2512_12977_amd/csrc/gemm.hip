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
// two floats -> packed bf16 pair with the hardware conversion (round to nearest even), one instruction
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
// x * sigmoid(x) with the hardware reciprocal (1 ulp) instead of an IEEE division (a dozen instructions per
// element in an epilogue during which the MFMAs are idle); the result is rounded to bf16 anyway
__device__ __forceinline__ float silu_f(float x) { return x * __builtin_amdgcn_rcpf(1.0f + __expf(-x)); }

// ---------------------------------------------------------------------------------------------
// tile id -> (tile_m, tile_n).  Workgroups are dealt round-robin to the 8 XCDs, each with its own
// L2; the remap hands every XCD one contiguous range of tile ids, and inside a range tiles are
// walked in groups of GROUP_M row-tiles so that concurrently resident tiles share A and W panels.
// ---------------------------------------------------------------------------------------------
constexpr int kXcds = 8;
constexpr int kGroupM = 8;

__device__ __forceinline__ int xcd_contiguous(int pid, int total) {
  const int per = total / kXcds;
  return pid < per * kXcds ? (pid % kXcds) * per + pid / kXcds : pid;
}

template <bool REMAP = true>
__device__ __forceinline__ void tile_coords(int pid, int total, int tiles_m, int tiles_n, int* tm, int* tn) {
  const int vid = REMAP ? xcd_contiguous(pid, total) : pid;
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
// Workgroup tile BM x BN, WGM x WGN wavefronts, wavefront tile (BM/WGM) x (BN/WGN) made of 32x32
// MFMA tiles.  The MFMA "A" operand is the W fragment and the "B" operand the activation fragment,
// so an accumulator tile is indexed [n][m]: lane l holds, for m = l % 32, the outputs
// n = 8*(j/4) + 4*(l/32) + j%4 (j = register index): four consecutive n per lane, i.e. 8 contiguous
// bytes of a bf16 C row.
//
// Operands reach LDS straight from global memory (global_load_lds, 16 bytes per lane, no register
// staging) through a ring of STAGES k-tiles of 64 columns, so the next k-tile is in flight while
// the current one is consumed.  Inside a k-tile the instruction stream is laid out in groups of four
// MFMAs, each preceded by its share of the next k-step's fragment reads and - in the first half of
// the k-tile only, so every load has at least half a k-tile of latency cover - of the next k-tile's
// global loads; sched_barrier keeps the compiler from regrouping them.  A wavefront-level load writes 64 consecutive 16-byte chunks of LDS
// in lane order; the XOR swizzle that keeps the later 16-byte fragment reads of consecutive rows
// in different banks is therefore applied on the global side (which chunk of its row each lane
// fetches).  Fragments are double-buffered in registers across the four 16-wide k-steps.
//
// SPLIT > 1 (few output tiles): each workgroup reduces one contiguous range of k-tiles and
// writes float partials; splitk_epilogue_kernel sums them and applies the epilogue.
//
// Tail split: when the tile count is not a multiple of the workgroups the chip holds at once, the
// last, partly filled round would cost as much as a full one.  The tiles of that round (ids from
// full_tiles on) are then shared out over tail_splits workgroups each, along k; these write their
// accumulators as float blocks to tail_ws and tail_reduce_kernel sums them and applies the epilogue.
constexpr int BK = 64;

__device__ __forceinline__ int fswz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// One wavefront-level global -> LDS copy of 64 x 16 bytes: lane l's 16 bytes land at lds_byte_addr + 16*l.
// Written as inline assembly rather than through the builtin because the compiler, seeing an LDS
// write it cannot order against the fragment reads, waits for every outstanding LDS access before
// each k-step; issued this way the loads are tracked only by the explicit vmcnt waits below (the
// loop contains no other vector-memory instruction).  M0 holds the LDS address; the compiler never
// keeps a live value in M0 across statements (it is reserved and written right before each use).
// The global address is a wavefront-uniform base (scalar registers) plus a 32-bit byte offset per lane: the lane
// offsets never change, the base moves along k with scalar adds, so the k-loop holds no vector address arithmetic
// (a vector instruction of a wavefront does not overlap with its own MFMAs).
__device__ __forceinline__ void dma16(const void* uniform_base, uint32_t lane_byte_off, uint32_t lds_byte_addr) {
#ifdef VLC_ABLATE_GEMM_COPIES   // measurement build: no operand ever reaches LDS (results wrong, timing only)
  return;
#endif
#ifdef VLC_ABLATE_GEMM_LDS_WRITES   // measurement build: the same loads, into a register nobody reads instead of LDS
  u32x4 sink;
  asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(sink) : "v"(lane_byte_off), "s"(uniform_base) : "memory");
  return;
#endif
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_byte_addr), "v"(lane_byte_off), "s"(uniform_base)
               : "memory");
}

#define VLC_WAITCNT_VM(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (7 << 4) | (15 << 8) | (((N) >> 4) << 14))

enum { EPI_PARTIAL = 100 };   // internal: float partial sums of one k-range (split-K)

//
// GROUPED (mixture-of-experts): the row tiles come from a device-resident table; entry t holds an
// expert and the range [m0, m_end) of rows it owns (at most BM of them); the tile multiplies these
// rows - fetched through amap when given - with that expert's matrix W + expert * w_stride.
// Workgroups beyond the table's length (only known on the device) exit at once.
template <int BM, int BN, int WGM, int WGN, int STAGES, int OCC, int EPI, bool GROUPED = false>
__global__ __launch_bounds__(WGM * WGN * 64, OCC) void gemm_bf16_kernel(
    const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ W, uint16_t* __restrict__ C,
    int64_t ldc, int M, int N, int K, const uint16_t* __restrict__ bias, const uint16_t* __restrict__ resid,
    int64_t ldr, const int32_t* __restrict__ rmap, int tiles_m, int tiles_n, int kt_per_split, int full_tiles,
    int tail_splits, float* __restrict__ tail_ws, const GroupTile* __restrict__ gtab,
    const int32_t* __restrict__ g_ntiles, const int32_t* __restrict__ amap, int64_t w_stride) {
  constexpr int NW = WGM * WGN;
  constexpr int WM = BM / WGM, WN = BN / WGN;      // wavefront tile
  constexpr int MT = WM / 32, NT = WN / 32;        // MFMA tiles per wavefront
  constexpr int STAGE_CHUNKS = (BM + BN) * 8;      // 16-byte chunks per stage
  constexpr int A_INSTR = BM * 8 / 64 / NW, W_INSTR = BN * 8 / 64 / NW;   // wavefront loads per k-tile
  constexpr int LOADS = A_INSTR + W_INSTR;
  constexpr int KS = BK / 16;
  // columns of C covered by this tile: SwiGLU consumes a gate and an up row per output column
  constexpr int CN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  static_assert(STAGES >= 2 && STAGES <= 4, "ring depth");
  // SwiGLU pairs a gate and an up column inside a lane.  Even NT: the wavefront's first NT/2 tiles are gate columns,
  // the others the up columns of the same outputs.  Odd NT (MIXED): FT = NT/2 such pairs of tiles, then one tile
  // whose columns 0-15 are gate and 16-31 up columns of 16 more outputs (registers j and j + 8 of a lane).
  constexpr bool MIXED = EPI == EPI_SWIGLU && NT % 2 == 1;
  constexpr int FT = NT / 2;
  static_assert(!MIXED || WN == 64 * FT + 32, "mixed SwiGLU tile: wavefront columns");
  // W row of the tile (= LDS row) -> row of the weight matrix relative to n0; the up rows lie N rows further
  auto swiglu_row = [&](int r, bool* up) {
    if constexpr (MIXED) {
      const int wv = r / WN, lr = r - wv * WN;
      int c;
      if (lr < 32 * FT) { *up = false; c = lr; }
      else if (lr < 64 * FT) { *up = true; c = lr - 32 * FT; }
      else { const int m = lr - 64 * FT; *up = m >= 16; c = 32 * FT + (m & 15); }
      return wv * (WN / 2) + c;
    } else {
      *up = r >= BN / 2;
      return *up ? r - BN / 2 : r;
    }
  };

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* lds = reinterpret_cast<u32x4*>(smem);

  const int tiles = tiles_m * tiles_n;
  int split = 0, pid = blockIdx.x, tail_block = -1;   // tail_block >= 0: this workgroup owns one k-range of a tail tile
  if constexpr (EPI == EPI_PARTIAL) {
    // the whole grid (k range major) is dealt to the XCDs in contiguous pieces: an XCD then works on one or two
    // k ranges and its L2 holds only their slices of A, instead of every XCD streaming all of A
    const int b = xcd_contiguous(blockIdx.x, gridDim.x);
    split = b / tiles;
    pid = b - split * tiles;
  } else if ((int)blockIdx.x >= full_tiles) {
    tail_block = blockIdx.x - full_tiles;
    const int t = tail_block / tail_splits;
    split = tail_block - t * tail_splits;
    pid = full_tiles + t;
  }
  int tm, tn;
  tile_coords<EPI != EPI_PARTIAL>(pid, tiles, tiles_m, tiles_n, &tm, &tn);
  int m0 = tm * BM;
  const int n0 = tn * CN;
  if constexpr (GROUPED) {
    if (tm >= *g_ntiles) return;
    const GroupTile g = gtab[tm];
    m0 = g.m0;
    M = g.m_end;
    W += (int64_t)g.expert * w_stride;
  }

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int l32 = lane & 31, x = lane >> 5;

  const int kt_begin = split * kt_per_split;
  const int kt_end = (EPI == EPI_PARTIAL || tail_block >= 0) ? min(K / BK, kt_begin + kt_per_split) : K / BK;
  const int KT = kt_end - kt_begin;

  // ---- global source of each of this wavefront's loads: a uniform base (first row of the tile, k-tile
  // kt_begin) and a per-lane byte offset.  Rows fetched through amap are offsets from A itself.
  uint32_t a_lane[A_INSTR], w_lane[W_INSTR];
  const bool mapped = GROUPED && amap != nullptr;
  const uint16_t* a_base = A + (mapped ? (int64_t)0 : (int64_t)m0 * lda) + (int64_t)kt_begin * BK;
  const uint16_t* w_base = W + (int64_t)n0 * K + (int64_t)kt_begin * BK;
#pragma unroll
  for (int i = 0; i < A_INSTR; ++i) {
    const int p = (wave * A_INSTR + i) * 64 + lane;        // LDS chunk this lane fills
    const int r = p >> 3, c = (p & 7) ^ fswz(r);
    int gr = m0 + r;
    gr = gr < M ? gr : M - 1;                              // ragged tail: re-read the last row
    int64_t rel = gr - m0;
    if constexpr (GROUPED) {
      if (mapped) rel = amap[gr];
    }
    a_lane[i] = (uint32_t)((rel * lda + c * 8) * 2);
  }
#pragma unroll
  for (int i = 0; i < W_INSTR; ++i) {
    const int p = (wave * W_INSTR + i) * 64 + lane;
    const int r = p >> 3, c = (p & 7) ^ fswz(r);
    int gr;
    if constexpr (EPI == EPI_SWIGLU) {
      bool up;
      const int c = swiglu_row(r, &up);
      gr = (up ? N : 0) + n0 + c;
    } else {
      gr = n0 + r;
    }
    const int limit = (EPI == EPI_SWIGLU) ? 2 * N : N;
    gr = gr < limit ? gr : limit - 1;
    w_lane[i] = (uint32_t)(((int64_t)(gr - n0) * K + c * 8) * 2);
  }
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds;
  // LDS byte address of this wavefront's i-th load of a stage (A part first, then W)
#define VLC_LDS_DST(stage_, i_)                                                                              \
  (lds_base + (uint32_t)(((stage_) * STAGE_CHUNKS +                                                           \
                          ((i_) < A_INSTR ? wave * A_INSTR * 64 + (i_) * 64                                  \
                                          : BM * 8 + wave * W_INSTR * 64 + ((i_) - A_INSTR) * 64)) * 16))
#ifdef VLC_ABLATE_GEMM_COPY_MISSES   // measurement build: every copy re-reads the tile's first two k-tiles (cache hits)
#define VLC_DMA_KT(kt_) ((kt_) & 1)
#else
#define VLC_DMA_KT(kt_) (kt_)
#endif
#define VLC_DMA(kt_, i_, stage_)                                                                              \
  dma16(((i_) < A_INSTR ? a_base : w_base) + VLC_DMA_KT(kt_) * BK,                                                \
        (i_) < A_INSTR ? a_lane[(i_) < A_INSTR ? (i_) : 0] : w_lane[(i_) >= A_INSTR ? (i_) - A_INSTR : 0],     \
        VLC_LDS_DST(stage_, i_))
#define VLC_ISSUE(kt_, stage_) _Pragma("unroll") for (int i = 0; i < LOADS; ++i) VLC_DMA(kt_, i, stage_);

  // fragment positions inside a stage (chunk units) for every 16-wide k-step
  int w_off[NT][KS], a_off[MT][KS];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int r;
    if constexpr (EPI == EPI_SWIGLU && !MIXED)
      r = (nt < NT / 2 ? wn * (WN / 2) + nt * 32 : BN / 2 + wn * (WN / 2) + (nt - NT / 2) * 32) + l32;
    else
      r = wn * WN + nt * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) w_off[nt][ks] = BM * 8 + r * 8 + ((2 * ks + x) ^ fswz(r));
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int r = wm * WM + mt * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a_off[mt][ks] = r * 8 + ((2 * ks + x) ^ fswz(r));
  }

  f32x16 acc[NT][MT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // One k-tile: KS k-steps of G groups of four MFMAs.  WITH_LOADS: the loads of k-tile nkt_ (into
  // stage nst_) are issued in the first half of the groups.
  constexpr int MPG = (NT * MT) % 4 == 0 ? 4 : 2;   // MFMAs per group
  constexpr int G = NT * MT / MPG;             // groups per k-step
  constexpr int TG = KS * G;                   // groups per k-tile
  constexpr int NF = NT + MT;                  // fragments per k-step
  static_assert(NT * MT % MPG == 0, "wavefront tile must hold whole groups of MFMA tiles");
#define VLC_COMPUTE_TILE(cst_, WITH_LOADS, nkt_, nst_)                                                        \
  {                                                                                                           \
    const u32x4* st_ = lds + (cst_) * STAGE_CHUNKS;                                                           \
    bf16x8 wf[2][NT], af[2][MT];                                                                              \
    _Pragma("unroll") for (int nt = 0; nt < NT; ++nt) wf[0][nt] = __builtin_bit_cast(bf16x8, VLC_GEMM_FRAG(st_[w_off[nt][0]])); \
    _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) af[0][mt] = __builtin_bit_cast(bf16x8, VLC_GEMM_FRAG(st_[a_off[mt][0]])); \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                                       \
      _Pragma("unroll") for (int g = 0; g < G; ++g) {                                                         \
        if (WITH_LOADS) {                                                                                     \
          _Pragma("unroll") for (int i = 0; i < LOADS; ++i)                                                   \
            if (i * (TG / 2) / LOADS == ks * G + g) VLC_DMA(nkt_, i, nst_);                                    \
        }                                                                                                     \
        if (ks + 1 < KS) {                                                                                    \
          _Pragma("unroll") for (int f = 0; f < NF; ++f) {                                                    \
            if (f * G / NF == g) {                                                                            \
              if (f < NT) wf[(ks + 1) & 1][f < NT ? f : 0] = __builtin_bit_cast(bf16x8, VLC_GEMM_FRAG(st_[w_off[f < NT ? f : 0][ks + 1]])); \
              else af[(ks + 1) & 1][f >= NT ? f - NT : 0] = __builtin_bit_cast(bf16x8, VLC_GEMM_FRAG(st_[a_off[f >= NT ? f - NT : 0][ks + 1]])); \
            }                                                                                                 \
          }                                                                                                   \
        }                                                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                                    \
        _Pragma("unroll") for (int j = 0; j < MPG; ++j) {                                                     \
          const int t_ = g * MPG + j;                                                                         \
          acc[t_ / MT][t_ % MT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[ks & 1][t_ / MT], af[ks & 1][t_ % MT], \
                                                                          acc[t_ / MT][t_ % MT], 0, 0, 0);    \
        }                                                                                                     \
        __builtin_amdgcn_sched_barrier(0);                                                                    \
      }                                                                                                       \
    }                                                                                                         \
  }

#if defined(VLC_ABLATE_GEMM_COPIES) || defined(VLC_ABLATE_GEMM_LDS_WRITES)
  // measurement build: the ring is filled once with pseudo-random finite bf16 values (so that the MFMAs draw the power
  // of a real product) and no copy is ever issued
  for (int i = tid; i < STAGES * STAGE_CHUNKS; i += NW * 64) {
    uint32_t h = (uint32_t)i * 2654435761u + blockIdx.x * 40503u;
    u32x4 v;
    for (int e = 0; e < 4; ++e) {
      h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
      v[e] = (h & 0x807f807fu) | 0x3f003f00u;
    }
    lds[i] = v;
  }
  __syncthreads();
#endif
#ifdef VLC_ABLATE_GEMM_FRAG_READS
  // measurement build: every MFMA operand is one register-resident pseudo-random fragment, nothing is read from LDS
  u32x4 frag_rand;
  {
    uint32_t h = (uint32_t)tid * 2654435761u + 12345u;
    for (int e = 0; e < 4; ++e) {
      h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
      frag_rand[e] = (h & 0x807f807fu) | 0x3f003f00u;
    }
  }
#define VLC_GEMM_FRAG(x_) frag_rand
#else
#define VLC_GEMM_FRAG(x_) (x_)
#endif
  // prologue: fill STAGES-1 stages
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < KT) { VLC_ISSUE(s, s) }
  int kt = 0;
  if constexpr (STAGES == 2) {
    // two k-tiles per trip, so that the stage every fragment address refers to is a constant of the code
    // and the addresses of both stages stay in registers (no address arithmetic inside the loop)
    for (; kt + 2 < KT; kt += 2) {
      VLC_WAITCNT_VM(0);
      __syncthreads();
      VLC_COMPUTE_TILE(0, true, kt + 1, 1)
      VLC_WAITCNT_VM(0);
      __syncthreads();
      VLC_COMPUTE_TILE(1, true, kt + 2, 0)
    }
  }
  for (; kt + STAGES - 1 < KT; ++kt) {   // steady state: k-tile kt+STAGES-1 is fetched while kt is consumed
    VLC_WAITCNT_VM((STAGES - 2) * LOADS);          // this wavefront's part of k-tile kt has landed
    __syncthreads();                               // everyone's part has; stage (kt-1)%STAGES is free
    VLC_COMPUTE_TILE(kt % STAGES, true, kt + STAGES - 1, (kt + STAGES - 1) % STAGES)
  }
  for (; kt < KT; ++kt) {                // drain
    const int later = KT - 1 - kt;
    if (later >= 2) { VLC_WAITCNT_VM(2 * LOADS); } else if (later == 1) { VLC_WAITCNT_VM(LOADS); } else { VLC_WAITCNT_VM(0); }
    __syncthreads();
    VLC_COMPUTE_TILE(kt % STAGES, false, 0, 0)
  }
#undef VLC_ISSUE
#undef VLC_DMA
#undef VLC_LDS_DST
#undef VLC_COMPUTE_TILE
#undef VLC_GEMM_FRAG

  // ---- tail tile: raw accumulators as a float block [BN/4][BM][4] (lanes of consecutive m write 512 contiguous bytes)
  if constexpr (EPI != EPI_PARTIAL) {
    if (tail_block >= 0) {
      float* P = tail_ws + (int64_t)tail_block * (BM * BN);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int ml = wm * WM + mt * 32 + l32;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          int j0;   // gate | up position (gate columns of the tile first, then its up columns) this tile starts at
          if constexpr (EPI == EPI_SWIGLU)
            j0 = nt < FT ? wn * (WN / 2) + nt * 32 : BN / 2 + wn * (WN / 2) + (nt - FT) * 32;
          else
            j0 = wn * WN + nt * 32;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            int j = j0 + 4 * x + 8 * q;
            if constexpr (MIXED) {
              if (nt == NT - 1) j = (q < 2 ? 0 : BN / 2) + wn * (WN / 2) + 32 * FT + 4 * x + 8 * (q & 1);
            }
            *reinterpret_cast<float4*>(P + ((int64_t)(j >> 2) * BM + ml) * 4) =
                make_float4(acc[nt][mt][4 * q], acc[nt][mt][4 * q + 1], acc[nt][mt][4 * q + 2], acc[nt][mt][4 * q + 3]);
          }
        }
      }
      return;
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  constexpr int ONT = (EPI == EPI_SWIGLU) ? NT / 2 : NT;   // output tiles along n per wavefront
  constexpr int OWN = (EPI == EPI_SWIGLU) ? WN / 2 : WN;   // output columns per wavefront
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = m0 + wm * WM + mt * 32 + l32;
    if (m >= M) continue;
    int64_t rrow = 0;
    if constexpr (EPI == EPI_RESIDUAL) rrow = rmap ? (int64_t)rmap[m] : (int64_t)m;
#pragma unroll
    for (int nt = 0; nt < ONT; ++nt) {
      const int nbase = n0 + wn * OWN + nt * 32 + 4 * x;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nbase + 8 * q;
        if (n >= N) continue;                                  // N is a multiple of 4
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[nt][mt][4 * q + e];
        if constexpr (EPI == EPI_PARTIAL) {
          float* P = reinterpret_cast<float*>(C) + ((int64_t)split * M + m) * ldc + n;
          *reinterpret_cast<float4*>(P) = make_float4(v[0], v[1], v[2], v[3]);
          continue;
        }
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
        } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = silu_f(v[e]) * acc[nt + NT / 2][mt][4 * q + e];
        }
        if constexpr (EPI == EPI_BIAS_F32) {   // unrounded float output (C is a float matrix)
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + (int64_t)m * ldc + n) =
              make_float4(v[0], v[1], v[2], v[3]);
        } else {
          uint2 o;
          o.x = pack_bf16x2(v[0], v[1]);
          o.y = pack_bf16x2(v[2], v[3]);
#ifdef VLC_ABLATE_GEMM_STORES   // measurement build: the SwiGLU epilogue computes, and stores only what can never occur
          if (EPI == EPI_SWIGLU && o.x != 0x7fc17fc1u) continue;   // (its own inputs stay what they are; only the product after it sees stale data)
#endif
          *reinterpret_cast<uint2*>(C + (int64_t)m * ldc + n) = o;
        }
      }
    }
    if constexpr (MIXED) {   // the last tile: gate columns in registers 0-7, the up columns of the same outputs in 8-15
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int n = n0 + wn * OWN + 32 * FT + 4 * x + 8 * q;
        if (n >= N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = silu_f(acc[NT - 1][mt][4 * q + e]) * acc[NT - 1][mt][4 * (q + 2) + e];
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>(C + (int64_t)m * ldc + n) = o;
      }
    }
  }
}

// Sum of the split-K partials [splits][M][N] (float) + epilogue; one thread per 4 columns.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_epilogue_kernel(const float* __restrict__ P, int splits,
                                                              uint16_t* __restrict__ C, int64_t ldc, int M, int N,
                                                              const uint16_t* __restrict__ bias,
                                                              const uint16_t* __restrict__ resid, int64_t ldr,
                                                              const int32_t* __restrict__ rmap) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int nq = N / 4;
  const int64_t m = id / nq;
  const int n = (int)(id - m * nq) * 4;
  if (m >= M) return;
  // all loads first (independent), then the sum in split order
  float4 part[8];
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (k < splits) part[k] = *reinterpret_cast<const float4*>(P + ((int64_t)k * M + m) * N + n);
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int k = 0; k < 8; ++k)
    if (k < splits) { s.x += part[k].x; s.y += part[k].y; s.z += part[k].z; s.w += part[k].w; }
  if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_F32) {
    if (bias) {
      const uint2 b = *reinterpret_cast<const uint2*>(bias + n);
      s.x += __uint_as_float(b.x << 16); s.y += __uint_as_float(b.x & 0xffff0000u);
      s.z += __uint_as_float(b.y << 16); s.w += __uint_as_float(b.y & 0xffff0000u);
    }
  } else if constexpr (EPI == EPI_RESIDUAL) {
    const int64_t rrow = rmap ? (int64_t)rmap[m] : m;
    const uint2 b = *reinterpret_cast<const uint2*>(resid + rrow * ldr + n);
    s.x += __uint_as_float(b.x << 16); s.y += __uint_as_float(b.x & 0xffff0000u);
    s.z += __uint_as_float(b.y << 16); s.w += __uint_as_float(b.y & 0xffff0000u);
  }
  if constexpr (EPI == EPI_BIAS_F32) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + m * ldc + n) = s;
  } else {
    uint2 o;
    o.x = pack_bf16x2(s.x, s.y);
    o.y = pack_bf16x2(s.z, s.w);
    *reinterpret_cast<uint2*>(C + m * ldc + n) = o;
  }
}

// Sum over k-ranges of the tail tiles' float blocks + epilogue.  grid (BM * QN / 256, tail tiles), QN = quads of
// output columns per tile; a thread owns four consecutive columns of one row.
template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void tail_reduce_kernel(const float* __restrict__ P, int splits, int full_tiles,
                                                          int tiles_m, int tiles_n, uint16_t* __restrict__ C,
                                                          int64_t ldc, int M, int N,
                                                          const uint16_t* __restrict__ bias,
                                                          const uint16_t* __restrict__ resid, int64_t ldr,
                                                          const int32_t* __restrict__ rmap) {
  constexpr int CN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int t = blockIdx.y;
  int tm, tn;
  tile_coords(full_tiles + t, tiles_m * tiles_n, tiles_m, tiles_n, &tm, &tn);
  const int id = blockIdx.x * 256 + threadIdx.x;
  const int jq = id / BM, ml = id - jq * BM;          // consecutive threads: consecutive rows (contiguous float4 reads)
  const int m = tm * BM + ml, n = tn * CN + 4 * jq;
  if (m >= M || n >= N) return;
  const float* base = P + (int64_t)t * splits * (BM * BN) + ((int64_t)jq * BM + ml) * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f), u = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int k = 0; k < splits; ++k) {
    const float4 a = *reinterpret_cast<const float4*>(base + (int64_t)k * (BM * BN));
    s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
    if constexpr (EPI == EPI_SWIGLU) {
      const float4 b = *reinterpret_cast<const float4*>(base + (int64_t)k * (BM * BN) + (int64_t)(BN / 8) * BM * 4);
      u.x += b.x; u.y += b.y; u.z += b.z; u.w += b.w;
    }
  }
  if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_F32) {
    if (bias) {
      const uint2 b = *reinterpret_cast<const uint2*>(bias + n);
      s.x += __uint_as_float(b.x << 16); s.y += __uint_as_float(b.x & 0xffff0000u);
      s.z += __uint_as_float(b.y << 16); s.w += __uint_as_float(b.y & 0xffff0000u);
    }
  } else if constexpr (EPI == EPI_RESIDUAL) {
    const int64_t rrow = rmap ? (int64_t)rmap[m] : (int64_t)m;
    const uint2 b = *reinterpret_cast<const uint2*>(resid + rrow * ldr + n);
    s.x += __uint_as_float(b.x << 16); s.y += __uint_as_float(b.x & 0xffff0000u);
    s.z += __uint_as_float(b.y << 16); s.w += __uint_as_float(b.y & 0xffff0000u);
  } else if constexpr (EPI == EPI_SWIGLU) {
    s.x = silu_f(s.x) * u.x; s.y = silu_f(s.y) * u.y; s.z = silu_f(s.z) * u.z; s.w = silu_f(s.w) * u.w;
  }
  if constexpr (EPI == EPI_BIAS_F32) {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + (int64_t)m * ldc + n) = s;
  } else {
    uint2 o;
    o.x = pack_bf16x2(s.x, s.y);
    o.y = pack_bf16x2(s.z, s.w);
    *reinterpret_cast<uint2*>(C + (int64_t)m * ldc + n) = o;
  }
}

// ---------------------------------------------------------------------------------------------
// f32 SIMT kernel: 64 x 64 tile, 256 threads, 4 x 4 outputs per thread, k-tile 16
// ---------------------------------------------------------------------------------------------
template <int EPI, bool GROUPED = false>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ A, int64_t lda,
                                                       const float* __restrict__ W, float* __restrict__ C,
                                                       int64_t ldc, int M, int N, int K,
                                                       const float* __restrict__ bias,
                                                       const float* __restrict__ resid, int64_t ldr,
                                                       const int32_t* __restrict__ rmap,
                                                       const GroupTile* __restrict__ gtab,
                                                       const int32_t* __restrict__ g_ntiles,
                                                       const int32_t* __restrict__ amap, int64_t w_stride) {
  constexpr int T = 64, KB = 16;
  constexpr int NW = (EPI == EPI_SWIGLU) ? 2 : 1;
  __shared__ float As[KB][T + 1];
  __shared__ float Ws[NW][KB][T + 1];
  int m0 = blockIdx.y * T;
  const int n0 = blockIdx.x * T;
  if constexpr (GROUPED) {       // see gemm_bf16_kernel
    if ((int)blockIdx.y >= *g_ntiles) return;
    const GroupTile g = gtab[blockIdx.y];
    m0 = g.m0;
    M = g.m_end;
    W += (int64_t)g.expert * w_stride;
  }
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  float acc[NW][4][4] = {};
  for (int k0 = 0; k0 < K; k0 += KB) {
    for (int e = threadIdx.x; e < T * KB; e += 256) {
      const int r = e / KB, kk = e % KB;
      const int m = m0 + r, n = n0 + r, k = k0 + kk;
      int64_t am = m;
      if constexpr (GROUPED) {
        if (amap && m < M) am = amap[m];
      }
      As[kk][r] = (m < M && k < K) ? A[am * lda + k] : 0.f;
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

template <int BM, int BN, int WGM, int WGN, int STAGES, int OCC, int EPI>
int launch_bf16(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                int64_t K, const void* bias, const void* resid, int64_t ldr, const int32_t* rmap, int splits,
                int kt_per_split, void* tail_ws, int64_t tail_ws_bytes, hipStream_t st) {
  constexpr int CN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + CN - 1) / CN);
  const int tiles = tiles_m * tiles_n;
  const size_t lds = (size_t)STAGES * (BM + BN) * BK * 2;
  auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, STAGES, OCC, EPI>;
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds)) return rc;
  // Tail split: the chip holds `slots` workgroups at once; the tiles of the last, partly filled round are
  // shared out over as many k-ranges as fit into the idle slots (at least 8 k-tiles each).
  constexpr int slots = 256 * OCC;
  const int KT = (int)(K / BK);
  int full = tiles * splits, tail = 0, tsp = 1, tkt = kt_per_split;
  if constexpr (EPI != EPI_PARTIAL) {
    tail = tiles % slots;
    if (tail_ws && tail > 0 && tiles > tail) {
      tsp = slots / tail;
      if (tsp > KT / 8) tsp = KT / 8;
      const int64_t fit = tail_ws_bytes / ((int64_t)tail * BM * BN * 4);
      if (tsp > fit) tsp = (int)fit;
    }
    if (tsp >= 2) {
      tkt = (KT + tsp - 1) / tsp;
      tsp = (KT + tkt - 1) / tkt;
      full = tiles - tail;
    } else {
      tail = 0;
      tsp = 1;
    }
  }
  hipLaunchKernelGGL(kern, dim3(full + tail * tsp), dim3(WGM * WGN * 64), lds, st, (const uint16_t*)A, lda,
                     (const uint16_t*)W, (uint16_t*)C, ldc, (int)M, (int)N, (int)K, (const uint16_t*)bias,
                     (const uint16_t*)resid, ldr, rmap, tiles_m, tiles_n, tkt, full, tsp, (float*)tail_ws,
                     (const GroupTile*)nullptr, (const int32_t*)nullptr, (const int32_t*)nullptr, (int64_t)0);
  VLC_CHECK_LAUNCH("gemm_bf16");
  if constexpr (EPI != EPI_PARTIAL) {
    if (tail > 0) {
      hipLaunchKernelGGL((tail_reduce_kernel<BM, BN, EPI>), dim3(BM * (CN / 4) / 256, tail), dim3(256), 0, st,
                         (const float*)tail_ws, tsp, full, tiles_m, tiles_n, (uint16_t*)C, ldc, (int)M, (int)N,
                         (const uint16_t*)bias, (const uint16_t*)resid, ldr, rmap);
      VLC_CHECK_LAUNCH("gemm_tail_reduce");
    }
  }
  return VLC_OK;
}

// Tile choice.  Many rows: 256 x 256 tiles, 4 wavefronts of 128 x 128 or 8 of 64 x 128.  Few rows: two workgroups per CU, on
// 128 x 192 tiles for gate|up (4 wavefronts of 64 x 96: 32 gate, 32 up and a mixed tile of 16 + 16 columns, so that
// each holds the gate and the up columns of its 48 outputs), and on 128 x 128 (4 wavefronts of 64 x 64) or 128 x 192
// tiles (4 of 64 x 96) for the others, whose k range is split as well if the tiles still leave most of the 256 CUs idle.
template <int EPI>
int dispatch_bf16(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                  int64_t K, const void* bias, const void* resid, int64_t ldr, const int32_t* rmap,
                  void* splitk_ws, int64_t splitk_ws_bytes, int* deferred, hipStream_t st) {
  const int KT = (int)(K / BK);
  // 256 x 256 tiles (one workgroup per CU) against the small tiles (two per CU).
  bool big;
  if constexpr (EPI == EPI_SWIGLU) {
    // Both in rounds of resident workgroups, the last round shortened by the tail split as launch_bf16 does it.
    // A round of 256 x 256 tiles takes 1.09 rounds of 128 x 192 tiles (measured rates 1.26 and 1.03 PFLOP/s with
    // thousands of tiles); its workgroups have nobody beside them on the CU to cover their start, their end and the
    // float blocks of a split tile, which with few rounds costs about a quarter round per launch and a fifth per
    // split tail (fitted on 596 ... 1600 rows at three shapes: the small tile wins up to about 1000 rows).
    auto rounds = [KT](int64_t tiles, int slots, float split_cost) {
      const int64_t full = tiles / slots, tail = tiles % slots;
      float r = (float)full;
      if (tail > 0) {
        const int64_t tsp = full > 0 ? (slots / tail < KT / 8 ? slots / tail : KT / 8) : 1;
        r += tsp >= 2 ? 1.0f / (float)tsp + split_cost : 1.0f;
      }
      return r;
    };
    const int64_t tiles_big = ((M + 255) / 256) * ((N + 127) / 128), tiles_small = ((M + 127) / 128) * ((N + 95) / 96);
    big = 1.09f * rounds(tiles_big, 256, 0.2f) + 0.25f < rounds(tiles_small, 512, 0.1f);
  } else {
    // with few output columns (the o, down and qkv products) there are not enough 256 x 256 tiles for the 256 CUs
    // until several thousand rows: the small tiles with a split k range stay ahead
    big = M >= 1536 && ((M + 255) / 256) * ((N + 255) / 256) >= 200;
  }
  if (big) {
    // gate|up: 4 wavefronts of 128 x 128; the others: 8 wavefronts of 64 x 128 (no spilled registers around the
    // loop; the projection with float output gains 8 %, gate|up would lose 2 %)
    if constexpr (EPI == EPI_SWIGLU)
      return launch_bf16<256, 256, 2, 2, 2, 1, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, 1, KT,
                                                    splitk_ws, splitk_ws_bytes, st);
    else
      return launch_bf16<256, 256, 4, 2, 2, 1, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, 1, KT,
                                                    splitk_ws, splitk_ws_bytes, st);
  }
  if constexpr (EPI == EPI_SWIGLU) {
    return launch_bf16<128, 192, 2, 2, 2, 2, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, 1, KT, splitk_ws,
                                                  splitk_ws_bytes, st);
  } else {
    // Tile width (128 or 192 columns) and number of k ranges, by cost in units of one 128 x 128 workgroup's
    // k-tile (~1.2 us; 1.35 of them for a 128 x 192 k-tile): (rounds of the 512 resident workgroups) x (k-tiles
    // per workgroup), plus, when the k range is split, a second kernel (2 units) and per split one float
    // matrix written and read back (8 bytes per element at ~4 TB/s = 1.7e-6 units per element).  At least
    // 8 k-tiles per split; no split from 384 tiles on.
    if constexpr (EPI == EPI_BIAS_F32) {
      // At most one 64-row tile of rows (the first-token head: a few requests against the whole output matrix): the
      // product is bound by reading the matrix once, so 64 x 128 tiles on a four-stage ring, one workgroup per CU -
      // 4 % faster there than 128 x 192 tiles (195-200 us against 203-208 at 152064 x 3584).
      if (M <= 64)
        return launch_bf16<64, 128, 2, 2, 4, 1, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, 1, KT, nullptr, 0, st);
    }
    int splits = 1, width = 128;
    float best = 0.f;
    for (int tn = 128; tn <= 192; tn += 64) {
      const int64_t tiles = ((M + 127) / 128) * ((N + tn - 1) / tn);
      const float unit = tn == 128 ? 1.0f : 1.35f;
      const float whole = (float)((tiles + 511) / 512) * (float)KT * unit;
      if (tn == 128 || whole < best) {
        best = whole;
        splits = 1;
        width = tn;
      }
      if (!splitk_ws || tiles >= 384) continue;
      for (int sp = 2; sp <= 8; ++sp) {
        if (KT / sp < 8 || (int64_t)sp * M * N * 4 > splitk_ws_bytes) break;
        const float cost = (float)(((tiles * sp + 511) / 512) * ((KT + sp - 1) / sp)) * unit + 2.0f +
                           (float)sp * (float)(M * N) * 1.7e-6f;
        if (cost < best) {
          best = cost;
          splits = sp;
          width = tn;
        }
      }
    }
    if (splits <= 1) {
      if (width == 192)
        return launch_bf16<128, 192, 2, 2, 2, 2, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, 1, KT,
                                                      splitk_ws, splitk_ws_bytes, st);
      return launch_bf16<128, 128, 2, 2, 2, 2, EPI>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, 1, KT,
                                                    splitk_ws, splitk_ws_bytes, st);
    }
    const int per = (KT + splits - 1) / splits;
    splits = (KT + per - 1) / per;
    int rc;
    if (width == 192)
      rc = launch_bf16<128, 192, 2, 2, 2, 2, EPI_PARTIAL>(A, lda, W, splitk_ws, N, M, N, K, nullptr, nullptr, 0,
                                                          nullptr, splits, per, nullptr, 0, st);
    else
      rc = launch_bf16<128, 128, 2, 2, 2, 2, EPI_PARTIAL>(A, lda, W, splitk_ws, N, M, N, K, nullptr, nullptr, 0,
                                                          nullptr, splits, per, nullptr, 0, st);
    if (rc) return rc;
    if (deferred) {   // the caller's next kernel sums the partials and applies the epilogue
      *deferred = splits;
      return VLC_OK;
    }
    const int64_t threads = M * (N / 4);
    hipLaunchKernelGGL(splitk_epilogue_kernel<EPI>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st,
                       (const float*)splitk_ws, splits, (uint16_t*)C, ldc, (int)M, (int)N, (const uint16_t*)bias,
                       (const uint16_t*)resid, ldr, rmap);
    VLC_CHECK_LAUNCH("splitk_epilogue");
    return VLC_OK;
  }
}

template <int EPI>
int launch_f32(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
               int64_t K, const void* bias, const void* resid, int64_t ldr, const int32_t* rmap,
               hipStream_t st) {
  const dim3 grid((unsigned)((N + 63) / 64), (unsigned)((M + 63) / 64));
  hipLaunchKernelGGL(gemm_f32_kernel<EPI>, grid, dim3(256), 0, st, (const float*)A, lda, (const float*)W,
                     (float*)C, ldc, (int)M, (int)N, (int)K, (const float*)bias, (const float*)resid, ldr,
                     rmap, (const GroupTile*)nullptr, (const int32_t*)nullptr, (const int32_t*)nullptr, (int64_t)0);
  VLC_CHECK_LAUNCH("gemm_f32");
  return VLC_OK;
}

// Grouped launches: the grid covers the largest number of row tiles the table can hold.
template <int BM, int BN, int WGM, int WGN, int STAGES, int OCC, int EPI>
int launch_bf16_grouped(const void* A, int64_t lda, const int32_t* amap, const void* W, int64_t w_stride, void* C,
                        int64_t ldc, int64_t N, int64_t K, const GroupTile* gtab, const int32_t* g_ntiles,
                        int max_tiles_m, hipStream_t st) {
  constexpr int CN = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  const int tiles_n = (int)((N + CN - 1) / CN);
  const size_t lds = (size_t)STAGES * (BM + BN) * BK * 2;
  auto kern = gemm_bf16_kernel<BM, BN, WGM, WGN, STAGES, OCC, EPI, true>;
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), (int)lds)) return rc;
  const int grid = max_tiles_m * tiles_n;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WGM * WGN * 64), lds, st, (const uint16_t*)A, lda, (const uint16_t*)W,
                     (uint16_t*)C, ldc, 0, (int)N, (int)K, (const uint16_t*)nullptr, (const uint16_t*)nullptr,
                     (int64_t)0, (const int32_t*)nullptr, max_tiles_m, tiles_n, (int)(K / BK), grid, 1,
                     (float*)nullptr, gtab, g_ntiles, amap, w_stride);
  VLC_CHECK_LAUNCH("gemm_bf16_grouped");
  return VLC_OK;
}

template <int EPI>
int launch_f32_grouped(const void* A, int64_t lda, const int32_t* amap, const void* W, int64_t w_stride, void* C,
                       int64_t ldc, int64_t N, int64_t K, const GroupTile* gtab, const int32_t* g_ntiles,
                       int max_tiles_m, hipStream_t st) {
  const dim3 grid((unsigned)((N + 63) / 64), (unsigned)max_tiles_m);
  hipLaunchKernelGGL((gemm_f32_kernel<EPI, true>), grid, dim3(256), 0, st, (const float*)A, lda, (const float*)W,
                     (float*)C, ldc, 0, (int)N, (int)K, (const float*)nullptr, (const float*)nullptr, (int64_t)0,
                     (const int32_t*)nullptr, gtab, g_ntiles, amap, w_stride);
  VLC_CHECK_LAUNCH("gemm_f32_grouped");
  return VLC_OK;
}

}  // namespace

// Whole-GEMM split-K only runs when a GEMM has fewer than 384 tiles of 128 x 128, and then uses about
// 512 / tiles splits: splits * M * N floats stay below 2 * 512 * 128 * 128 * 4 bytes.  The tail split
// writes at most one float block per resident workgroup: 256 x (256 x 256) or 512 x (128 x 128) floats.
int64_t gemm_splitk_ws_bytes(int64_t n_rows, int64_t max_n) {
  (void)max_n;
  return n_rows > 0 ? (int64_t)64 << 20 : 0;
}

// Rows per tile of the grouped GEMMs, from the mean number of rows per group.  Few rows per group: every
// matrix is streamed from HBM exactly once and nothing is reused, so the tile is small (64 x 128) and the
// ring three stages deep - with two workgroups per CU that keeps 64 KB of matrix data in flight per CU,
// what the HBM latency needs; a two-stage ring of 128 x 128 tiles stalls at half of that.
int gemm_group_tile_rows(int64_t rows, int n_groups, int dtype) {
  if (dtype != VLC_BF16) return 64;
  const int64_t mean = rows / (n_groups > 0 ? n_groups : 1);
  return mean >= 192 ? 256 : (mean >= 56 ? 128 : 64);
}

int launch_gemm_grouped(const void* A, int64_t lda, const int32_t* amap, const void* W, int64_t w_stride, void* C,
                        int64_t ldc, int64_t rows, int n_groups, int64_t N, int64_t K, int epilogue,
                        const GroupTile* tiles, const int32_t* n_tiles, int tile_rows, int dtype, hipStream_t st,
                        int64_t a_rows) {
  if (rows <= 0 || N <= 0) return VLC_OK;
  if (K <= 0 || n_groups <= 0) return fail(VLC_ERR_SHAPE, "grouped gemm: K=%lld groups=%d", (long long)K, n_groups);
  if (rows > INT32_MAX || N > INT32_MAX / 2 || K > INT32_MAX)
    return fail(VLC_ERR_SHAPE, "grouped gemm: dimension exceeds 32-bit tile indexing");
  if (tile_rows != gemm_group_tile_rows(rows, n_groups, dtype))
    return fail(VLC_ERR_SHAPE, "grouped gemm: the tile table was built for %d rows per tile", tile_rows);
  const int max_tiles = (int)(rows / tile_rows) + n_groups;
  if (epilogue != EPI_BIAS && epilogue != EPI_SWIGLU)
    return fail(VLC_ERR_SHAPE, "grouped gemm: epilogue=%d", epilogue);
  if (dtype == VLC_BF16) {
    if (K % BK || N % 4 || lda % 8 || ldc % 4)
      return fail(VLC_ERR_SHAPE, "grouped gemm(bf16): K=%lld must be a multiple of %d, N, lda, ldc aligned", (long long)K, BK);
    // 32-bit lane offsets: rows fetched through amap are offsets from A itself (amap values are below a_rows)
    if ((amap ? a_rows : 256) * lda * 2 >= ((int64_t)1 << 31) || ((epilogue == EPI_SWIGLU ? N : 0) + 256) * K * 2 >= ((int64_t)1 << 31))
      return fail(VLC_ERR_SHAPE, "grouped gemm(bf16): operand rows span more than 2 GiB");
    if (tile_rows == 256) {
      if (epilogue == EPI_SWIGLU)
        return launch_bf16_grouped<256, 256, 2, 2, 2, 1, EPI_SWIGLU>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
      return launch_bf16_grouped<256, 256, 2, 2, 2, 1, EPI_BIAS>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
    }
    if (tile_rows == 64) {
      if (epilogue == EPI_SWIGLU)
        return launch_bf16_grouped<64, 128, 2, 2, 3, 2, EPI_SWIGLU>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
      return launch_bf16_grouped<64, 128, 2, 2, 3, 2, EPI_BIAS>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
    }
    if (epilogue == EPI_SWIGLU)
      return launch_bf16_grouped<128, 128, 2, 2, 2, 2, EPI_SWIGLU>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
    return launch_bf16_grouped<128, 128, 2, 2, 2, 2, EPI_BIAS>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
  }
  if (dtype == VLC_F32) {
    if (epilogue == EPI_SWIGLU)
      return launch_f32_grouped<EPI_SWIGLU>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
    return launch_f32_grouped<EPI_BIAS>(A, lda, amap, W, w_stride, C, ldc, N, K, tiles, n_tiles, max_tiles, st);
  }
  return fail(VLC_ERR_DTYPE, "grouped gemm: dtype=%d", dtype);
}

int launch_gemm(const void* A, int64_t lda, const void* W, void* C, int64_t ldc, int64_t M, int64_t N,
                int64_t K, int epilogue, const void* bias, const void* resid, int64_t ldr,
                const int32_t* rmap, int dtype, void* splitk_ws, int64_t splitk_ws_bytes, hipStream_t st,
                int* deferred) {
  if (deferred) *deferred = 0;
  if (M <= 0 || N <= 0) return VLC_OK;
  if (K <= 0) return fail(VLC_ERR_SHAPE, "gemm: K=%lld", (long long)K);
  if (M > INT32_MAX || N > INT32_MAX / 2 || K > INT32_MAX)
    return fail(VLC_ERR_SHAPE, "gemm: dimension exceeds 32-bit tile indexing");
  if (dtype == VLC_BF16) {
    if (K % BK) return fail(VLC_ERR_SHAPE, "gemm(bf16): K=%lld must be a multiple of %d", (long long)K, BK);
    if (N % 4 || lda % 8 || ldc % 4 || (epilogue == EPI_RESIDUAL && ldr % 4))
      return fail(VLC_ERR_SHAPE, "gemm(bf16): N, lda, ldc, ldr must keep 8-byte (A: 16-byte) alignment");
    // lane offsets of the loads are 32-bit byte offsets from the tile's first row (SwiGLU: up rows sit N rows on)
    if (256 * lda * 2 >= ((int64_t)1 << 31) || ((epilogue == EPI_SWIGLU ? N : 0) + 256) * K * 2 >= ((int64_t)1 << 31))
      return fail(VLC_ERR_SHAPE, "gemm(bf16): a tile's rows span more than 2 GiB (lda=%lld N=%lld K=%lld)",
                  (long long)lda, (long long)N, (long long)K);
    switch (epilogue) {
      case EPI_BIAS: return dispatch_bf16<EPI_BIAS>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, splitk_ws, splitk_ws_bytes, deferred, st);
      case EPI_BIAS_F32: return dispatch_bf16<EPI_BIAS_F32>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, splitk_ws, splitk_ws_bytes, deferred, st);
      case EPI_RESIDUAL: return dispatch_bf16<EPI_RESIDUAL>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, splitk_ws, splitk_ws_bytes, deferred, st);
      case EPI_SWIGLU: return dispatch_bf16<EPI_SWIGLU>(A, lda, W, C, ldc, M, N, K, bias, resid, ldr, rmap, splitk_ws, splitk_ws_bytes, deferred, st);
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
