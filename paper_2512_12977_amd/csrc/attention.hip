// Attention for the recomputed query rows only, over the whole blended K/V of their request
// (Fig. 4 of the paper: row blocks of the recomputed tokens, each spanning its full causal key range).
//   bf16: MFMA flash-style kernel, one workgroup per (block of query rows, kv head); the g = Hq/Hkv
//         query heads that share a kv head are stacked into the same tile so K/V are streamed once
//         for all of them.
//   f32 : one wavefront per (row, head), online softmax (the small fp32 configuration).
#include <hip/hip_runtime.h>

#include "vlc_internal.h"

namespace vlc {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

__device__ __forceinline__ uint32_t f32_to_bf16(float f) {   // round to nearest, ties to even
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) { return f32_to_bf16(a) | (f32_to_bf16(b) << 16); }

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel, D = 128
// ---------------------------------------------------------------------------------------------
// Tile: VR = 128 "virtual rows" = (query row, head of the kv group) pairs, head fastest; 4 wavefronts
// of 32 virtual rows each, two workgroups per CU.  Keys are consumed in blocks of 64.
//
// Both products are computed transposed so that every lane owns exactly one virtual row:
//   S^T[key, vr] = K[key, :] . Q[vr, :]      MFMA A = K fragment (LDS), B = Q fragment (registers)
//   O^T[d,  vr] += V^T[d, key] P^T[key, vr]  MFMA A = V^T fragment (LDS), B = P^T (from S^T registers)
// In the 32x32 accumulator layout lane l holds column vr = l % 32 and rows 8*(j/4) + 4*(l/32) + j%4,
// so a row's running max / sum / rescale factor are per-lane scalars and the only cross-lane step is
// one exchange between lanes l and l^32.  The S^T accumulators feed the second MFMA directly: its
// contraction index is just a relabeling of keys, as long as the V^T fragment uses the same
// relabeling, which is how V^T is laid out in LDS.
//
// K/V blocks go through a two-stage LDS ring: while block kb is consumed, the K and V tiles of block
// kb+1 are copied global -> LDS directly, both row-major [key][d] (the XOR swizzles are applied by
// permuting which 16-byte chunk each lane fetches).  The V^T fragments are read with the transposing
// LDS load (ds_read_b64_tr_b16): inside a group of 16 lanes, lane i receives element i%4 of the four
// 8-byte chunks addressed by lanes i/4, i/4+4, i/4+8, i/4+12; with lane s of the group pointing at
// row key0 + s/4, columns d0 + 4*(s%4), lane i ends up with V[key0 .. key0+3][d0 + i].
constexpr int ATT_D = 128;
constexpr int KB = 64;        // keys per block
constexpr int VR = 128;       // virtual rows per workgroup
constexpr int K_TILE_CHUNKS = KB * 16;      // [64 keys][16 chunks of 8 d]
constexpr int V_TILE_CHUNKS = KB * 16;      // same shape
constexpr int ATT_STAGE_CHUNKS = K_TILE_CHUNKS + V_TILE_CHUNKS;   // one K tile + one V tile

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// K tile: chunk XOR key%16 (16-byte fragment reads of consecutive keys hit different banks).
// V tile: chunk XOR (key%4)*4 (a transposing read touches 4 consecutive keys x 64 bytes).
__device__ __forceinline__ int k_swz(int key, int c) { return c ^ (key & 15); }
__device__ __forceinline__ int v_swz(int key, int c) { return c ^ ((key & 3) << 2); }

// One wavefront-level global -> LDS copy of 64 x 16 bytes (lane l's 16 bytes land at dst + l).  Issued
// as inline assembly: through the builtin the compiler, unable to tell the LDS write apart from the
// fragment reads that follow, waits for every outstanding copy (vmcnt(0)) before the first of them,
// which serialises the prefetch with the block it was meant to overlap.  This way the copies are
// tracked only by the explicit waits at the end of each key block (the key loop has no other
// vector-memory instruction).  M0 holds the LDS address and is written right before each use.
__device__ __forceinline__ void dma16(const void* gptr, u32x4* lds_dst) {
#ifdef VLC_ABLATE_ATT_COPIES   // measurement build: no K/V tile ever reaches LDS (the rings hold pseudo-random values)
  return;
#endif
  const uint32_t a = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_dst;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
               :
               : "s"(a), "v"(gptr)
               : "memory");
}

// max / sum over the two lanes (l, l ^ 32) that share a virtual row, in both of them: the swap puts
// the upper half's values beside the lower half's without an LDS round trip (a ds_bpermute here
// would also make the wavefront wait for every fragment read in flight)
__device__ __forceinline__ float pair_max(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

#define VLC_ATT_WAIT_VM0() __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8) | (0 << 14))

// Measurement variants (python -m paper_2512_12977_amd.build --tag T --define VLC_ABLATE_...): each takes one
// ingredient of the key loop out - the results are wrong, only the timing is of interest - to show what that
// ingredient costs: the K or V^T fragment reads from LDS (all or every other one), the exponentials, the scale-and-subtract
// in front of them, the S^T or the PV MFMAs, the workgroup barrier of a key block, the K/V copies into LDS.
#ifdef VLC_ABLATE_K_READS
#define VLC_ATT_KFRAG(expr_) (u32x4{(uint32_t)lane, 0x3c003c00u, (uint32_t)wave, 0x3c003c00u})
#else
#define VLC_ATT_KFRAG(expr_) (expr_)
#endif
#ifdef VLC_ABLATE_V_READS
#define VLC_ATT_VFRAG(expr_) (s16x4{(short)lane, (short)0x3c00, (short)wave, (short)0x3c00})
#else
#define VLC_ATT_VFRAG(expr_) (expr_)
#endif
#ifdef VLC_ABLATE_EXP
#define VLC_ATT_EXP2(x_) (x_)
#else
#define VLC_ATT_EXP2(x_) __builtin_amdgcn_exp2f(x_)
#endif
#ifdef VLC_ABLATE_SOFTMAX_FMA   // the exponent's argument without the scale-and-subtract (one vector op per score less)
#define VLC_ATT_EXP_ARG(s_, scale_, m_) (s_)
#else
#define VLC_ATT_EXP_ARG(s_, scale_, m_) fmaf(s_, scale_, -(m_))
#endif
#ifdef VLC_ABLATE_HALF_READS    // every other K / V^T fragment read left out: each fragment read feeds two MFMAs
#define VLC_ATT_READ_NOW(i_) (((i_) & 1) == 0)
#define VLC_ATT_FRAG_BUF(i_) (((i_) >> 1) & 1)
#else
#define VLC_ATT_READ_NOW(i_) true
#define VLC_ATT_FRAG_BUF(i_) ((i_) & 1)
#endif
#ifdef VLC_ABLATE_BLOCK_BARRIER // no workgroup barrier per key block (LDS addresses do not depend on what is read)
#define VLC_ATT_BLOCK_BARRIER()
#else
#define VLC_ATT_BLOCK_BARRIER() __syncthreads()
#endif
#if defined(VLC_ABLATE_QK_MFMA) || defined(VLC_ABLATE_PV_MFMA)
__device__ __forceinline__ f32x16 ablated_mfma(bf16x8 a, bf16x8 b, f32x16 c) {   // one vector op that keeps the data flow
  c[0] += (float)a[0] * (float)b[0];
  return c;
}
#endif
#ifdef VLC_ABLATE_QK_MFMA
#define VLC_ATT_MFMA_QK(a_, b_, c_) ablated_mfma(a_, b_, c_)
#else
#define VLC_ATT_MFMA_QK(a_, b_, c_) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, b_, c_, 0, 0, 0)
#endif
#ifdef VLC_ABLATE_PV_MFMA
#define VLC_ATT_MFMA_PV(a_, b_, c_) ablated_mfma(a_, b_, c_)
#else
#define VLC_ATT_MFMA_PV(a_, b_, c_) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, b_, c_, 0, 0, 0)
#endif

// SPLIT: blockIdx.z handles the z-th share of split_blocks key blocks of each run (the last share also what
// lies beyond) and leaves an un-normalised partial (O as float, running max, running sum) for
// attention_merge_kernel; a workgroup whose share starts beyond the tile's longest row leaves at once and writes
// nothing.  Used when there are too few (row tile, kv head) pairs to occupy the chip and the key loop is the
// critical path: rows with few keys then stay whole and only the long ones are shared out.
// RT: 32-row tiles of virtual rows per wavefront.  RT = 1: 128 virtual rows per workgroup, two
// workgroups per CU.  RT = 2: 256 virtual rows, one workgroup per CU; every K and V fragment read
// from LDS then feeds two MFMAs, which halves the LDS traffic per flop (with one row tile the
// fragment reads alone would need the whole LDS bandwidth at full MFMA rate).
template <bool SPLIT, int RT>
__global__ __launch_bounds__(256, RT == 1 ? 2 : 1) void attention_bf16_kernel(
    const uint16_t* __restrict__ q, int64_t q_stride, const uint16_t* __restrict__ kc,
    const uint16_t* __restrict__ vc, const int32_t* __restrict__ row_kv_start,
    const int32_t* __restrict__ row_kv_len, int n, int Hq, int Hkv, int g, int rows_per_tile,
    float scale_log2, uint16_t* __restrict__ out, int split_blocks, float* __restrict__ part_o,
    float* __restrict__ part_ml) {
  __shared__ u32x4 lds[2 * ATT_STAGE_CHUNKS];     // 64 KB: K ring (2 tiles), then V ring (2 tiles)
  __shared__ int s_start[VR * RT];
  __shared__ int s_len[VR * RT];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, x = lane >> 5;
#ifdef VLC_ABLATE_ATT_COPIES
  // pseudo-random finite bf16 values, so that the MFMAs draw the power of a real product
  for (int i = tid; i < 2 * ATT_STAGE_CHUNKS; i += 256) {
    uint32_t h = (uint32_t)i * 2654435761u + blockIdx.x * 40503u;
    u32x4 v;
    for (int e = 0; e < 4; ++e) {
      h ^= h >> 13; h *= 0x5bd1e995u; h ^= h >> 15;
      v[e] = (h & 0x807f807fu) | 0x3f003f00u;
    }
    lds[i] = v;
  }
#endif
  // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  The remap hands every XCD
  // one contiguous range of (kv head, row tile) pairs, so the workgroups resident on an XCD at the
  // same time are neighbouring row tiles of one request and kv head and stream the same K/V.
  const int lin = blockIdx.y * gridDim.x + blockIdx.x, total = gridDim.x * gridDim.y;
  const int per = total / 8;
  const int vid = lin < per * 8 ? (lin % 8) * per + lin / 8 : lin;
  const int kvh = vid / gridDim.x;
  const int row0 = (vid - kvh * gridDim.x) * rows_per_tile;
  const int rows_here = min(rows_per_tile, n - row0);

  if (tid < rows_per_tile) {                       // rows_per_tile <= 128 * RT <= 256 threads
    const bool ok = tid < rows_here;
    s_start[tid] = ok ? row_kv_start[row0 + tid] : -1;
    s_len[tid] = ok ? row_kv_len[row0 + tid] : 0;
  }
  __syncthreads();
  if (SPLIT) {   // nothing of this tile reaches this share's first key: attention_merge_kernel will not read it
    int tile_max = 0;
    for (int r = 0; r < rows_here; ++r) tile_max = max(tile_max, s_len[r]);
    if ((int64_t)blockIdx.z * split_blocks * KB >= tile_max) return;
  }

  // this lane's virtual rows (one per row tile)
  int r_local[RT], head[RT], my_len[RT];
  bool vr_ok[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int vr = (wave * RT + rt) * 32 + l32;
    r_local[rt] = vr / g;
    head[rt] = kvh * g + (vr - r_local[rt] * g);
    vr_ok[rt] = r_local[rt] < rows_here;
    my_len[rt] = vr_ok[rt] ? s_len[r_local[rt]] : 0;
  }

  // Q fragments: Q[vr][16*ks + 8*x .. +8).  They are fetched together with the first K and V tiles of the first
  // run of rows (one memory latency instead of two, which counts when a workgroup has only a few key blocks).
  bf16x8 qf[RT][ATT_D / 16];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int ks = 0; ks < ATT_D / 16; ++ks) qf[rt][ks] = __builtin_bit_cast(bf16x8, u32x4{0u, 0u, 0u, 0u});
  bool q_loaded = false;

  f32x16 o_acc[RT][ATT_D / 32];
  float m_run[RT], l_run[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = -INFINITY;
    l_run[rt] = 0.f;
#pragma unroll
    for (int i = 0; i < ATT_D / 32; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) o_acc[rt][i][e] = 0.f;
  }

  const int64_t kv_row_elems = (int64_t)Hkv * ATT_D;

  // K and V tiles: this lane fills LDS chunks (wave*4 + i)*64 + lane, i < 4, of each tile, i.e.
  // key = chunk / 16 and the logical 8-element chunk that the tile's swizzle places there.  Its
  // byte offset from the block's first row is loop-invariant; the block base is wavefront-uniform.
  const uint32_t kv_row_bytes = (uint32_t)Hkv * ATT_D * 2;
  int t_key[4], k_c[4], v_c[4];
  uint32_t k_go[4], v_go[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int p = (wave * 4 + i) * 64 + lane;
    t_key[i] = p >> 4;
    k_c[i] = k_swz(t_key[i], p & 15);
    v_c[i] = v_swz(t_key[i], p & 15);
    k_go[i] = (uint32_t)t_key[i] * kv_row_bytes + k_c[i] * 16;
    v_go[i] = (uint32_t)t_key[i] * kv_row_bytes + v_c[i] * 16;
  }
  // K fragment reads: key 32*mt + l32, chunk (2*ks + x) ^ (key % 16); byte offset for mt = 0, stage 0
  int k_rd[ATT_D / 16];
#pragma unroll
  for (int ks = 0; ks < ATT_D / 16; ++ks) k_rd[ks] = (l32 * 16 + k_swz(l32, 2 * ks + x)) * 16;
  // transposing V reads: lane s of a 16-lane group points at key s/4, columns 4*(s%4) of the group's
  // 16-wide d range; groups 0/1 take the two d halves of a 32-wide tile, groups 0-1 / 2-3 are x = 0 / 1.
  // Byte offset for t = r = 0, stage 0, per 32-wide d tile (the swizzle term (key%4)*4 is lane-constant).
  const int tr_key = 4 * x + ((lane & 15) >> 2);                 // + 16*t + 8*r
  const int tr_d = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);      // + 32*md
  int v_rd[ATT_D / 32];
#pragma unroll
  for (int md = 0; md < ATT_D / 32; ++md) {
    const int d0 = 32 * md + tr_d;
    v_rd[md] = (tr_key * 16 + v_swz(tr_key, d0 >> 3)) * 16 + (d0 & 4) * 2;
  }

  // Rows of different requests (different row_kv_start) may share a tile: handle one run of equal
  // start at a time; lanes outside the run see every key masked.
  int seg_begin = 0;
  while (seg_begin < rows_here) {
    const int seg_start = s_start[seg_begin];
    int seg_end = seg_begin + 1;
    while (seg_end < rows_here && s_start[seg_end] == seg_start) ++seg_end;
    int seg_max = 0;
    for (int r = seg_begin; r < seg_end; ++r) seg_max = max(seg_max, s_len[r]);

    int len[RT];
    int w_max = 0, w_min = 0x7fffffff;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const bool in_seg = vr_ok[rt] && r_local[rt] >= seg_begin && r_local[rt] < seg_end;
      len[rt] = in_seg ? my_len[rt] : 0;
      w_max = max(w_max, len[rt]);
      // padding lanes (no row behind them) are left out: nothing of theirs is stored, so they need no
      // masking - otherwise the wavefront that holds the tile's padding would mask every block
      w_min = min(w_min, vr_ok[rt] ? len[rt] : 0x7fffffff);
    }
    // longest / shortest visible range among this wavefront's rows (uniform per wavefront)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      w_max = max(w_max, __shfl_xor(w_max, o));
      w_min = min(w_min, __shfl_xor(w_min, o));
    }

    const uint16_t* kbase = kc + (int64_t)seg_start * kv_row_elems + (int64_t)kvh * ATT_D;
    const uint16_t* vbase = vc + (int64_t)seg_start * kv_row_elems + (int64_t)kvh * ATT_D;
    const int all_blocks = (seg_max + KB - 1) / KB;
    int kb_first = 0, n_blocks = all_blocks;        // this workgroup's share of the run's key blocks
    if (SPLIT) {
      kb_first = min(all_blocks, (int)blockIdx.z * split_blocks);
      n_blocks = (blockIdx.z + 1 == gridDim.z ? all_blocks : min(all_blocks, kb_first + split_blocks)) - kb_first;
    }
    const int last_key = seg_max - 1;               // loads never leave the run's key range

    // LDS: K ring = chunks [0, 2*K_TILE), V ring = the next 2*V_TILE.
#define VLC_ATT_ISSUE_TILE(base_, go_, c_, kb_, lds_chunk0_)                                                   \
  {                                                                                                            \
    const int key0_ = (kb_) * KB;                                                                              \
    u32x4* dst_ = lds + (lds_chunk0_) + wave * 256;                                                            \
    if (key0_ + KB <= seg_max) { /* whole block inside the run: uniform base + invariant lane offset */        \
      const char* blk_ = reinterpret_cast<const char*>(base_) + (int64_t)key0_ * kv_row_bytes;                 \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) dma16(blk_ + go_[i], dst_ + i * 64);                       \
    } else { /* last block of the run: rows past the end re-read the last row */                               \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                                          \
        const int64_t gk_ = (int64_t)min(key0_ + t_key[i], last_key) * kv_row_elems;                           \
        dma16(base_ + gk_ + c_[i] * 8, dst_ + i * 64);                                                         \
      }                                                                                                        \
    }                                                                                                          \
  }
#define VLC_ATT_ISSUE_K(kb_, stage_) VLC_ATT_ISSUE_TILE(kbase, k_go, k_c, kb_, (stage_) * K_TILE_CHUNKS)
#define VLC_ATT_ISSUE_V(kb_, stage_) VLC_ATT_ISSUE_TILE(vbase, v_go, v_c, kb_, 2 * K_TILE_CHUNKS + (stage_) * V_TILE_CHUNKS)
    // S^T of one key block: ST[rt][mt] = K Q^T from K ring stage kst_; a K fragment serves every row tile
#define VLC_ATT_QK(ST, kst_)                                                                                   \
  {                                                                                                            \
    const unsigned char* sk_ = reinterpret_cast<const unsigned char*>(lds) + (kst_) * (K_TILE_CHUNKS * 16);    \
    _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                          \
      _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                                         \
        _Pragma("unroll") for (int e = 0; e < 16; ++e) ST[rt][mt][e] = 0.f;                                    \
    u32x4 kf_[2];   /* fragment i+1 is read while fragment i is multiplied */                                  \
    kf_[0] = VLC_ATT_KFRAG(*reinterpret_cast<const u32x4*>(sk_ + k_rd[0]));                                    \
    _Pragma("unroll") for (int i = 0; i < 2 * (ATT_D / 16); ++i) {                                             \
      const int mt = i / (ATT_D / 16), ks = i % (ATT_D / 16);                                                  \
      if (i + 1 < 2 * (ATT_D / 16) && VLC_ATT_READ_NOW(i + 1))                                                 \
        kf_[VLC_ATT_FRAG_BUF(i + 1)] = VLC_ATT_KFRAG(*reinterpret_cast<const u32x4*>(sk_ + k_rd[(i + 1) % (ATT_D / 16)] +  \
                                                                         ((i + 1) / (ATT_D / 16)) * (32 * 256))); \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                        \
        ST[rt][mt] = VLC_ATT_MFMA_QK(__builtin_bit_cast(bf16x8, kf_[VLC_ATT_FRAG_BUF(i)]), qf[rt][ks], ST[rt][mt]); \
    }                                                                                                          \
  }
    // keys of the block beyond a lane's visible range are masked (only where the block crosses it)
#define VLC_ATT_MASK(ST, key0_)                                                                                \
  {                                                                                                            \
    if ((key0_) + KB > w_min) {                                                                                \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                        \
        _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                                       \
          _Pragma("unroll") for (int j = 0; j < 16; ++j) {                                                     \
            const int key_ = (key0_) + 32 * mt + 8 * (j >> 2) + 4 * x + (j & 3);                               \
            ST[rt][mt][j] = key_ < len[rt] ? ST[rt][mt][j] : -INFINITY;                                        \
          }                                                                                                    \
    }                                                                                                          \
  }
    // online softmax (base 2) of ST: branch-free, so that it shares a basic block with the next
    // block's S^T MFMAs; leaves probabilities in ST and the rescale factors in alpha_ / grew_
#define VLC_ATT_SOFTMAX(ST)                                                                                    \
    float alpha_[RT];                                                                                          \
    bool grew_ = false;                                                                                        \
    _Pragma("unroll") for (int rt = 0; rt < RT; ++rt) {                                                        \
      float mx_ = -INFINITY;                                                                                   \
      _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                                         \
        _Pragma("unroll") for (int j = 0; j < 16; ++j) mx_ = fmaxf(mx_, ST[rt][mt][j]);                        \
      mx_ = pair_max(mx_) * scale_log2;   /* scale > 0: max commutes with it */                                \
      const float m_new_ = fmaxf(m_run[rt], mx_);                                                              \
      const float m_use_ = (m_new_ == -INFINITY) ? 0.f : m_new_;                                               \
      alpha_[rt] = __builtin_amdgcn_exp2f(m_run[rt] - m_use_);   /* m_run = -inf -> 0 */                       \
      grew_ = grew_ || (m_new_ > m_run[rt]);                                                                   \
      m_run[rt] = m_new_;                                                                                      \
      float psum_ = 0.f;                                                                                       \
      _Pragma("unroll") for (int mt = 0; mt < 2; ++mt)                                                         \
        _Pragma("unroll") for (int j = 0; j < 16; ++j) {                                                       \
          const float p_ = VLC_ATT_EXP2(VLC_ATT_EXP_ARG(ST[rt][mt][j], scale_log2, m_use_));                             \
          ST[rt][mt][j] = p_;                                                                                  \
          psum_ += p_;                                                                                         \
        }                                                                                                      \
      l_run[rt] = l_run[rt] * alpha_[rt] + psum_;                                                              \
    }
    // order template for the shared block: two K fragment reads up front, then per fragment RT MFMAs,
    // eight vector ops each, and the read of the fragment after next
#define VLC_ATT_INTERLEAVE()                                                                                   \
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                                         \
    _Pragma("unroll") for (int g_ = 0; g_ < 16; ++g_) {                                                        \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt) {                                                      \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                     \
        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);                                                     \
      }                                                                                                        \
      if (g_ < 14) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                          \
    }
    // O rescale (only when some row's maximum moved) and O^T += V^T P^T from V ring stage vst_;
    // a V^T fragment serves every row tile
#define VLC_ATT_RESCALE_PV(ST, vst_)                                                                           \
  {                                                                                                            \
    if (__any(grew_)) {                                                                                        \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                        \
        _Pragma("unroll") for (int i = 0; i < ATT_D / 32; ++i)                                                 \
          _Pragma("unroll") for (int e = 0; e < 16; ++e) o_acc[rt][i][e] *= alpha_[rt];                        \
    }                                                                                                          \
    const unsigned char* sv_ = reinterpret_cast<const unsigned char*>(lds + 2 * K_TILE_CHUNKS + (vst_) * V_TILE_CHUNKS); \
    bf16x8 pf_[RT];                                                                                            \
    s16x4 vh_[2][2];   /* V^T fragment i+1 is read while fragment i is multiplied */                           \
    _Pragma("unroll") for (int r = 0; r < 2; ++r)                                                              \
      vh_[0][r] = VLC_ATT_VFRAG(__builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)( \
          const_cast<unsigned char*>(sv_) + v_rd[0] + (8 * r) * 256)));                                        \
    _Pragma("unroll") for (int i = 0; i < 4 * (ATT_D / 32); ++i) {                                             \
      const int t = i / (ATT_D / 32), md = i % (ATT_D / 32);                                                   \
      if (i + 1 < 4 * (ATT_D / 32) && VLC_ATT_READ_NOW(i + 1)) {                                               \
        const int t1 = (i + 1) / (ATT_D / 32), md1 = (i + 1) % (ATT_D / 32);                                   \
        _Pragma("unroll") for (int r = 0; r < 2; ++r)                                                          \
          vh_[VLC_ATT_FRAG_BUF(i + 1)][r] = VLC_ATT_VFRAG(__builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)( \
              const_cast<unsigned char*>(sv_) + v_rd[md1] + (16 * t1 + 8 * r) * 256)));                        \
      }                                                                                                        \
      if (md == 0) {                                                                                           \
        _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                      \
          _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                                      \
            f32x2 pr_ = {ST[rt][t >> 1][8 * (t & 1) + 2 * e], ST[rt][t >> 1][8 * (t & 1) + 2 * e + 1]};        \
            const bf16x2 pb_ = __builtin_convertvector(pr_, bf16x2);                                           \
            pf_[rt][2 * e] = pb_[0];                                                                           \
            pf_[rt][2 * e + 1] = pb_[1];                                                                       \
          }                                                                                                    \
      }                                                                                                        \
      const s16x8 vv_ = __builtin_shufflevector(vh_[VLC_ATT_FRAG_BUF(i)][0], vh_[VLC_ATT_FRAG_BUF(i)][1], 0, 1, 2, 3, 4, 5, 6, 7); \
      _Pragma("unroll") for (int rt = 0; rt < RT; ++rt)                                                        \
        o_acc[rt][md] = VLC_ATT_MFMA_PV(__builtin_bit_cast(bf16x8, vv_), pf_[rt], o_acc[rt][md]);              \
    }                                                                                                          \
  }
    // One key block j (S^T already in CUR): fetch ahead, start the next block's S^T into NXT (its MFMAs
    // are independent of this block's softmax arithmetic, so the two interleave), finish this block.
    // The PV product runs at a raised wave priority: two wavefronts share a SIMD, and a wavefront's own vector
    // instructions do not overlap with its MFMAs, so the matrix pipe is only kept busy when one wavefront
    // multiplies while the other does its softmax arithmetic.  With equal priorities two wavefronts that reach
    // their MFMA phases together alternate instruction by instruction and stay in step; the priority lets the
    // one already in its pure-MFMA phase run ahead, which puts the pair out of step (-6 % kernel time).
#define VLC_ATT_BLOCK(j_, PAR, CUR, NXT)                                                                       \
  {                                                                                                            \
    if ((j_) + 2 < n_blocks) VLC_ATT_ISSUE_K(kb_first + (j_) + 2, PAR)                                         \
    if ((j_) + 1 < n_blocks) VLC_ATT_ISSUE_V(kb_first + (j_) + 1, (PAR) ^ 1)                                   \
    const int key0b_ = (kb_first + (j_)) * KB;                                                                 \
    if (key0b_ < w_max) { /* something visible for this wavefront in this block */                             \
      VLC_ATT_MASK(CUR, key0b_)                                                                                \
      VLC_ATT_QK(NXT, (PAR) ^ 1)   /* past the last block this reads a stale tile; the result is unused */     \
      VLC_ATT_SOFTMAX(CUR)                                                                                     \
      VLC_ATT_INTERLEAVE()                                                                                     \
      __builtin_amdgcn_s_setprio(1);   /* see below */                                                         \
      VLC_ATT_RESCALE_PV(CUR, PAR)                                                                             \
      __builtin_amdgcn_s_setprio(0);                                                                           \
    }                                                                                                          \
    VLC_ATT_WAIT_VM0();   /* this wavefront's shares of the tiles fetched above have landed */                 \
    VLC_ATT_BLOCK_BARRIER();                                                                                   \
  }

    __syncthreads();                 // the rings are free (previous run finished reading them)
    f32x16 st_a[RT][2], st_b[RT][2];
    if (n_blocks > 0) {
      VLC_ATT_ISSUE_K(kb_first, 0)
      VLC_ATT_ISSUE_V(kb_first, 0)
      if (n_blocks > 1) VLC_ATT_ISSUE_K(kb_first + 1, 1)
    }
    if (!q_loaded) {
      q_loaded = true;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        const u32x4* qp = reinterpret_cast<const u32x4*>(q + (int64_t)(row0 + (vr_ok[rt] ? r_local[rt] : 0)) * q_stride +
                                                         (int64_t)head[rt] * ATT_D);
#pragma unroll
        for (int ks = 0; ks < ATT_D / 16; ++ks)
          if (vr_ok[rt]) qf[rt][ks] = __builtin_bit_cast(bf16x8, qp[2 * ks + x]);
      }
    }
    // The Q loads are the only vector-memory reads the compiler knows of; completing them here, together with
    // this wavefront's shares of the tiles fetched above, keeps it from placing a vmcnt(0) wait (which would
    // also wait for freshly issued K/V copies) at their first use inside the key loop.
    VLC_ATT_WAIT_VM0();
    __syncthreads();
    if (n_blocks > 0 && kb_first * KB < w_max) VLC_ATT_QK(st_a, 0)
    __syncthreads();                 // K stage 0 may be refilled from here on
    for (int j = 0; j < n_blocks; j += 2) {
      VLC_ATT_BLOCK(j, 0, st_a, st_b)
      if (j + 1 < n_blocks) VLC_ATT_BLOCK(j + 1, 1, st_b, st_a)
    }
#undef VLC_ATT_ISSUE_TILE
#undef VLC_ATT_ISSUE_K
#undef VLC_ATT_ISSUE_V
#undef VLC_ATT_QK
#undef VLC_ATT_MASK
#undef VLC_ATT_SOFTMAX
#undef VLC_ATT_INTERLEAVE
#undef VLC_ATT_RESCALE_PV
#undef VLC_ATT_BLOCK
    seg_begin = seg_end;
  }

  // ---- normalise and store: lane holds d = 32*md + 8*(j/4) + 4*x + j%4 of its virtual rows ------
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const float l_tot = pair_sum(l_run[rt]);
    if (!vr_ok[rt]) continue;
    if (SPLIT) {
      const int64_t rh = ((int64_t)blockIdx.z * n + (row0 + r_local[rt])) * Hq + head[rt];
      float* po = part_o + rh * ATT_D;
#pragma unroll
      for (int md = 0; md < ATT_D / 32; ++md)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
          *reinterpret_cast<float4*>(po + 32 * md + 8 * qd + 4 * x) =
              make_float4(o_acc[rt][md][4 * qd], o_acc[rt][md][4 * qd + 1], o_acc[rt][md][4 * qd + 2],
                          o_acc[rt][md][4 * qd + 3]);
      if (x == 0) {
        part_ml[2 * rh] = m_run[rt];
        part_ml[2 * rh + 1] = l_tot;
      }
    } else {
      const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
      uint16_t* op = out + ((int64_t)(row0 + r_local[rt]) * Hq + head[rt]) * ATT_D;
#pragma unroll
      for (int md = 0; md < ATT_D / 32; ++md)
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) {
          f32x2 a0 = {o_acc[rt][md][4 * qd] * inv, o_acc[rt][md][4 * qd + 1] * inv};
          f32x2 a1 = {o_acc[rt][md][4 * qd + 2] * inv, o_acc[rt][md][4 * qd + 3] * inv};
          u32x2 w;
          w[0] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a0, bf16x2));
          w[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a1, bf16x2));
          *reinterpret_cast<u32x2*>(op + 32 * md + 8 * qd + 4 * x) = w;
        }
    }
  }
}

// Merge of the split partials: out = sum_z O_z 2^(m_z - m) / sum_z l_z 2^(m_z - m), m = max_z m_z, over the
// shares that hold keys of the row (share z starts at key block z * split_blocks; the others were not written).
// One thread per 8 output elements.
__global__ __launch_bounds__(256) void attention_merge_kernel(const float* __restrict__ part_o,
                                                              const float* __restrict__ part_ml, int max_split,
                                                              int split_blocks, const int32_t* __restrict__ row_kv_len,
                                                              int Hq, int64_t rows_heads, uint16_t* __restrict__ out) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t rh = id / (ATT_D / 8);
  const int c = (int)(id - rh * (ATT_D / 8));
  if (rh >= rows_heads) return;
  const int blocks = (row_kv_len[rh / Hq] + KB - 1) / KB;
  const int nsplit = min(max_split, (blocks + split_blocks - 1) / split_blocks);
  // all loads of a pass are issued together (max_split <= 8): running maxima and sums first, then the outputs
  constexpr int MAXZ = 8;
  float mz[MAXZ], lz[MAXZ];
#pragma unroll
  for (int z = 0; z < MAXZ; ++z) {
    mz[z] = -INFINITY;
    lz[z] = 0.f;
    if (z < nsplit) {
      const float2 ml = *reinterpret_cast<const float2*>(part_ml + 2 * (z * rows_heads + rh));
      mz[z] = ml.x;
      lz[z] = ml.y;
    }
  }
  float m = -INFINITY;
#pragma unroll
  for (int z = 0; z < MAXZ; ++z) m = fmaxf(m, mz[z]);
  float4 pa[MAXZ], pb[MAXZ];
  float wz[MAXZ];
#pragma unroll
  for (int z = 0; z < MAXZ; ++z) {
    wz[z] = mz[z] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mz[z] - m);   // -inf: this share saw no visible key
    pa[z] = pb[z] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (z < nsplit && mz[z] != -INFINITY) {
      const float4* po = reinterpret_cast<const float4*>(part_o + (z * rows_heads + rh) * ATT_D + 8 * c);
      pa[z] = po[0];
      pb[z] = po[1];
    }
  }
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
#pragma unroll
  for (int z = 0; z < MAXZ; ++z) {      // in share order, as before
    l += lz[z] * wz[z];
    acc[0] += pa[z].x * wz[z]; acc[1] += pa[z].y * wz[z]; acc[2] += pa[z].z * wz[z]; acc[3] += pa[z].w * wz[z];
    acc[4] += pb[z].x * wz[z]; acc[5] += pb[z].y * wz[z]; acc[6] += pb[z].z * wz[z]; acc[7] += pb[z].w * wz[z];
  }
  const float inv = l > 0.f ? 1.0f / l : 0.f;
  u32x4 w4;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f32x2 pr = {acc[2 * e] * inv, acc[2 * e + 1] * inv};
    w4[e] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2));
  }
  *reinterpret_cast<u32x4*>(out + rh * ATT_D + 8 * c) = w4;
}

// ---------------------------------------------------------------------------------------------
// f32 kernel: one wavefront per (row, head); lanes stride over keys with a private online softmax,
// merged across lanes at the end.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(64) void attention_f32_kernel(const float* __restrict__ q, int64_t q_stride,
                                                           const float* __restrict__ kc,
                                                           const float* __restrict__ vc,
                                                           const int32_t* __restrict__ row_kv_start,
                                                           const int32_t* __restrict__ row_kv_len, int Hq,
                                                           int Hkv, int g, float scale,
                                                           float* __restrict__ out) {
  __shared__ float sq[D];
  const int row = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
  const int kvh = head / g;
  const float* qp = q + (int64_t)row * q_stride + (int64_t)head * D;
  for (int d = lane; d < D; d += 64) sq[d] = qp[d] * scale;
  __syncthreads();
  const int len = row_kv_len[row];
  const int64_t start = row_kv_start[row];
  const int64_t kv_row = (int64_t)Hkv * D;
  float m = -INFINITY, l = 0.f;
  float acc[D];
#pragma unroll
  for (int d = 0; d < D; ++d) acc[d] = 0.f;
  for (int j = lane; j < len; j += 64) {
    const float4* kp = reinterpret_cast<const float4*>(kc + (start + j) * kv_row + (int64_t)kvh * D);
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      const float4 kv = kp[c];
      s = fmaf(kv.x, sq[4 * c], s);
      s = fmaf(kv.y, sq[4 * c + 1], s);
      s = fmaf(kv.z, sq[4 * c + 2], s);
      s = fmaf(kv.w, sq[4 * c + 3], s);
    }
    const float m_new = fmaxf(m, s);
    const float alpha = expf(m - m_new);      // m = -inf on the first key -> 0
    const float p = expf(s - m_new);
    l = l * alpha + p;
    const float4* vp = reinterpret_cast<const float4*>(vc + (start + j) * kv_row + (int64_t)kvh * D);
#pragma unroll
    for (int c = 0; c < D / 4; ++c) {
      const float4 vv = vp[c];
      acc[4 * c] = acc[4 * c] * alpha + p * vv.x;
      acc[4 * c + 1] = acc[4 * c + 1] * alpha + p * vv.y;
      acc[4 * c + 2] = acc[4 * c + 2] * alpha + p * vv.z;
      acc[4 * c + 3] = acc[4 * c + 3] * alpha + p * vv.w;
    }
    m = m_new;
  }
  // merge the 64 partial softmaxes
  float m_all = m;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, o));
  const float w = (m == -INFINITY) ? 0.f : expf(m - m_all);
  float l_all = l * w;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) l_all += __shfl_xor(l_all, o);
  const float inv = l_all > 0.f ? 1.0f / l_all : 0.f;
  float* op = out + ((int64_t)row * Hq + head) * D;
#pragma unroll
  for (int d = 0; d < D; ++d) {
    float v = acc[d] * w;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if (lane == (d & 63)) op[d] = v * inv;
  }
}

}  // namespace

int64_t attention_ws_bytes(int64_t n, int Hq, int Hkv, int D, int dtype) {
  if (dtype != VLC_BF16 || D != ATT_D || Hq % Hkv || Hq / Hkv > VR) return 0;
  const int64_t wgs = ((n + VR / (Hq / Hkv) - 1) / (VR / (Hq / Hkv))) * Hkv;
  if (wgs >= 512 || n <= 0) return 0;                  // enough workgroups without splitting
  const int64_t nsplit = 8;
  return nsplit * n * Hq * (ATT_D + 2) * 4;
}

int launch_attention(const void* q, int64_t q_stride, const void* k_cache, const void* v_cache,
                     const int32_t* row_kv_start, const int32_t* row_kv_len, int64_t n, int Hq, int Hkv,
                     int D, float scale, void* out, int dtype, void* ws, int64_t ws_bytes, int64_t max_kv_len,
                     hipStream_t st) {
  if (n <= 0) return VLC_OK;
  const int g = Hq / Hkv;
  if (dtype == VLC_BF16) {
    if (D != ATT_D) return fail(VLC_ERR_SHAPE, "attention(bf16): D=%d unsupported (128 only)", D);
    if (g > VR) return fail(VLC_ERR_SHAPE, "attention(bf16): Hq/Hkv=%d exceeds %d", g, VR);
    if (q_stride % 8) return fail(VLC_ERR_SHAPE, "attention(bf16): q row stride must be a multiple of 8");
    // 128 virtual rows per workgroup, two workgroups per CU (RT = 1).  The kernel is also written for two row
    // tiles per wavefront (RT = 2: 256 virtual rows, one workgroup per CU), which is not launched: it needs
    // more registers than a wavefront has (147 spilled) and one wavefront per SIMD overlaps nothing.
    const int rows_per_tile = VR / g;
    const int64_t tiles = (n + rows_per_tile - 1) / rows_per_tile;
    // Few workgroups (512 are resident at once, two per CU): the key loop of the longest rows is the
    // critical path, so their key range is shared out in pieces of split_blocks key blocks: as few blocks as
    // keep the grid within 1024 workgroups and 8 shares (the workspace), but at least 4 (shorter shares cost
    // more in partials and merging than they save).  Without a bound on the lengths: 8 blocks per share, the
    // last share takes the rest.
    int nsplit = 1, split_blocks = 8;
    if (ws && tiles * Hkv < 512) {
      nsplit = (int)(1024 / (tiles * Hkv));
      if (nsplit > 8) nsplit = 8;
      while (nsplit > 1 && (int64_t)nsplit * n * Hq * (ATT_D + 2) * 4 > ws_bytes) --nsplit;
      if (max_kv_len > 0) {
        const int64_t blocks = (max_kv_len + KB - 1) / KB;
        split_blocks = (int)((blocks + nsplit - 1) / nsplit);
        if (split_blocks < 4) split_blocks = 4;
        nsplit = (int)((blocks + split_blocks - 1) / split_blocks);
      }
    }
    if (nsplit > 1) {
      float* part_o = static_cast<float*>(ws);
      float* part_ml = part_o + (int64_t)nsplit * n * Hq * ATT_D;
      const dim3 grid((unsigned)tiles, (unsigned)Hkv, (unsigned)nsplit);
      hipLaunchKernelGGL((attention_bf16_kernel<true, 1>), grid, dim3(256), 0, st, (const uint16_t*)q, q_stride,
                         (const uint16_t*)k_cache, (const uint16_t*)v_cache, row_kv_start, row_kv_len, (int)n,
                         Hq, Hkv, g, rows_per_tile, scale * 1.4426950408889634f, (uint16_t*)out, split_blocks, part_o,
                         part_ml);
      VLC_CHECK_LAUNCH("attention_bf16(split)");
      const int64_t threads = n * Hq * (ATT_D / 8);
      hipLaunchKernelGGL(attention_merge_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, part_o,
                         part_ml, nsplit, split_blocks, row_kv_len, Hq, n * Hq, (uint16_t*)out);
      VLC_CHECK_LAUNCH("attention_merge");
      return VLC_OK;
    }
    const dim3 grid((unsigned)tiles, (unsigned)Hkv);
    hipLaunchKernelGGL((attention_bf16_kernel<false, 1>), grid, dim3(256), 0, st, (const uint16_t*)q, q_stride,
                       (const uint16_t*)k_cache, (const uint16_t*)v_cache, row_kv_start, row_kv_len, (int)n,
                       Hq, Hkv, g, rows_per_tile, scale * 1.4426950408889634f, (uint16_t*)out, 1, nullptr,
                       nullptr);
    VLC_CHECK_LAUNCH("attention_bf16");
    return VLC_OK;
  }
  if (dtype == VLC_F32) {
    if (n > 0x7fffffff || Hq > 65535) return fail(VLC_ERR_SHAPE, "attention(f32): grid too large");
    const dim3 grid((unsigned)n, (unsigned)Hq);
    if (D == 64)
      hipLaunchKernelGGL(attention_f32_kernel<64>, grid, dim3(64), 0, st, (const float*)q, q_stride,
                         (const float*)k_cache, (const float*)v_cache, row_kv_start, row_kv_len, Hq, Hkv, g,
                         scale, (float*)out);
    else if (D == 128)
      hipLaunchKernelGGL(attention_f32_kernel<128>, grid, dim3(64), 0, st, (const float*)q, q_stride,
                         (const float*)k_cache, (const float*)v_cache, row_kv_start, row_kv_len, Hq, Hkv, g,
                         scale, (float*)out);
    else
      return fail(VLC_ERR_SHAPE, "attention(f32): D=%d unsupported", D);
    VLC_CHECK_LAUNCH("attention_f32");
    return VLC_OK;
  }
  return fail(VLC_ERR_DTYPE, "attention: dtype=%d", dtype);
}

}  // namespace vlc

extern "C" int vlc_sparse_q_attention(const void* q, const void* k_cache, const void* v_cache,
                                      const int32_t* row_kv_start, const int32_t* row_kv_len, int64_t n,
                                      int Hq, int Hkv, int D, float scale, void* out, int dtype,
                                      void* stream) {
  using vlc::fail;
  if (dtype != VLC_F32 && dtype != VLC_BF16) return fail(VLC_ERR_DTYPE, "vlc_sparse_q_attention: dtype=%d", dtype);
  if (n < 0 || Hq <= 0 || Hkv <= 0 || Hq % Hkv || (D != 64 && D != 128))
    return fail(VLC_ERR_SHAPE, "vlc_sparse_q_attention: n=%lld Hq=%d Hkv=%d D=%d", (long long)n, Hq, Hkv, D);
  if (n == 0) return VLC_OK;
  if (!q || !k_cache || !v_cache || !row_kv_start || !row_kv_len || !out)
    return fail(VLC_ERR_NULL, "vlc_sparse_q_attention: NULL pointer");
  if (((uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)out) & 15)
    return fail(VLC_ERR_SHAPE, "vlc_sparse_q_attention: pointers must be 16-byte aligned");
  return vlc::launch_attention(q, (int64_t)Hq * D, k_cache, v_cache, row_kv_start, row_kv_len, n, Hq, Hkv, D,
                               scale, out, dtype, nullptr, 0, 0, (hipStream_t)stream);
}
