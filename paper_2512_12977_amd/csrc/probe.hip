// Measurement aid for the roofline discussion (no part of the method): a register-only MFMA loop.
// Every wavefront keeps four independent 32x32 accumulators and issues v_mfma_f32_32x32x16_bf16 back to back on
// operands it loaded once, so nothing but the matrix pipe (and the clock the chip sustains under that load) limits it.
// With operands of random bits the power draw - and with it the clock - is that of a real GEMM; with constant
// operands it is lower.  The rate a kernel reaches is set against this figure beside the published peak.
#include <hip/hip_runtime.h>

#include "vlc_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kProbeMfmaPerIter = 8;

__global__ __launch_bounds__(512) void mfma_probe_kernel(const u32x4* __restrict__ operands, float* __restrict__ out,
                                                         int iters) {
  // 128 chunks of 16 bytes per wavefront slot: A and B fragments of this lane
  const int slot = (blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) & 63, lane = threadIdx.x & 63;
  const bf16x8 a = __builtin_bit_cast(bf16x8, operands[slot * 128 + lane]);
  const bf16x8 b = __builtin_bit_cast(bf16x8, operands[slot * 128 + 64 + lane]);
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kProbeMfmaPerIter; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) s += acc[j][lane & 15];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace

extern "C" int vlc_probe_mfma_bf16(const void* operands, int64_t operand_bytes, float* out, int64_t out_elems,
                                   int iters, int waves_per_simd, double* flops, void* stream) {
  using vlc::fail;
  if (!operands || !out || !flops) return fail(VLC_ERR_NULL, "vlc_probe_mfma_bf16: NULL pointer");
  if (iters <= 0 || (waves_per_simd != 1 && waves_per_simd != 2))
    return fail(VLC_ERR_SHAPE, "vlc_probe_mfma_bf16: iters=%d waves_per_simd=%d (1 or 2)", iters, waves_per_simd);
  int dev = 0, cus = 0;
  VLC_CHECK_HIP(hipGetDevice(&dev));
  VLC_CHECK_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int threads = 256 * waves_per_simd;
  if (operand_bytes < 64 * 128 * 16 || out_elems < (int64_t)cus * threads)
    return fail(VLC_ERR_SHAPE, "vlc_probe_mfma_bf16: operands of %lld bytes (131072 needed), out of %lld floats (%lld needed)",
                (long long)operand_bytes, (long long)out_elems, (long long)cus * threads);
  if ((uintptr_t)operands & 15) return fail(VLC_ERR_SHAPE, "vlc_probe_mfma_bf16: operands must be 16-byte aligned");
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(cus), dim3(threads), 0, (hipStream_t)stream,
                     static_cast<const u32x4*>(operands), out, iters);
  VLC_CHECK_LAUNCH("mfma_probe");
  *flops = (double)cus * (threads / 64) * (double)iters * kProbeMfmaPerIter * (2.0 * 32 * 32 * 16);
  return VLC_OK;
}
