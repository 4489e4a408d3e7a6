// What the matrix pipes of this chip deliver when nothing else competes: a register-only stream of
// v_mfma_f32_32x32x16_bf16, two wavefronts per SIMD on every compute unit, operands with the bit activity of the
// attention kernels' data (pseudo-random bf16 of unit scale; all-zero operands would let the chip hold its full clock,
// which real data does not).  The attention numbers are read against this figure as well as against the nominal peak.
#include "mfma_ceiling.h"

namespace dit {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

// A value in (-2, 2) with a random mantissa.
__device__ __forceinline__ __bf16 unit_scale_value(uint32_t h) {
  return (__bf16)((float)(int32_t)(h & 0xffffu) * (1.0f / 16384.0f) - 2.0f);
}

__global__ void __launch_bounds__(512) mfma_ceiling_kernel(uint64_t* sample, float* sink, int iters) {
  const uint64_t c0 = __builtin_readcyclecounter(), t0 = __builtin_amdgcn_s_memrealtime();
  const uint32_t id = blockIdx.x * 512u + threadIdx.x;
  bf16x8 a[4], b[4];
  for (int r = 0; r < 4; ++r)
    for (int i = 0; i < 8; ++i) {
      a[r][i] = unit_scale_value(mix(id * 64u + r * 8u + i));
      b[r][i] = unit_scale_value(mix(id * 64u + 32u + r * 8u + i));
    }
  f32x16 acc[4] = {};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kCeilingMfmaPerIter; ++j)
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(j >> 2) & 3], b[j & 3], acc[j & 3], 0, 0, 0);
  }
  float s = 0.f;
  for (int r = 0; r < 4; ++r)
    for (int i = 0; i < 16; ++i) s += acc[r][i];
  if (s == 123.456f) sink[threadIdx.x & 63] = s;  // never true in practice; keeps the stream from being removed
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    sample[0] = __builtin_readcyclecounter() - c0;
    sample[1] = __builtin_amdgcn_s_memrealtime() - t0;
  }
}

}  // namespace

hipError_t mfma_ceiling_launch(uint64_t* sample, float* sink, int iters, int n_cus, hipStream_t stream) {
  static_assert(kCeilingWavesPerCu == 512 / 64, "one 512-thread workgroup per compute unit");
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(n_cus), dim3(512), 0, stream, sample, sink, iters);
  return hipGetLastError();
}

}  // namespace dit
