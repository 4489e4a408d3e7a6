// Merge of partial attention results over disjoint key sets, and the fill of output rows that have no keys.
//
// (O_p, lse_p), p < P, are results of the same queries against disjoint key sets (sequence parallelism along the
// sequence, the ring half of the unified sequence parallelism of paper Section 5, hands every GPU one key block per
// step; split-KV does the same inside one GPU).  With lse = ln sum_p exp(lse_p):
//     O = sum_p exp(lse_p - lse) O_p.
// Elementwise and HBM bound: P * (T*H*D*2 + T*H*4) bytes in, T*H*D*2 + T*H*4 out; one thread per 16 output bytes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "merge.h"

namespace dit {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack2(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  f32x2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));  // round to nearest even
}

template <int P, bool F32>
__global__ void __launch_bounds__(256) merge_kernel(MergeParams p) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte chunk of the output
  if (e >= p.n_chunks) return;
  const int64_t rh = e / p.chunks_per_row;                    // (row, head)
  float l[P], m = -__builtin_inff();
#pragma unroll
  for (int i = 0; i < P; ++i) {
    l[i] = p.lse[i][rh];
    m = __builtin_fmaxf(m, l[i]);
  }
  const float m_safe = m == -__builtin_inff() ? 0.f : m;
  float w[P], tot = 0.f;
#pragma unroll
  for (int i = 0; i < P; ++i) {
    w[i] = __expf(l[i] - m_safe);  // exp(-inf) = 0: a part without keys has no weight
    tot += w[i];
  }
  const float inv = tot > 0.f ? 1.0f / tot : 0.f;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < P; ++i) {
    const float wi = w[i] * inv;
    float xv[8];
    if (F32) {
      typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
      const f32x4* src = reinterpret_cast<const f32x4*>(p.o[i]) + 2 * e;
      const f32x4 x0 = src[0], x1 = src[1];
      xv[0] = x0[0]; xv[1] = x0[1]; xv[2] = x0[2]; xv[3] = x0[3];
      xv[4] = x1[0]; xv[5] = x1[1]; xv[6] = x1[2]; xv[7] = x1[3];
    } else {
      const u32x4 x = reinterpret_cast<const u32x4*>(p.o[i])[e];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        xv[2 * j] = bf16_lo(x[j]);
        xv[2 * j + 1] = bf16_hi(x[j]);
      }
    }
    // a weight of exactly 0 must also silence a non-finite value of a part that had no keys
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += wi == 0.f ? 0.f : wi * xv[j];
  }
  u32x4 y;
#pragma unroll
  for (int j = 0; j < 4; ++j) y[j] = pack2(acc[2 * j], acc[2 * j + 1]);
  reinterpret_cast<u32x4*>(p.out)[e] = y;
  if (p.lse_out != nullptr && e % p.chunks_per_row == 0) p.lse_out[rh] = tot > 0.f ? m_safe + __logf(tot) : -__builtin_inff();
}

hipError_t merge_launch(const MergeParams& p, int n_parts, hipStream_t stream) {
  if (p.n_chunks == 0) return hipSuccess;
  const int64_t blocks = (p.n_chunks + 255) / 256;
  if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), block(256);
  switch (n_parts) {
    case 1:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<1, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<1, false>), grid, block, 0, stream, p);
      break;
    case 2:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<2, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<2, false>), grid, block, 0, stream, p);
      break;
    case 3:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<3, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<3, false>), grid, block, 0, stream, p);
      break;
    case 4:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<4, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<4, false>), grid, block, 0, stream, p);
      break;
    case 5:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<5, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<5, false>), grid, block, 0, stream, p);
      break;
    case 6:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<6, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<6, false>), grid, block, 0, stream, p);
      break;
    case 7:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<7, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<7, false>), grid, block, 0, stream, p);
      break;
    case 8:
      if (p.in_f32) hipLaunchKernelGGL((merge_kernel<8, true>), grid, block, 0, stream, p);
      else hipLaunchKernelGGL((merge_kernel<8, false>), grid, block, 0, stream, p);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Rows [row0, row0 + n_rows) of out (n_rows * row_chunks 16-byte chunks) := 0 and of lse := -inf: query rows of a
// sequence that has no keys.  A kernel, not a memset, so that the call can be captured into a graph.
__global__ void __launch_bounds__(256) fill_rows_kernel(u32x4* out, float* lse, int64_t chunk0, int64_t n_chunks, int64_t lse0,
                                                         int64_t n_lse) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e < n_chunks) out[chunk0 + e] = u32x4{0u, 0u, 0u, 0u};
  if (lse != nullptr && e < n_lse) lse[lse0 + e] = -__builtin_inff();
}

__global__ void __launch_bounds__(256) fill_neg_inf_kernel(float* p, int64_t n) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e < n) p[e] = -__builtin_inff();
}

hipError_t fill_neg_inf_launch(float* p, int64_t n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  const int64_t blocks = (n + 255) / 256;
  if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fill_neg_inf_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t fill_rows_launch(void* out, float* lse, int64_t row0, int64_t n_rows, int n_heads, int head_dim, hipStream_t stream) {
  if (n_rows <= 0) return hipSuccess;
  const int64_t row_chunks = (int64_t)n_heads * head_dim * 2 / 16;
  const int64_t n_chunks = n_rows * row_chunks, n_lse = n_rows * n_heads;
  const int64_t blocks = (n_chunks + 255) / 256;
  if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fill_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<u32x4*>(out), lse, row0 * row_chunks,
                     n_chunks, row0 * n_heads, n_lse);
  return hipGetLastError();
}

}  // namespace dit
