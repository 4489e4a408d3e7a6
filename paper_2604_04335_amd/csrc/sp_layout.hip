// Single-GPU halves of the head-split sequence-parallel all-to-all (paper Section 4.3 elastic sequence parallelism,
// Section 5 unified sequence parallelism): pure index maps over 16-byte chunks, HBM bound.
//     pack    [n, H, D] -> [p, n, H/p, D]     send[g, r, h, :] = x[r, g*H/p + h, :]
//     unpack  [p, n, H/p, D] -> [n, H, D]     y[r, g*H/p + h, :] = recv[g, r, h, :]
// One thread per 16 bytes; consecutive threads walk the DESTINATION contiguously, and the source of a run of
// (H/p)*D*2 bytes is contiguous too, so both sides are coalesced.  Traffic: every byte read once and written once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sp_layout.h"

namespace dit {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// group_chunks: 16-byte chunks of one (row, head group) = (H/p) * D * 2 / 16.
template <bool PACK>
__global__ void __launch_bounds__(256) sp_layout_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n_rows,
                                                        int32_t p, int32_t group_chunks) {
  const int64_t total = n_rows * p * group_chunks;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int64_t c = e % group_chunks;
    const int64_t t = e / group_chunks;
    if (PACK) {  // e walks dst = [g][r][c]; src = [r][g][c]
      const int64_t r = t % n_rows, g = t / n_rows;
      dst[e] = src[(r * p + g) * group_chunks + c];
    } else {     // e walks dst = [r][g][c]; src = [g][r][c]
      const int64_t g = t % p, r = t / p;
      dst[e] = src[(g * n_rows + r) * group_chunks + c];
    }
  }
}

hipError_t sp_layout_launch(bool pack, const void* src, void* dst, int64_t n_rows, int n_heads, int head_dim, int sp_degree,
                            int n_cus, hipStream_t stream) {
  const int32_t group_chunks = (n_heads / sp_degree) * head_dim * 2 / 16;
  const int64_t total = n_rows * sp_degree * group_chunks;
  if (total == 0) return hipSuccess;
  int64_t blocks = (total + 255) / 256;
  const int64_t cap = (int64_t)n_cus * 16;  // grid-stride: enough workgroups to fill the chip, no more
  if (blocks > cap) blocks = cap;
  if (pack)
    hipLaunchKernelGGL(sp_layout_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<const u32x4*>(src),
                       static_cast<u32x4*>(dst), n_rows, sp_degree, group_chunks);
  else
    hipLaunchKernelGGL(sp_layout_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<const u32x4*>(src),
                       static_cast<u32x4*>(dst), n_rows, sp_degree, group_chunks);
  return hipGetLastError();
}

}  // namespace dit
