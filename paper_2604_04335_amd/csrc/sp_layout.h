// Launch interface of the sequence-parallel layout kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dit {

// pack: [n_rows, H, D] -> [p, n_rows, H/p, D]; !pack: the inverse.  bf16 elements, 16-byte aligned buffers.
hipError_t sp_layout_launch(bool pack, const void* src, void* dst, int64_t n_rows, int n_heads, int head_dim, int sp_degree,
                            int n_cus, hipStream_t stream);

}  // namespace dit
