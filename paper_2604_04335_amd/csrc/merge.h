// Launch interface of the merge and fill kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dit {

constexpr int kMaxMergeParts = 8;

struct MergeParams {
  const void* o[kMaxMergeParts];     // bf16 [T, H, D] each
  const float* lse[kMaxMergeParts];  // fp32 [T, H] each, natural log; -inf marks a part without keys for that row
  void* out;                         // bf16 [T, H, D]
  float* lse_out;                    // fp32 [T, H] or nullptr
  int64_t n_chunks;                  // T * H * D * 2 / 16
  int32_t chunks_per_row;            // D * 2 / 16: 16-byte chunks of one (row, head)
};

hipError_t merge_launch(const MergeParams& p, int n_parts, hipStream_t stream);

// out rows [row0, row0 + n_rows) := 0, lse (if not nullptr) := -inf.
hipError_t fill_rows_launch(void* out, float* lse, int64_t row0, int64_t n_rows, int n_heads, int head_dim, hipStream_t stream);

}  // namespace dit
