// Launch interface of the merge and fill kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dit {

constexpr int kMaxMergeParts = 8;

struct MergeParams {
  const void* o[kMaxMergeParts];     // bf16 [T, H, D] each (fp32 if in_f32)
  const float* lse[kMaxMergeParts];  // fp32 [T, H] each, natural log; -inf marks a part without keys for that row
  void* out;                         // bf16 [T, H, D]
  float* lse_out;                    // fp32 [T, H] or nullptr
  int64_t n_chunks;                  // T * H * D * 2 / 16
  int32_t chunks_per_row;            // D * 2 / 16: 16-byte chunks of one (row, head)
  int32_t in_f32;                    // parts are fp32 (split-KV workspace) instead of bf16
};

hipError_t merge_launch(const MergeParams& p, int n_parts, hipStream_t stream);

// out rows [row0, row0 + n_rows) := 0, lse (if not nullptr) := -inf.
// n floats at p := -inf (a kernel, so that it can be captured into a graph).
hipError_t fill_neg_inf_launch(float* p, int64_t n, hipStream_t stream);

hipError_t fill_rows_launch(void* out, float* lse, int64_t row0, int64_t n_rows, int n_heads, int head_dim, hipStream_t stream);

}  // namespace dit
