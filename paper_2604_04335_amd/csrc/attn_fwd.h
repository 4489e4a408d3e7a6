// Launch interface between the C ABI and the gfx950 attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace dit {

struct AttnParams {
  const void* q;            // bf16 [T, H, D]
  const void* k;
  const void* v;
  void* out;                // bf16 [T, H, D]
  const WorkItem* items;    // device work-list
  uint32_t* counter;        // device work counter (monotonic; see counter_base)
  uint32_t counter_base;    // value of *counter when this launch starts
  uint32_t n_items;
  int32_t n_heads;
  float c_log2;             // |scale| * log2(e)
  int32_t negate;           // 1 when scale < 0: the sign of Q is flipped on load
};

// Query rows per work item and resident workgroups per compute unit for a head dimension.
int attn_fwd_block_m(int head_dim);
int attn_fwd_wgs_per_cu(int head_dim);

// Enqueue the forward kernel with `grid` persistent workgroups.  Every workgroup takes exactly one
// counter value at or beyond n_items, so the counter ends at counter_base + n_items + grid.
hipError_t attn_fwd_launch(const AttnParams& p, int head_dim, int grid, hipStream_t stream);

}  // namespace dit
