// Launch interface between the C ABI and the gfx950 attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace dit {

struct AttnParams {
  const void* q;            // bf16 [Tq, H, D]
  const void* k;            // bf16 [Tk, H, D] (Tk = Tq and the same boundaries for self-attention)
  const void* v;
  void* out;                // bf16 [T, H, D]
  float* part_out;          // split-KV: fp32 [n_parts, Tq, H, D] workspace for normalised partial results, else nullptr;
                            // then out is not written and part_lse (fp32 [n_parts, Tq, H]) takes every part's lse
  float* part_lse;
  int64_t part_rows;        // Tq
  float* lse;               // fp32 [T, H] or nullptr: natural-log sum of exp(scale * score) of every (query row, head)
  const WorkItem* items;    // device work-list
  uint32_t* sync;           // device, 8 words (8-byte aligned): [0] items taken so far, [1] workgroups finished,
                            // [2..3] shader cycles and [4..5] 100 MHz ticks workgroup 0 of the last launch ran for.
                            // Words 0 and 1 are zero
                            // between launches: the last workgroup to finish clears them (so a launch can be
                            // replayed from a captured graph, and the host keeps no count).
  uint32_t n_items;
  int32_t n_heads;
  float c_log2;             // |scale| * log2(e), at least 1e-30: never zero, so that a masked score of -inf times it
                            // stays -inf (scale 0 then gives every live key the same weight, as it must)
  int32_t negate;           // 1 when scale < 0: the sign of Q is flipped on load
};

// Two kernels share the tile code.
//   kIndependent128: 4 wavefronts, 128 query rows per item, two unsynchronised workgroups per compute unit.
//   kPingPong256:    8 wavefronts, 256 query rows per item, one workgroup per compute unit whose two wavefront
//                    groups alternate between the matrix and the vector phase of consecutive tiles.
enum class AttnKernel : int { kIndependent128 = 0, kPingPong256 = 1 };

// Which kernel a pack runs on a device with n_cus compute units (a pure function of the pack).
// cu_seqlens_k == nullptr: keys share the query boundaries.
AttnKernel attn_fwd_select(const int32_t* cu_seqlens, const int32_t* cu_seqlens_k, int32_t n_seqs, int32_t n_heads,
                           int n_cus);

// Query rows per work item and resident workgroups per compute unit of a kernel.
int attn_fwd_block_m(AttnKernel kernel);
int attn_fwd_wgs_per_cu(AttnKernel kernel);

// Load the code of every attention kernel on the current device and set its LDS limit (a launch would otherwise do both
// the first time, which allocates; dit_attn_create calls this so that no later launch has to).
hipError_t attn_fwd_prepare();

// Enqueue the forward kernel with `grid` persistent workgroups.
hipError_t attn_fwd_launch(const AttnParams& p, AttnKernel kernel, int head_dim, int grid, hipStream_t stream);

}  // namespace dit

