// Interface of the fixed device scratch behind dit_attn_varlen_fwd_noalloc (see noalloc.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.h"

namespace dit {

constexpr int32_t kNoAllocMaxSeqs = 64;       // sequences per pack (their boundaries travel as a kernel argument)
constexpr int32_t kNoAllocMaxItems = 16384;   // work items per pack: 256 KB of work-list in the device array

// Once per device, with that device current (dit_attn_create calls it): resolves the address of this device's copy of
// the scratch array, clears the work counters and loads the plan kernel.  Repeated calls are no-ops.
hipError_t noalloc_init(int device);

// Enqueues on `stream` the kernel that writes the work-list of this pack (block_m query rows per item; n_items as
// counted by the caller) into the device's scratch and clears the work counters there; returns the device addresses of
// the list and of the sync words for the attention launch that follows on the same stream.  Allocates nothing.
// cu_seqlens: host, n_seqs + 1 entries, validated by the caller.  n_seqs <= kNoAllocMaxSeqs, n_items <= kNoAllocMaxItems.
hipError_t noalloc_plan_launch(int device, const int32_t* cu_seqlens, int32_t n_seqs, int32_t n_heads, int32_t block_m,
                               uint32_t n_items, hipStream_t stream, const WorkItem** items_out, uint32_t** sync_out);

}  // namespace dit
