// Device scratch and device-side work-list build of the entry point that allocates nothing
// (dit_attn_varlen_fwd_noalloc): for callers that cannot call hipMalloc, such as code under HIP graph capture.
//
// The ordinary entry point builds a pack's work-list on the host, allocates a device buffer for it and copies it over
// the first time the pack is seen.  Here the list and the kernels' work counters live in one file-scope device array of
// fixed size, and the list is written by a small kernel on the caller's stream from the sequence boundaries, which
// travel as a kernel argument: no allocation, no copy, nothing that a stream capture cannot record.
//
// Every call on a GPU shares that GPU's copy of the array: calls that overlap on one GPU (two streams, two contexts,
// two threads) race.  The array keeps the last call's contents; the plan kernel rewrites every item that the next
// launch reads and clears the two work counters, so nothing is assumed about what an earlier call left.
#include "noalloc.h"

namespace dit {
namespace {

// [0, 256): the attention kernels' sync words (AttnParams::sync);  [256, 256 + 16 * kNoAllocMaxItems): the work-list.
constexpr size_t kScratchBytes = 256 + sizeof(WorkItem) * static_cast<size_t>(kNoAllocMaxItems);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// The address of this device's copy of `scratch`, per device id; filled by noalloc_init.  In host code the array's name
// is only a stand-in for the symbol, not an address a kernel can use.
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

struct PackArg {
  int32_t n_seqs;
  int32_t cu[kNoAllocMaxSeqs + 1];
};

// The list that plan_build makes on the host (sequences by descending length, ties in pack order; inside a sequence
// heads are the slow index and whole query tiles the fast one, then the ragged last tile of every head), written by
// one workgroup.
__global__ void __launch_bounds__(256) noalloc_plan_kernel(PackArg pack, int32_t n_heads, int32_t block_m, WorkItem* items,
                                                           uint32_t* sync, uint32_t n_items) {
  __shared__ int32_t order[kNoAllocMaxSeqs];
  __shared__ uint32_t first[kNoAllocMaxSeqs + 1];  // index of the first item of the i-th sequence in list order
  if (threadIdx.x == 0) {
    sync[0] = 0u;
    sync[1] = 0u;
    int32_t n = 0;
    for (int32_t i = 0; i < pack.n_seqs; ++i) {  // stable insertion sort by descending length, empty sequences dropped
      const int32_t len = pack.cu[i + 1] - pack.cu[i];
      if (len <= 0) continue;
      int32_t pos = n;
      while (pos > 0 && pack.cu[order[pos - 1] + 1] - pack.cu[order[pos - 1]] < len) {
        order[pos] = order[pos - 1];
        --pos;
      }
      order[pos] = i;
      ++n;
    }
    uint32_t acc = 0;
    for (int32_t j = 0; j < n; ++j) {
      first[j] = acc;
      const int32_t len = pack.cu[order[j] + 1] - pack.cu[order[j]];
      acc += static_cast<uint32_t>((len + block_m - 1) / block_m) * static_cast<uint32_t>(n_heads);
    }
    for (int32_t j = n; j <= kNoAllocMaxSeqs; ++j) first[j] = acc;
  }
  __syncthreads();
  for (uint32_t idx = threadIdx.x; idx < n_items; idx += blockDim.x) {
    int32_t j = 0;
    while (j + 1 < kNoAllocMaxSeqs && first[j + 1] <= idx) ++j;
    const int32_t seq = order[j];
    const int32_t start = pack.cu[seq], len = pack.cu[seq + 1] - start;
    const uint32_t whole = static_cast<uint32_t>(len / block_m);  // whole query tiles per head
    const uint32_t local = idx - first[j], n_whole = whole * static_cast<uint32_t>(n_heads);
    const int32_t head = static_cast<int32_t>(local < n_whole ? local / whole : local - n_whole);
    const int32_t m0 = static_cast<int32_t>(local < n_whole ? local % whole : whole) * block_m;
    const int32_t rows = len - m0 < block_m ? len - m0 : block_m;
    items[idx] = WorkItem{start + m0, start, len, (rows << 16) | head};
  }
}

}  // namespace

hipError_t noalloc_init(int device) {
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  if (g_scratch_ptr[device]) return hipSuccess;
  unsigned char* ptr = nullptr;
  hipError_t e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!ptr) return hipErrorInvalidSymbol;
  e = hipMemset(ptr, 0, 256);  // the work counters start at zero; set-up time, never part of a capture
  if (e != hipSuccess) return e;
  // Load the plan kernel's code now, so that the first call of the entry point finds it resident.
  hipFuncAttributes attr;
  e = hipFuncGetAttributes(&attr, reinterpret_cast<const void*>(noalloc_plan_kernel));
  if (e != hipSuccess) return e;
  g_scratch_ptr[device] = ptr;
  return hipSuccess;
}

hipError_t noalloc_plan_launch(int device, const int32_t* cu_seqlens, int32_t n_seqs, int32_t n_heads, int32_t block_m,
                               uint32_t n_items, hipStream_t stream, const WorkItem** items_out, uint32_t** sync_out) {
  if (device < 0 || device >= kMaxDevices || !g_scratch_ptr[device]) return hipErrorNotInitialized;
  if (n_seqs < 0 || n_seqs > kNoAllocMaxSeqs || n_items > static_cast<uint32_t>(kNoAllocMaxItems)) return hipErrorInvalidValue;
  unsigned char* ptr = g_scratch_ptr[device];
  PackArg pack;
  pack.n_seqs = n_seqs;
  for (int32_t i = 0; i <= kNoAllocMaxSeqs; ++i) pack.cu[i] = i <= n_seqs ? cu_seqlens[i] : cu_seqlens[n_seqs];
  WorkItem* items = reinterpret_cast<WorkItem*>(ptr + 256);
  uint32_t* sync = reinterpret_cast<uint32_t*>(ptr);
  hipLaunchKernelGGL(noalloc_plan_kernel, dim3(1), dim3(256), 0, stream, pack, n_heads, block_m, items, sync, n_items);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  *items_out = items;
  *sync_out = sync;
  return hipSuccess;
}

}  // namespace dit
