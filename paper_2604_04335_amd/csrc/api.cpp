// C ABI of the DiT denoising-step attention library: argument checks, plan cache, launch.
#include "../../include/dit_attn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "attn_fwd.h"
#include "merge.h"
#include "noalloc.h"
#include "plan.h"
#include "sp_layout.h"

namespace {

struct CachedPlan {
  std::vector<int32_t> cu;  // key: cu_seqlens contents (of the queries)
  std::vector<int32_t> cu_k;  // key: key boundaries, empty when they are the query boundaries
  int32_t n_heads = 0;
  int32_t head_dim = 0;
  dit::AttnKernel kernel = dit::AttnKernel::kIndependent128;
  int32_t n_splits = 1;  // key chunks per sequence (split-KV); part of the key
  std::vector<dit::WorkItem> host_items;
  dit::WorkItem* dev_items = nullptr;
  uint64_t last_use = 0;
  bool pinned = false;  // a launch that reads dev_items was recorded into a HIP graph: never evicted
};

constexpr size_t kMaxCachedPlans = 32;
constexpr int kMi355xComputeUnits = 256;  // what dit_attn_plan assumes when it has no device to ask
constexpr size_t kMaxItems = size_t(1) << 30;

thread_local std::string g_create_error;

}  // namespace

struct dit_attn_ctx {
  int device = 0;
  int n_cus = 0;
  uint32_t* sync = nullptr;     // device, 8 words: work counters (zero between launches) and the last launch's clock sample
  uint64_t tick = 0;
  int force_kernel = -1;        // -1: chosen per pack; else a dit::AttnKernel value (dit_attn_set_kernel)
  int last_kernel = -1;         // kernel of the last attention launch (dit_attn_last_launch_kernel)
  int max_splits = 1;           // split-KV: at most this many key chunks per sequence (dit_attn_set_split_kv); 1 = off
  float* workspace = nullptr;   // split-KV partial results and their lse
  size_t workspace_bytes = 0;
  bool workspace_pinned = false;        // a captured graph refers to `workspace`: kept until destroy when it is outgrown
  std::vector<float*> retired_workspaces;
  std::vector<std::unique_ptr<CachedPlan>> plans;
  std::string error;
};

namespace {

int fail(dit_attn_ctx* ctx, int code, const std::string& msg) {
  if (ctx) ctx->error = msg;
  return code;
}

int fail_hip(dit_attn_ctx* ctx, hipError_t e, const char* what) {
  // Clear the sticky error so that it is not reported by an unrelated later call.
  (void)hipGetLastError();
  return fail(ctx, DIT_ATTN_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t enter(int dev) {
    hipError_t e = hipGetDevice(&prev);
    if (e != hipSuccess) return e;
    if (prev != dev) {
      e = hipSetDevice(dev);
      if (e != hipSuccess) return e;
      switched = true;
    }
    return hipSuccess;
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

int check_shape_args(const int32_t* cu_seqlens, int32_t n_seqs, int32_t n_heads, int32_t head_dim, std::string& msg) {
  if (!cu_seqlens) {
    msg = "cu_seqlens is NULL";
    return DIT_ATTN_ERR_NULL;
  }
  if (head_dim != 64 && head_dim != 128) {
    msg = "head_dim must be 64 or 128, got " + std::to_string(head_dim);
    return DIT_ATTN_ERR_HEAD_DIM;
  }
  if (n_heads < 1 || n_heads > 65535) {
    msg = "n_heads must be in 1..65535, got " + std::to_string(n_heads);
    return DIT_ATTN_ERR_N_HEADS;
  }
  if (dit::plan_validate(cu_seqlens, n_seqs) != 0) {
    msg = "cu_seqlens must start at 0 and be non-decreasing, n_seqs >= 0";
    return DIT_ATTN_ERR_CU_SEQLENS;
  }
  return DIT_ATTN_OK;
}

}  // namespace

extern "C" {

const char* dit_attn_version(void) { return "dit_attn 0.1 gfx950"; }

int dit_attn_create(dit_attn_ctx** out_ctx, int device_id) {
  if (!out_ctx) {
    g_create_error = "out_ctx is NULL";
    return DIT_ATTN_ERR_NULL;
  }
  int n_dev = 0;
  hipError_t e = hipGetDeviceCount(&n_dev);
  if (e != hipSuccess || device_id < 0 || device_id >= n_dev) {
    (void)hipGetLastError();
    g_create_error = "no HIP device " + std::to_string(device_id) + " (" +
                     (e != hipSuccess ? hipGetErrorString(e) : "device count " + std::to_string(n_dev)) + ")";
    return DIT_ATTN_ERR_HIP;
  }
  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, device_id);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    g_create_error = std::string("hipGetDeviceProperties: ") + hipGetErrorString(e);
    return DIT_ATTN_ERR_HIP;
  }
  if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
    g_create_error = std::string("device is ") + prop.gcnArchName + ", this library holds gfx950 code only";
    return DIT_ATTN_ERR_HIP;
  }
  dit_attn_ctx* ctx = new (std::nothrow) dit_attn_ctx();
  if (!ctx) {
    g_create_error = "out of host memory";
    return DIT_ATTN_ERR_HIP;
  }
  ctx->device = device_id;
  ctx->n_cus = prop.multiProcessorCount;
  DeviceGuard guard;
  e = guard.enter(device_id);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&ctx->sync), 8 * sizeof(uint32_t));
  if (e == hipSuccess) e = hipMemset(ctx->sync, 0, 8 * sizeof(uint32_t));
  // Kernel code resident and LDS limits set before the first launch; this device's fixed scratch resolved.
  if (e == hipSuccess) e = dit::attn_fwd_prepare();
  if (e == hipSuccess) e = dit::noalloc_init(device_id);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    g_create_error = std::string("context set-up: ") + hipGetErrorString(e);
    if (ctx->sync) (void)hipFree(ctx->sync);
    delete ctx;
    return DIT_ATTN_ERR_HIP;
  }
  *out_ctx = ctx;
  return DIT_ATTN_OK;
}

void dit_attn_destroy(dit_attn_ctx* ctx) {
  if (!ctx) return;
  DeviceGuard guard;
  if (guard.enter(ctx->device) == hipSuccess) {
    for (auto& p : ctx->plans)
      if (p->dev_items) (void)hipFree(p->dev_items);
    if (ctx->sync) (void)hipFree(ctx->sync);
    if (ctx->workspace) (void)hipFree(ctx->workspace);
    for (float* w : ctx->retired_workspaces) (void)hipFree(w);
  }
  (void)hipGetLastError();
  delete ctx;
}

int dit_attn_set_kernel(dit_attn_ctx* ctx, int kernel) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  if (kernel < -1 || kernel > static_cast<int>(dit::AttnKernel::kPingPong256))
    return fail(ctx, DIT_ATTN_ERR_KERNEL, "kernel must be -1 (automatic), 0 (128-row) or 1 (ping-pong)");
  ctx->force_kernel = kernel;
  return DIT_ATTN_OK;
}

int dit_attn_set_split_kv(dit_attn_ctx* ctx, int max_splits) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  if (max_splits < 1 || max_splits > dit::kMaxMergeParts)
    return fail(ctx, DIT_ATTN_ERR_PARTS, "max_splits must be in 1.." + std::to_string(dit::kMaxMergeParts));
  ctx->max_splits = max_splits;
  return DIT_ATTN_OK;
}

int dit_attn_last_launch_clock(dit_attn_ctx* ctx, double* shader_mhz, double* kernel_ms) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  e = hipDeviceSynchronize();
  if (e != hipSuccess) return fail_hip(ctx, e, "hipDeviceSynchronize");
  uint64_t sample[2] = {0, 0};
  e = hipMemcpy(sample, ctx->sync + 2, sizeof(sample), hipMemcpyDeviceToHost);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipMemcpy(clock sample)");
  const double ticks = static_cast<double>(sample[1]);
  if (shader_mhz) *shader_mhz = ticks > 0 ? 100.0 * static_cast<double>(sample[0]) / ticks : 0.0;
  if (kernel_ms) *kernel_ms = ticks * 1e-5;
  return DIT_ATTN_OK;
}

int dit_attn_last_launch_kernel(const dit_attn_ctx* ctx) { return ctx ? ctx->last_kernel : -1; }

const char* dit_attn_last_error(const dit_attn_ctx* ctx) {
  return ctx ? ctx->error.c_str() : g_create_error.c_str();
}

int32_t dit_attn_plan_cache_victim(const uint64_t* last_use, const uint8_t* pinned, int32_t n) {
  if (n < 0 || (n > 0 && (!last_use || !pinned))) return -1;
  return dit::plan_cache_victim(last_use, pinned, n);
}

int64_t dit_attn_plan(const int32_t* cu_seqlens, int32_t n_seqs, int32_t n_heads, int32_t head_dim, int32_t* items,
                      int64_t capacity_items, int32_t* block_m) {
  std::string msg;
  const int rc = check_shape_args(cu_seqlens, n_seqs, n_heads, head_dim, msg);
  if (rc != DIT_ATTN_OK) return rc;
  if (capacity_items > 0 && !items) return DIT_ATTN_ERR_NULL;
  const dit::AttnKernel kernel = dit::attn_fwd_select(cu_seqlens, nullptr, n_seqs, n_heads, kMi355xComputeUnits);
  const int bm = dit::attn_fwd_block_m(kernel);
  if (block_m) *block_m = bm;
  std::vector<dit::WorkItem> list;
  try {
    dit::plan_build(cu_seqlens, n_seqs, n_heads, bm, list);
  } catch (...) {
    return DIT_ATTN_ERR_CAPACITY;
  }
  const int64_t n = static_cast<int64_t>(list.size());
  if (capacity_items > 0) {
    if (capacity_items < n) return DIT_ATTN_ERR_CAPACITY;
    if (n > 0) std::memcpy(items, list.data(), static_cast<size_t>(n) * sizeof(dit::WorkItem));
  }
  return n;
}

}  // extern "C"

namespace {

// cu_k == nullptr: self-attention (keys share the query boundaries).  lse may be nullptr.
int forward(dit_attn_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* cu_seqlens, const int32_t* cu_k,
            int32_t n_seqs, int32_t n_heads, int32_t head_dim, float scale, void* out, float* lse, void* stream) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  ctx->error.clear();
  std::string msg;
  int rc = check_shape_args(cu_seqlens, n_seqs, n_heads, head_dim, msg);
  if (rc != DIT_ATTN_OK) return fail(ctx, rc, msg);
  if (cu_k && dit::plan_validate(cu_k, n_seqs) != 0)
    return fail(ctx, DIT_ATTN_ERR_CU_SEQLENS, "cu_seqlens_k must start at 0 and be non-decreasing");
  if (!std::isfinite(scale)) return fail(ctx, DIT_ATTN_ERR_SCALE, "scale must be finite");
  const int64_t total = n_seqs > 0 ? cu_seqlens[n_seqs] : 0;
  if (n_seqs == 0 || total == 0) return DIT_ATTN_OK;
  if (!q || !k || !v || !out) return fail(ctx, DIT_ATTN_ERR_NULL, "q, k, v and out must be non-NULL");
  const uintptr_t bits = reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) |
                         reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(out);
  if (bits & 15u) return fail(ctx, DIT_ATTN_ERR_ALIGN, "q, k, v and out must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(lse) & 3u) return fail(ctx, DIT_ATTN_ERR_ALIGN, "lse must be 4-byte aligned");

  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  hipStream_t s = static_cast<hipStream_t>(stream);

  // A call that is being recorded into a HIP graph may neither allocate nor copy synchronously, and what it records
  // keeps reading the work-list (and the split-KV workspace) on every replay.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  const bool capturing = hipStreamIsCapturing(s, &cap) == hipSuccess && cap == hipStreamCaptureStatusActive;
  (void)hipGetLastError();

  // Plan cache: the same pack comes back for every DiT block of every step.
  CachedPlan* plan = nullptr;
  const size_t cu_n = static_cast<size_t>(n_seqs) + 1;
  const dit::AttnKernel kernel = ctx->force_kernel >= 0 ? static_cast<dit::AttnKernel>(ctx->force_kernel)
                                                        : dit::attn_fwd_select(cu_seqlens, cu_k, n_seqs, n_heads, ctx->n_cus);
  // Split-KV (opt-in): a pack of the 128-row kernel with fewer items than compute units cuts every sequence's keys into
  // chunks of at least four key tiles, as many as it takes to reach two items per compute unit, and merges the parts.
  int32_t n_splits = 1;
  if (ctx->max_splits > 1 && kernel == dit::AttnKernel::kIndependent128) {
    const int32_t* ck = cu_k ? cu_k : cu_seqlens;
    int64_t items = 0, min_tiles = INT64_MAX;
    for (int32_t i = 0; i < n_seqs; ++i) {
      const int64_t lq = cu_seqlens[i + 1] - cu_seqlens[i], lk = ck[i + 1] - ck[i];
      if (lq == 0 || lk == 0) continue;
      items += (lq + 127) / 128 * n_heads;
      min_tiles = std::min<int64_t>(min_tiles, (lk + 63) / 64);
    }
    if (items > 0 && items < ctx->n_cus) {
      const int64_t want = (2 * static_cast<int64_t>(ctx->n_cus) + items - 1) / items;
      const int64_t n = std::max<int64_t>(1, std::min<int64_t>({want, ctx->max_splits, min_tiles / 4}));
      // Measured on MI355X (128-row kernel, one workgroup per compute unit, head dimension 128): an unsplit call takes
      // about 10 us + 1.1 us per key tile, a call split n ways 37 us (fill and merge launches, fp32 partials, one more
      // start-up per chunk) + 1.7 / n of the unsplit time.  Split only where that is a gain: from 49 key tiles on for
      // n = 4, 68 for n = 3, 34 for n = 8.
      const double t_unsplit = 10.0 + 1.1 * static_cast<double>(min_tiles);
      if (n > 1 && t_unsplit * (1.0 - 1.7 / static_cast<double>(n)) > 37.0) n_splits = static_cast<int32_t>(n);
    }
  }
  for (auto& p : ctx->plans) {
    if (p->n_heads == n_heads && p->head_dim == head_dim && p->kernel == kernel && p->n_splits == n_splits && p->cu.size() == cu_n &&
        p->cu_k.size() == (cu_k ? cu_n : 0) && std::memcmp(p->cu.data(), cu_seqlens, cu_n * sizeof(int32_t)) == 0 &&
        (!cu_k || std::memcmp(p->cu_k.data(), cu_k, cu_n * sizeof(int32_t)) == 0)) {
      plan = p.get();
      break;
    }
  }
  if (!plan && capturing)
    return fail(ctx, DIT_ATTN_ERR_CAPTURE, "the stream is capturing and this pack has no cached work-list: call once outside the capture first");
  if (!plan) {
    std::unique_ptr<CachedPlan> np;
    try {
      np.reset(new CachedPlan());
      np->cu.assign(cu_seqlens, cu_seqlens + cu_n);
      if (cu_k) np->cu_k.assign(cu_k, cu_k + cu_n);
      np->n_heads = n_heads;
      np->head_dim = head_dim;
      np->kernel = kernel;
      np->n_splits = n_splits;
      dit::plan_build_cross(cu_seqlens, cu_k ? cu_k : cu_seqlens, n_seqs, n_heads, dit::attn_fwd_block_m(np->kernel), np->host_items,
                            n_splits);
    } catch (...) {
      return fail(ctx, DIT_ATTN_ERR_HIP, "out of host memory while building the work-list");
    }
    if (np->host_items.size() > kMaxItems) return fail(ctx, DIT_ATTN_ERR_CU_SEQLENS, "pack has too many work items");
    const size_t bytes = np->host_items.size() * sizeof(dit::WorkItem);
    e = hipMalloc(reinterpret_cast<void**>(&np->dev_items), bytes);
    if (e != hipSuccess) return fail_hip(ctx, e, "hipMalloc(work-list)");
    // Synchronous: the list may be read next by a launch on another stream than this call's.
    e = hipMemcpy(np->dev_items, np->host_items.data(), bytes, hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      (void)hipFree(np->dev_items);
      return fail_hip(ctx, e, "hipMemcpy(work-list)");
    }
    if (ctx->plans.size() >= kMaxCachedPlans) {
      // Evict the least recently used plan that no captured graph refers to (if all are pinned the cache grows).
      // hipFree waits for the device, so no kernel still reads the list.
      std::vector<uint64_t> last_use;
      std::vector<uint8_t> pinned;
      for (auto& pl : ctx->plans) {
        last_use.push_back(pl->last_use);
        pinned.push_back(pl->pinned ? 1 : 0);
      }
      const int victim = dit::plan_cache_victim(last_use.data(), pinned.data(), static_cast<int>(last_use.size()));
      if (victim >= 0) {
        (void)hipFree(ctx->plans[static_cast<size_t>(victim)]->dev_items);
        ctx->plans.erase(ctx->plans.begin() + victim);
      }
    }
    plan = np.get();
    ctx->plans.push_back(std::move(np));
  }
  plan->last_use = ++ctx->tick;
  if (capturing) plan->pinned = true;

  // Query rows of a sequence without keys: O = 0, lse = -inf (an empty sum).
  if (cu_k) {
    for (int32_t i = 0; i < n_seqs; ++i) {
      if (cu_k[i + 1] == cu_k[i] && cu_seqlens[i + 1] > cu_seqlens[i]) {
        e = dit::fill_rows_launch(out, lse, cu_seqlens[i], cu_seqlens[i + 1] - cu_seqlens[i], n_heads, head_dim, s);
        if (e != hipSuccess) return fail_hip(ctx, e, "fill kernel launch");
      }
    }
  }
  const uint32_t n_items = static_cast<uint32_t>(plan->host_items.size());
  if (n_items == 0) return DIT_ATTN_OK;
  const int64_t max_grid = static_cast<int64_t>(ctx->n_cus) * dit::attn_fwd_wgs_per_cu(plan->kernel);
  const int grid = static_cast<int>(n_items < max_grid ? n_items : max_grid);

  const int64_t total_q = cu_seqlens[n_seqs];
  if (n_splits > 1) {
    const size_t need = static_cast<size_t>(n_splits) * static_cast<size_t>(total_q) * static_cast<size_t>(n_heads) *
                        (static_cast<size_t>(head_dim) + 1) * sizeof(float);
    if (need > ctx->workspace_bytes) {
      if (capturing)
        return fail(ctx, DIT_ATTN_ERR_CAPTURE, "the stream is capturing and the split-KV workspace would have to grow: call once outside the capture first");
      if (ctx->workspace && ctx->workspace_pinned) {
        ctx->retired_workspaces.push_back(ctx->workspace);  // a captured graph still writes there on replay
        ctx->workspace_pinned = false;
      } else if (ctx->workspace) {
        (void)hipFree(ctx->workspace);  // waits for the device: no kernel still uses it
      }
      ctx->workspace = nullptr;
      ctx->workspace_bytes = 0;
      e = hipMalloc(reinterpret_cast<void**>(&ctx->workspace), need);
      if (e != hipSuccess) return fail_hip(ctx, e, "hipMalloc(split-KV workspace)");
      ctx->workspace_bytes = need;
    }
  }
  if (n_splits > 1 && capturing) ctx->workspace_pinned = true;
  float* part_out = n_splits > 1 ? ctx->workspace : nullptr;
  float* part_lse = n_splits > 1 ? ctx->workspace + static_cast<size_t>(n_splits) * total_q * n_heads * head_dim : nullptr;
  if (n_splits > 1) {
    // A sequence with fewer chunks than n_splits (or without keys) leaves parts unwritten: their weight must be 0.
    // Packs whose sequences all fill every part (the common single-shape pack) skip that launch.
    bool complete = true;
    const int32_t* ck = cu_k ? cu_k : cu_seqlens;
    for (int32_t i = 0; i < n_seqs && complete; ++i) {
      const int64_t lq = cu_seqlens[i + 1] - cu_seqlens[i], lk = ck[i + 1] - ck[i];
      if (lq == 0) continue;
      const int64_t tiles = (lk + 63) / 64, per_part = (tiles + n_splits - 1) / n_splits;
      complete = lk > 0 && (tiles + per_part - 1) / per_part == n_splits;
    }
    if (!complete) {
      e = dit::fill_neg_inf_launch(part_lse, static_cast<int64_t>(n_splits) * total_q * n_heads, s);
      if (e != hipSuccess) return fail_hip(ctx, e, "fill kernel launch");
    }
  }

  dit::AttnParams p;
  p.part_out = part_out;
  p.part_lse = part_lse;
  p.part_rows = total_q;
  p.q = q;
  p.k = k;
  p.v = v;
  p.out = out;
  p.lse = lse;
  p.items = plan->dev_items;
  p.sync = ctx->sync;
  p.n_items = n_items;
  p.n_heads = n_heads;
  p.c_log2 = std::max(std::fabs(scale) * 1.44269504088896340736f, 1e-30f);
  p.negate = scale < 0.f ? 1 : 0;
  e = dit::attn_fwd_launch(p, plan->kernel, head_dim, grid, s);
  if (e != hipSuccess) return fail_hip(ctx, e, "kernel launch");
  ctx->last_kernel = static_cast<int>(plan->kernel);
  if (n_splits > 1) {
    dit::MergeParams m{};
    for (int32_t i = 0; i < n_splits; ++i) {
      m.o[i] = part_out + static_cast<size_t>(i) * total_q * n_heads * head_dim;
      m.lse[i] = part_lse + static_cast<size_t>(i) * total_q * n_heads;
    }
    m.out = out;
    m.lse_out = lse;
    m.chunks_per_row = head_dim * 2 / 16;
    m.n_chunks = total_q * n_heads * m.chunks_per_row;
    m.in_f32 = 1;
    e = dit::merge_launch(m, n_splits, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "merge kernel launch");
  }
  return DIT_ATTN_OK;
}

}  // namespace

extern "C" {

int dit_attn_varlen_fwd(dit_attn_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                        int32_t n_seqs, int32_t n_heads, int32_t head_dim, float scale, void* out, void* stream) {
  return forward(ctx, q, k, v, cu_seqlens, nullptr, n_seqs, n_heads, head_dim, scale, out, nullptr, stream);
}

int dit_attn_varlen_fwd_lse(dit_attn_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                            int32_t n_seqs, int32_t n_heads, int32_t head_dim, float scale, void* out, float* lse,
                            void* stream) {
  if (ctx && !lse && n_seqs > 0 && cu_seqlens && cu_seqlens[n_seqs] > 0) return fail(ctx, DIT_ATTN_ERR_NULL, "lse must be non-NULL");
  return forward(ctx, q, k, v, cu_seqlens, nullptr, n_seqs, n_heads, head_dim, scale, out, lse, stream);
}

int dit_attn_cross_varlen_fwd(dit_attn_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* cu_seqlens_q,
                              const int32_t* cu_seqlens_k, int32_t n_seqs, int32_t n_heads, int32_t head_dim, float scale,
                              void* out, float* lse, void* stream) {
  if (ctx && !cu_seqlens_k) return fail(ctx, DIT_ATTN_ERR_NULL, "cu_seqlens_k is NULL");
  return forward(ctx, q, k, v, cu_seqlens_q, cu_seqlens_k, n_seqs, n_heads, head_dim, scale, out, lse, stream);
}

int dit_attn_varlen_fwd_noalloc(dit_attn_ctx* ctx, const void* q, const void* k, const void* v, const int32_t* cu_seqlens,
                                int32_t n_seqs, int32_t n_heads, int32_t head_dim, float scale, void* out, void* stream) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  ctx->error.clear();
  std::string msg;
  const int rc = check_shape_args(cu_seqlens, n_seqs, n_heads, head_dim, msg);
  if (rc != DIT_ATTN_OK) return fail(ctx, rc, msg);
  if (!std::isfinite(scale)) return fail(ctx, DIT_ATTN_ERR_SCALE, "scale must be finite");
  const int64_t total = n_seqs > 0 ? cu_seqlens[n_seqs] : 0;
  if (n_seqs == 0 || total == 0) return DIT_ATTN_OK;
  if (!q || !k || !v || !out) return fail(ctx, DIT_ATTN_ERR_NULL, "q, k, v and out must be non-NULL");
  const uintptr_t bits = reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) |
                         reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(out);
  if (bits & 15u) return fail(ctx, DIT_ATTN_ERR_ALIGN, "q, k, v and out must be 16-byte aligned");
  if (n_seqs > dit::kNoAllocMaxSeqs)
    return fail(ctx, DIT_ATTN_ERR_LIMIT, "dit_attn_varlen_fwd_noalloc takes at most " + std::to_string(dit::kNoAllocMaxSeqs) + " sequences per pack");
  const dit::AttnKernel kernel = ctx->force_kernel >= 0 ? static_cast<dit::AttnKernel>(ctx->force_kernel)
                                                        : dit::attn_fwd_select(cu_seqlens, nullptr, n_seqs, n_heads, ctx->n_cus);
  const int32_t bm = dit::attn_fwd_block_m(kernel);
  int64_t n_items = 0;
  for (int32_t i = 0; i < n_seqs; ++i) n_items += static_cast<int64_t>((cu_seqlens[i + 1] - cu_seqlens[i] + bm - 1) / bm) * n_heads;
  if (n_items > dit::kNoAllocMaxItems)
    return fail(ctx, DIT_ATTN_ERR_LIMIT, "dit_attn_varlen_fwd_noalloc takes at most " + std::to_string(dit::kNoAllocMaxItems) +
                                             " work items per pack, this pack has " + std::to_string(n_items));
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  hipStream_t s = static_cast<hipStream_t>(stream);
  dit::AttnParams p{};
  const dit::WorkItem* items = nullptr;
  e = dit::noalloc_plan_launch(ctx->device, cu_seqlens, n_seqs, n_heads, bm, static_cast<uint32_t>(n_items), s, &items, &p.sync);
  if (e != hipSuccess) return fail_hip(ctx, e, "work-list kernel launch");
  p.q = q;
  p.k = k;
  p.v = v;
  p.out = out;
  p.items = items;
  p.n_items = static_cast<uint32_t>(n_items);
  p.n_heads = n_heads;
  p.c_log2 = std::max(std::fabs(scale) * 1.44269504088896340736f, 1e-30f);
  p.negate = scale < 0.f ? 1 : 0;
  const int64_t max_grid = static_cast<int64_t>(ctx->n_cus) * dit::attn_fwd_wgs_per_cu(kernel);
  e = dit::attn_fwd_launch(p, kernel, head_dim, static_cast<int>(n_items < max_grid ? n_items : max_grid), s);
  if (e != hipSuccess) return fail_hip(ctx, e, "kernel launch");
  ctx->last_kernel = static_cast<int>(kernel);
  return DIT_ATTN_OK;
}

static int sp_layout(dit_attn_ctx* ctx, bool pack, const void* src, void* dst, int64_t n_rows, int32_t n_heads,
                     int32_t head_dim, int32_t sp_degree, void* stream) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  ctx->error.clear();
  if (head_dim != 64 && head_dim != 128) return fail(ctx, DIT_ATTN_ERR_HEAD_DIM, "head_dim must be 64 or 128");
  if (n_heads < 1 || n_heads > 65535) return fail(ctx, DIT_ATTN_ERR_N_HEADS, "n_heads must be in 1..65535");
  if (sp_degree < 1 || n_heads % sp_degree != 0)
    return fail(ctx, DIT_ATTN_ERR_N_HEADS, "sp_degree must be >= 1 and divide n_heads");
  if (n_rows < 0) return fail(ctx, DIT_ATTN_ERR_CU_SEQLENS, "n_rows must be >= 0");
  if (n_rows == 0) return DIT_ATTN_OK;
  if (!src || !dst) return fail(ctx, DIT_ATTN_ERR_NULL, "src and dst must be non-NULL");
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u)
    return fail(ctx, DIT_ATTN_ERR_ALIGN, "src and dst must be 16-byte aligned");
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  e = dit::sp_layout_launch(pack, src, dst, n_rows, n_heads, head_dim, sp_degree, ctx->n_cus, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(ctx, e, "layout kernel launch");
  return DIT_ATTN_OK;
}

int dit_attn_sp_pack_heads(dit_attn_ctx* ctx, const void* src, void* dst, int64_t n_rows, int32_t n_heads, int32_t head_dim,
                           int32_t sp_degree, void* stream) {
  return sp_layout(ctx, true, src, dst, n_rows, n_heads, head_dim, sp_degree, stream);
}

int dit_attn_sp_unpack_heads(dit_attn_ctx* ctx, const void* src, void* dst, int64_t n_rows, int32_t n_heads, int32_t head_dim,
                             int32_t sp_degree, void* stream) {
  return sp_layout(ctx, false, src, dst, n_rows, n_heads, head_dim, sp_degree, stream);
}

int dit_attn_merge(dit_attn_ctx* ctx, const void* const* o_parts, const float* const* lse_parts, int32_t n_parts,
                   int64_t total_rows, int32_t n_heads, int32_t head_dim, void* out, float* lse_out, void* stream) {
  if (!ctx) return DIT_ATTN_ERR_NULL;
  ctx->error.clear();
  if (head_dim != 64 && head_dim != 128) return fail(ctx, DIT_ATTN_ERR_HEAD_DIM, "head_dim must be 64 or 128");
  if (n_heads < 1 || n_heads > 65535) return fail(ctx, DIT_ATTN_ERR_N_HEADS, "n_heads must be in 1..65535");
  if (n_parts < 1 || n_parts > dit::kMaxMergeParts)
    return fail(ctx, DIT_ATTN_ERR_PARTS, "n_parts must be in 1.." + std::to_string(dit::kMaxMergeParts));
  if (total_rows < 0) return fail(ctx, DIT_ATTN_ERR_CU_SEQLENS, "total_rows must be >= 0");
  if (total_rows == 0) return DIT_ATTN_OK;
  if (!o_parts || !lse_parts || !out) return fail(ctx, DIT_ATTN_ERR_NULL, "o_parts, lse_parts and out must be non-NULL");
  dit::MergeParams p{};
  uintptr_t bits = reinterpret_cast<uintptr_t>(out), bits4 = reinterpret_cast<uintptr_t>(lse_out);
  for (int32_t i = 0; i < n_parts; ++i) {
    if (!o_parts[i] || !lse_parts[i]) return fail(ctx, DIT_ATTN_ERR_NULL, "a part pointer is NULL");
    p.o[i] = o_parts[i];
    p.lse[i] = lse_parts[i];
    bits |= reinterpret_cast<uintptr_t>(o_parts[i]);
    bits4 |= reinterpret_cast<uintptr_t>(lse_parts[i]);
  }
  if ((bits & 15u) || (bits4 & 3u)) return fail(ctx, DIT_ATTN_ERR_ALIGN, "o parts and out must be 16-byte, lse arrays 4-byte aligned");
  p.out = out;
  p.lse_out = lse_out;
  p.chunks_per_row = head_dim * 2 / 16;
  p.n_chunks = total_rows * n_heads * p.chunks_per_row;
  DeviceGuard guard;
  hipError_t e = guard.enter(ctx->device);
  if (e != hipSuccess) return fail_hip(ctx, e, "hipSetDevice");
  e = dit::merge_launch(p, n_parts, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(ctx, e, "merge kernel launch");
  return DIT_ATTN_OK;
}

}  // extern "C"
