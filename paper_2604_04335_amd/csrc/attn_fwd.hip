// DiT denoising-step self-attention forward for gfx950 (MI355X): the 128-row and the ping-pong kernel, and the launch
// interface.  The tile code they share (and its description) is in attn_device.h.
#include "attn_device.h"

namespace dit {

// ---------------------------------------------------------------------------------------------
// Kernel A: 4 wavefronts, 128 query rows per workgroup, two independent workgroups per compute unit.
// Per tile every wave runs QK, softmax, PV back to back; the two workgroups of a CU overlap each
// other's matrix and vector work without synchronising.  One barrier per tile.
// ---------------------------------------------------------------------------------------------
template <class T>
__global__ void __attribute__((amdgpu_flat_work_group_size(T::NT, T::NT), amdgpu_waves_per_eu(2, 2)))
attn_fwd_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char* smem = (lds_char*)smem_generic;
  volatile uint32_t* s_item = reinterpret_cast<volatile uint32_t*>(smem_generic + T::ITEM_OFF);

  const LaunchClock clock0 = launch_clock_begin();
  const int tid = threadIdx.x;
  const int64_t row_stride_b = (int64_t)p.n_heads * T::D * 2;
  const float c = p.c_log2;
  Lane<T> L;
  L.init(tid, row_stride_b);

  // The index of the next item is requested towards the end of an item, into the slot of the other parity; a barrier
  // between that write and the end of the item makes it visible to every wave before it is read.
  if (tid == 0) s_item[0] = blockIdx.x;
  wg_barrier();
  int par = 0;

  for (;;) {
    const uint32_t item_idx = __builtin_amdgcn_readfirstlane(s_item[par]);
    if (item_idx >= p.n_items) break;
    par ^= 1;  // the next index goes to s_item[par], see below
    const ItemCtx<T> X = begin_item<T>(p, L, item_idx, row_stride_b);
    const int kv_len = X.it.kv_len, nt = X.nt;

    auto load_tile = [&](int ti) {  // K(ti), V(ti) -> buffers of parity ti&1
      tile_load_one<T>(X.kbase, row_stride_b, tile_first_key<T>(ti, kv_len), kv_len, L.lrow, L.kcol, L.kvoff, smem, T::K_OFF + (ti & 1) * T::TILE_B, L.wave);
      tile_load_one<T>(X.vbase, row_stride_b, tile_first_key<T>(ti, kv_len), kv_len, L.lrow, L.vcol, L.vvoff, smem, T::V_OFF + (ti & 1) * T::TILE_B, L.wave);
    };
    load_tile(0);

    bf16x8 qf[T::NKS];
    load_q<T>(p, L, X.it, row_stride_b, X.head_off, X.qrow, qf);

    f32x16 o[T::NDB];
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m_ref = -1.0e30f;  // finite, so that (m_ref - m) * 0 is 0 when scale is 0
    float l_run = 0.f;
    f32x16 s[T::NKB];
    uint32_t pb[T::NKB][8];
    int ka[T::NKS], va[T::NDB];  // operand addresses in the buffers of the current tile's parity
    L.operand_addrs((uint32_t)(uintptr_t)smem, (uint32_t)(uintptr_t)smem, ka, va);

    if (nt == 1 && tid == 0) s_item[par] = take_item(p);  // visible after the barrier below
    for (int t = 0; t + 1 < nt; ++t) {
      // Tile t has landed (this wave's loads), and after the barrier everyone's; everyone is also done
      // reading the other buffers (tile t-1), so they can be refilled with tile t+1 while tile t is used.
      wait_loads();
      wg_barrier();
      if (t + 2 == nt && tid == 0) s_item[par] = take_item(p);  // visible after the barrier of the last tile
      load_tile(t + 1);
      mfma_stream<T, false, 0, T::NQK, kPrefetch>(smem, va, ka, pb, qf, o, s);
      tile_softmax<T, false>(s, L.hh, TailRows{0, T::BN}, c, pb, o, m_ref, l_run);
      mfma_stream<T, true, 0, 0, kPrefetch>(smem, va, ka, pb, qf, o, s);
#pragma unroll
      for (int ks = 0; ks < T::NKS; ++ks) ka[ks] ^= T::TILE_B;
#pragma unroll
      for (int db = 0; db < T::NDB; ++db) va[db] ^= T::TILE_B;
    }
    // The last tile (masked), outside the loop: one copy of each softmax variant, no test per tile.
    wait_loads();
    wg_barrier();
    mfma_stream<T, false, 0, T::NQK, kPrefetch>(smem, va, ka, pb, qf, o, s);
    tile_softmax<T, true>(s, L.hh, tail_rows<T>(kv_len), c, pb, o, m_ref, l_run);
    mfma_stream<T, true, 0, 0, kPrefetch>(smem, va, ka, pb, qf, o, s);

    store_out<T>(p, L, X.it, row_stride_b, X.head_off, X.qrow, X.row_valid, o, l_run, m_ref);
    wg_barrier();  // the next item's first loads overwrite the buffers of parity 0
  }
  launch_clock_end(p, clock0);
  if (tid == 0) finish_workgroup(p);
}

// ---------------------------------------------------------------------------------------------
// Kernel B (ping-pong): 8 wavefronts, 256 query rows per workgroup, one workgroup per compute unit.
//
// Wavefronts w and w+4 share a SIMD.  Group 0 (waves 0-3) and group 1 (waves 4-7) run the same
// per-tile program  softmax(t) | PV(t) + QK(t+1)  but one phase apart, with a workgroup barrier
// after every phase: while one group keeps the matrix pipe busy (32 MFMAs), the other does its
// softmax on the vector ALU.  Phase p of an item (p = 0 after the first barrier):
//     group 0:  QK(0) at p=0,  softmax(t) at p=2t+1,  PV(t)+QK(t+1) at p=2t+2
//     group 1:  idle  at p=0,  QK(0) at p=1, softmax(t) at p=2t+2, PV(t)+QK(t+1) at p=2t+3
// K(t+1) and V(t) are therefore read in phases 2t+2 and 2t+3 only; their buffers (parity of the
// tile index) are refilled with K(t+3) / V(t+2) from phase 2t+4 on.  The pair {K(t+2), V(t+1)} is
// issued at the start of phase 2t+2 by group 1, which is then in its vector phase, for both groups
// (measured: +10 % over each group loading its own share, because a wavefront in its matrix phase is
// the critical path), and awaited by group 1 at the end of phase 2t+3, before the barrier that lets
// group 0 read it.
// ---------------------------------------------------------------------------------------------
template <class T>
__global__ void __attribute__((amdgpu_flat_work_group_size(T::NT, T::NT), amdgpu_waves_per_eu(2, 2)))
attn_fwd_pp_kernel(AttnParams p) {
  static_assert(T::NWAVES == 8, "two groups of four wavefronts");
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char* smem = (lds_char*)smem_generic;
  volatile uint32_t* s_item = reinterpret_cast<volatile uint32_t*>(smem_generic + T::ITEM_OFF);

  const LaunchClock clock0 = launch_clock_begin();
  const int tid = threadIdx.x;
  const int64_t row_stride_b = (int64_t)p.n_heads * T::D * 2;
  const float c = p.c_log2;
  Lane<T> L;
  L.init(tid, row_stride_b);
  const int group = L.wave >> 2;

  // The index of the next item is requested towards the end of an item, into the slot of the other parity; a barrier
  // between that write and the end of the item makes it visible to every wave before it is read.
  if (tid == 0) s_item[0] = blockIdx.x;
  wg_barrier();
  int par = 0;

  for (;;) {
    const uint32_t item_idx = __builtin_amdgcn_readfirstlane(s_item[par]);
    if (item_idx >= p.n_items) break;
    par ^= 1;  // the next index goes to s_item[par], see below
    const ItemCtx<T> X = begin_item<T>(p, L, item_idx, row_stride_b);
    const int kv_len = X.it.kv_len, nt = X.nt;

    auto load_k = [&](int ti) {  // K(ti) -> K buffer of parity ti&1
      tile_load_one<T>(X.kbase, row_stride_b, tile_first_key<T>(ti, kv_len), kv_len, L.lrow, L.kcol, L.kvoff, smem, T::K_OFF + (ti & 1) * T::TILE_B, L.wave);
    };
    auto load_v = [&](int ti) {  // V(ti) -> V buffer of parity ti&1
      tile_load_one<T>(X.vbase, row_stride_b, tile_first_key<T>(ti, kv_len), kv_len, L.lrow, L.vcol, L.vvoff, smem, T::V_OFF + (ti & 1) * T::TILE_B, L.wave);
    };
    auto load_pair = [&](int t) {  // what phases 2t+2 / 2t+3 read: K(t+1) and V(t)
      if (t + 1 < nt) load_k(t + 1);
      load_v(t);
    };

    // Inside the tile loop group 1 issues the loads of both groups (its own rows and those of wave-4) at the start of
    // its vector phase: the wavefronts that are in their matrix phase issue nothing but MFMAs and operand reads.
    auto load_pair_all = [&](int t) {
      load_pair(t);
      const int w2 = L.wave - 4;
      const int lrow2 = L.lrow - 4 * T::RPI;
      const uint32_t d = (uint32_t)(4 * T::RPI) * (uint32_t)row_stride_b;
      if (t + 1 < nt) tile_load_one<T>(X.kbase, row_stride_b, tile_first_key<T>(t + 1, kv_len), kv_len, lrow2, L.kcol, L.kvoff - d, smem, T::K_OFF + ((t + 1) & 1) * T::TILE_B, w2);
      tile_load_one<T>(X.vbase, row_stride_b, tile_first_key<T>(t, kv_len), kv_len, lrow2, L.vcol, L.vvoff - d, smem, T::V_OFF + (t & 1) * T::TILE_B, w2);
    };
    load_k(0);
    load_pair(0);

    bf16x8 qf[T::NKS];
    load_q<T>(p, L, X.it, row_stride_b, X.head_off, X.qrow, qf);

    f32x16 o[T::NDB];
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m_ref = -1.0e30f;  // finite, so that (m_ref - m) * 0 is 0 when scale is 0
    float l_run = 0.f;
    f32x16 s[T::NKB];
    uint32_t pb[T::NKB][8];
    int ka[T::NKS], va[T::NDB];  // ka: K buffer the next QK reads; va: V buffer the next PV reads
    L.operand_addrs((uint32_t)(uintptr_t)smem, (uint32_t)(uintptr_t)smem, ka, va);

    wait_loads();
    wg_barrier();                  // K(0), K(1), V(0) of every wave have landed; phase 0 starts
    if (group == 1) wg_barrier();  // group 1 idles in phase 0
    mfma_stream<T, false, 0, T::NQK, kPrefetch>(smem, va, ka, pb, qf, o, s);  // QK(0)
#pragma unroll
    for (int ks = 0; ks < T::NKS; ++ks) ka[ks] ^= T::TILE_B;
    wg_barrier();

    if (nt == 1 && tid == 0) s_item[par] = take_item(p);  // two barriers follow in the last tile
    for (int t = 0; t + 1 < nt; ++t) {
      // ---- vector phase: softmax(t), a full tile
      if (t + 2 == nt && tid == 0) s_item[par] = take_item(p);
      if (group == 1) load_pair_all(t + 1);
      tile_softmax<T, false>(s, L.hh, TailRows{0, T::BN}, c, pb, o, m_ref, l_run);
      wg_barrier();
      // ---- matrix phase: PV(t), QK(t+1)
      __builtin_amdgcn_s_setprio(1);
      mfma_stream<T, true, 0, T::NQK, kPrefetch>(smem, va, ka, pb, qf, o, s);
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int ks = 0; ks < T::NKS; ++ks) ka[ks] ^= T::TILE_B;
#pragma unroll
      for (int db = 0; db < T::NDB; ++db) va[db] ^= T::TILE_B;
      if (group == 1) wait_loads();  // pair t+1, issued at the start of this group's softmax(t)
      wg_barrier();
    }
    // ---- last tile: masked softmax, PV only
    tile_softmax<T, true>(s, L.hh, tail_rows<T>(kv_len), c, pb, o, m_ref, l_run);
    wg_barrier();
    __builtin_amdgcn_s_setprio(1);
    mfma_stream<T, true, 0, 0, kPrefetch>(smem, va, ka, pb, qf, o, s);
    __builtin_amdgcn_s_setprio(0);
    wg_barrier();

    store_out<T>(p, L, X.it, row_stride_b, X.head_off, X.qrow, X.row_valid, o, l_run, m_ref);
    if (group == 0) wg_barrier();  // group 0 idles (after its stores) while group 1 runs its last matrix phase
  }
  launch_clock_end(p, clock0);
  if (tid == 0) finish_workgroup(p);
}

template <class T, void (*KERNEL)(AttnParams)>
static hipError_t launch_t(const AttnParams& p, int grid, hipStream_t stream) {
  static bool attr_set[16] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16 || !attr_set[dev]) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(KERNEL), hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 16) attr_set[dev] = true;
  }
  hipLaunchKernelGGL(KERNEL, dim3(grid), dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

int attn_fwd_block_m(AttnKernel kernel) { return kernel == AttnKernel::kIndependent128 ? 128 : 256; }
int attn_fwd_wgs_per_cu(AttnKernel kernel) { return kernel == AttnKernel::kIndependent128 ? 2 : 1; }

AttnKernel attn_fwd_select(const int32_t* cu_seqlens, const int32_t* cu_seqlens_k, int32_t n_seqs, int32_t n_heads,
                           int n_cus) {
  // Measured on MI355X with equal-length sequences (time of the 128-row kernel over the ping-pong kernel, by 256-row
  // items per compute unit): 0.5: 0.91;  0.75: 1.19;  0.94: 1.17;  1.0: 1.12;  1.25: 0.90;  1.5: 0.95;  1.6: 1.05;
  // 1.9: 1.10;  2.0: 1.10;  2.5: 0.96;  3.0: 1.15;  3.2: 1.02;  4 and more: 1.05-1.09.  The ping-pong kernel is ahead
  // whenever its items fill the compute units; the 128-row kernel, whose items are half as long, when there is well
  // under one 256-row item per compute unit or when the last round of 256-row items would be less than half full.
  // Items with few key tiles (cross-attention against a few hundred text keys) also run better on the 128-row kernel,
  // whose workgroups have no idle phase at the ends of an item: 128 keys +17 %, 256 +9 %, 512 +3 %, 1024 -4 %.  (Packs
  // of short self-attention sequences do not follow: 256 and 512 tokens -2 %, 640 +4 %, 768 -4 %; they stay as they are.)
  // Of the 256-row kernels the ping-pong one is ahead of the wide one at every sequence length once the chip has
  // warmed up (6-10 % at head dimension 128, 0-4 % at 64); measured on a cold chip, in the first ~20 ms after idle,
  // whichever kernel runs second looks faster.
  const int32_t* ck = cu_seqlens_k ? cu_seqlens_k : cu_seqlens;
  int64_t items256 = 0, tiles = 0;
  for (int32_t i = 0; i < n_seqs; ++i) {
    const int64_t lq = cu_seqlens[i + 1] - cu_seqlens[i], lk = ck[i + 1] - ck[i];
    if (lq == 0 || lk == 0) continue;
    const int64_t it = (lq + 255) / 256 * n_heads;
    items256 += it;
    tiles += it * ((lk + 63) / 64);
  }
  if (items256 * 8 < (int64_t)n_cus * 5) return AttnKernel::kIndependent128;
  if (cu_seqlens_k != nullptr && tiles <= 10 * items256) return AttnKernel::kIndependent128;
  const int64_t in_last_round = items256 % n_cus;
  if (items256 <= 3 * (int64_t)n_cus && in_last_round != 0 && 2 * in_last_round <= n_cus) return AttnKernel::kIndependent128;
  return AttnKernel::kPingPong256;
}

hipError_t attn_fwd_launch(const AttnParams& p, AttnKernel kernel, int head_dim, int grid, hipStream_t stream) {
  if (kernel == AttnKernel::kWide256 && !p.negate) return attn_fwd_wide_launch(p, head_dim, grid, stream);
  if (kernel != AttnKernel::kIndependent128) {
    if (head_dim == 128) return launch_t<Tile<128, 8, 64>, attn_fwd_pp_kernel<Tile<128, 8, 64>>>(p, grid, stream);
    if (head_dim == 64) return launch_t<Tile<64, 8, 64>, attn_fwd_pp_kernel<Tile<64, 8, 64>>>(p, grid, stream);
  } else {
    if (head_dim == 128) return launch_t<Tile<128, 4, 64>, attn_fwd_kernel<Tile<128, 4, 64>>>(p, grid, stream);
    if (head_dim == 64) return launch_t<Tile<64, 4, 64>, attn_fwd_kernel<Tile<64, 4, 64>>>(p, grid, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace dit
