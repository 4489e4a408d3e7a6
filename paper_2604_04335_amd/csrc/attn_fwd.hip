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
  lds_slot* s_item = reinterpret_cast<lds_slot*>(smem + T::ITEM_OFF);

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
    float m_ref = -1.0e30f;  // finite: (m_ref - m) * c stays finite
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
      // The next index is requested here and put into its slot at the end of the tile (visible after the barrier of
      // the last tile): the request takes about a microsecond to come back, which thread 0's wavefront spends on
      // the tile instead of waiting.
      const bool ask = t + 2 == nt && tid == 0;
      uint32_t next_item = 0;
      if (ask) next_item = take_item(p);
      load_tile(t + 1);
      mfma_stream<T, false, 0, T::NQK, kPrefetch>(smem, va, ka, pb, qf, o, s);
      tile_softmax<T, false>(s, L.hh, TailRows{0, T::BN}, c, pb, o, m_ref, l_run);
      mfma_stream<T, true, 0, 0, kPrefetch>(smem, va, ka, pb, qf, o, s);
      if (ask) s_item[par] = next_item;
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

    // The rows are staged in the buffers of the parity that the last tile does not use: every wavefront is done with
    // tile nt - 2 (the barrier of the last tile), nothing is being loaded there, and the next item's loads come after
    // the barrier below.  Wavefronts 0, 1 take the K buffer of that parity, wavefronts 2, 3 the V buffer.
    const uint32_t stage = (uint32_t)(uintptr_t)smem + (L.wave < 2 ? T::K_OFF : T::V_OFF) + (nt & 1) * T::TILE_B +
                           (uint32_t)(L.wave & 1) * (32 * T::ROW_B);
    store_out<T>(p, L, X.it, row_stride_b, X.head_off, X.qrow, X.row_valid, o, l_run, m_ref, stage);
    wg_barrier();  // the next item's first loads overwrite the buffers of parity 0
  }
  launch_clock_end(p, clock0);
  if (tid == 0) finish_workgroup(p);
}

// ---------------------------------------------------------------------------------------------
// Kernel B (ping-pong): 8 wavefronts, 256 query rows per workgroup, one workgroup per compute unit.
//
// Wavefronts w and w+4 share a SIMD.  Group 0 (waves 0-3) and group 1 (waves 4-7) run the same program one phase
// apart, with a workgroup barrier after every phase: while one group keeps the matrix pipe busy, the other does its
// softmax on the vector ALU.  A phase works through a PAIR of consecutive 64-key tiles (a K / V buffer holds a pair):
// half as many barriers and MFMA-stream start-ups per key as one tile per phase, which was worth 14 % fewer cycles per
// key.  The softmax stays per tile (one reference decision per row and 64 keys, exactly as in the 128-row kernel), so
// both kernels produce the same bits; the second tile's rescale of O^T, which in a tile-by-tile pass happens after the
// first tile's PV MFMAs, is deferred into the matrix phase (pp_stream).  With P(t) the pair of tiles 2t, 2t+1, phase p
// of an item (p = 0 after the first barrier):
//     group 0:  QK(P0) at p=0,  softmax(Pt) at p=2t+1,  PV(Pt)+QK(Pt+1) at p=2t+2
//     group 1:  idle   at p=0,  QK(P0) at p=1, softmax(Pt) at p=2t+2, PV(Pt)+QK(Pt+1) at p=2t+3
// K(Pt+1) and V(Pt) are therefore read in phases 2t+2 and 2t+3 only; their buffers (parity of the pair index) can be
// refilled with K(Pt+3) / V(Pt+2) from phase 2t+4 on.  Loads are issued by wavefronts in their vector phase only (a
// wavefront in its matrix phase is the critical path and issues nothing but MFMAs and operand reads; a direct load
// holds its wavefront for ~64 cycles), each for its own rows and those of the wavefront four away, and the two groups
// share the issue: group 1 issues V(Pt+1) at the start of phase 2t+2 and awaits it at the end of phase 2t+3, before the
// barrier that lets group 0 read it; group 0 issues K(Pt+1) at the start of phase 2t+1 (its buffer was last read in
// phase 2t-1) and awaits it at the end of the same phase, behind its two softmaxes (about 0.8 us later: K comes from
// L2 or the memory-side cache, whose latency that covers).  All of it in group 1 made that group's vector phase the
// longest phase by ~500 cycles.  A sequence with an odd number of tiles ends in a pair of one tile; the QK MFMAs of the
// missing tile run on whatever its buffer half holds and their scores are never read.
// ---------------------------------------------------------------------------------------------
template <class T>
__global__ void __attribute__((amdgpu_flat_work_group_size(T::NT, T::NT), amdgpu_waves_per_eu(2, 2)))
attn_fwd_pp_kernel(AttnParams p) {
  static_assert(T::NWAVES == 8 && T::SUBS == 2, "two groups of four wavefronts, two tiles per phase");
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char* smem = (lds_char*)smem_generic;
  lds_slot* s_item = reinterpret_cast<lds_slot*>(smem + T::ITEM_OFF);

  const LaunchClock clock0 = launch_clock_begin();
  const int tid = threadIdx.x;
  const int64_t row_stride_b = (int64_t)p.n_heads * T::D * 2;
  const float c = p.c_log2;
  // Per-lane constants.  Only the two load offsets stay in registers for the life of the kernel; everything else is
  // recomputed where an item starts or ends (fresh_lane: some twenty instructions), from a thread index that the
  // compiler cannot see through.  Kept live instead, they sit in registers that the pair loop needs and are spilled
  // around it: sixty scratch instructions per wavefront and item, on the one vector-memory path that the item's first
  // loads and output stores also go through.
  auto fresh_lane = [&]() {
    int t = tid;
    asm volatile("" : "+v"(t));
    Lane<T> l;
    l.init(t, row_stride_b);
    return l;
  };
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int group = wave >> 2;
  uint32_t kvoff, vvoff;
  {
    const Lane<T> L0 = fresh_lane();
    kvoff = L0.kvoff;
    vvoff = L0.vvoff;
  }

  // The index of the next item is requested towards the end of an item, into the slot of the other parity; a barrier
  // between that write and the end of the item makes it visible to every wave before it is read.
  if (tid == 0) s_item[0] = blockIdx.x;
  wg_barrier();
  int par = 0;

  for (;;) {
    const uint32_t item_idx = __builtin_amdgcn_readfirstlane(s_item[par]);
    if (item_idx >= p.n_items) break;
    par ^= 1;  // the next index goes to s_item[par], see below
    const ItemCtx<T> X = begin_item<T>(p, fresh_lane(), item_idx, row_stride_b);
    const int kv_len = X.it.kv_len, nt = X.nt;  // nt: 64-key tiles
    const int npairs = (nt + 1) >> 1;

    // Tile ti of K / V -> half ti&1 of the buffer of parity (ti>>1)&1, for the rows of wavefront `wave`.
    // dw: 0 for this wavefront's own rows, `other` for those of the wavefront four away
    auto load_k = [&](int ti, const Lane<T>& L, int dw) {
      if (ti < nt)
        tile_load_one<T>(X.kbase, row_stride_b, tile_first_key<T>(ti, kv_len), kv_len, L.lrow + dw * T::RPI, L.kcol,
                         kvoff + (uint32_t)(dw * T::RPI) * (uint32_t)row_stride_b, smem,
                         T::K_OFF + ((ti >> 1) & 1) * T::BUF_B + (ti & 1) * T::TILE_B, wave + dw);
    };
    auto load_v = [&](int ti, const Lane<T>& L, int dw) {
      if (ti < nt)
        tile_load_one<T>(X.vbase, row_stride_b, tile_first_key<T>(ti, kv_len), kv_len, L.lrow + dw * T::RPI, L.vcol,
                         vvoff + (uint32_t)(dw * T::RPI) * (uint32_t)row_stride_b, smem,
                         T::V_OFF + ((ti >> 1) & 1) * T::BUF_B + (ti & 1) * T::TILE_B, wave + dw);
    };
    // Inside the pair loop the group that is in its vector phase issues loads for both groups (its own rows and those
    // of the wavefront four away).  While the tiles are whole interior tiles (every tile but the last of a sequence)
    // their rows form one run of 2 * LPT load rounds, GROUP rows apart: the addresses come from one running pointer
    // and the load issue, which sits on the critical path of the vector phase, carries no per-tile tests or
    // multiplications.
    const int other = group == 1 ? -4 : 4;  // the wavefront whose rows this one also loads
    const uint32_t d4 = (uint32_t)(other * T::RPI) * (uint32_t)row_stride_b;
    const int64_t round_b = (int64_t)T::GROUP * row_stride_b;
    auto load_k_pair_all = [&](int tp) {  // K tiles 2tp, 2tp+1 -> K buffer tp&1
      if (2 * tp + 1 < nt - 1) {
        const char* kp = X.kbase + (int64_t)(2 * tp) * T::BN * row_stride_b;
        const uint32_t lk = (uint32_t)(uintptr_t)smem + T::K_OFF + (tp & 1) * T::BUF_B + (uint32_t)wave * 1024u;
#pragma unroll
        for (int j = 0; j < 2 * T::LPT; ++j) {
          lds_dma_16(kp + j * round_b, kvoff, lk + j * T::NWAVES * 1024);
          lds_dma_16(kp + j * round_b, kvoff + d4, lk + j * T::NWAVES * 1024 + other * 1024);
        }
      } else {
        const Lane<T> L = fresh_lane();
        load_k(2 * tp, L, 0);
        load_k(2 * tp + 1, L, 0);
        load_k(2 * tp, L, other);
        load_k(2 * tp + 1, L, other);
      }
    };
    auto load_v_pair_all = [&](int tp) {  // V tiles 2tp, 2tp+1 -> V buffer tp&1
      if (2 * tp + 1 < nt - 1) {
        const char* vp = X.vbase + (int64_t)(2 * tp) * T::BN * row_stride_b;
        const uint32_t lv = (uint32_t)(uintptr_t)smem + T::V_OFF + (tp & 1) * T::BUF_B + (uint32_t)wave * 1024u;
#pragma unroll
        for (int j = 0; j < 2 * T::LPT; ++j) {
          lds_dma_16(vp + j * round_b, vvoff, lv + j * T::NWAVES * 1024);
          lds_dma_16(vp + j * round_b, vvoff + d4, lv + j * T::NWAVES * 1024 + other * 1024);
        }
      } else {
        const Lane<T> L = fresh_lane();
        load_v(2 * tp, L, 0);
        load_v(2 * tp + 1, L, 0);
        load_v(2 * tp, L, other);
        load_v(2 * tp + 1, L, other);
      }
    };
    // A wavefront none of whose 32 query rows exists (the ragged last query tile of a sequence, a half-height item of
    // a pack's last round) takes its part in the loads and barriers of the item and computes nothing: its SIMD and the
    // power it would draw go to the wavefront it shares the SIMD with.  Wavefront 0 always has rows.
    if (wave * 32 >= X.it.q_rows) {
      if (group == 0) load_k_pair_all(0);
      wait_loads();
      wg_barrier();
      if (group == 1) {
        load_v_pair_all(0);
        wg_barrier();
        wait_loads();
      }
      wg_barrier();
      for (int t = 0; t + 1 < npairs; ++t) {
        if (group == 1) load_v_pair_all(t + 1);
        if (group == 0) load_k_pair_all(t + 1);
        if (group == 0) wait_loads();
        wg_barrier();
        if (group == 1) wait_loads();
        wg_barrier();
      }
      wg_barrier();
      wg_barrier();
      if (group == 0) wg_barrier();
      continue;
    }
    bf16x8 qf[T::NKS];
    {
      // Only what phase 0 needs, Q and K(P0): the loads of an item's start and the stores of its end go through the
      // compute unit's one path to L2 at some 30 bytes a cycle, and Q, three pairs of tiles and the output rows there
      // at once (224 KB) were 7 500 cycles of every item.  V(P0) and K(P1), first read in phase 2, follow in phases 0
      // and 1, when that path is idle.  Q first: its rows come from memory (no compute unit has read them before), K
      // and V mostly from L2.
      // K(P0) is loaded by group 0 for both groups: group 1, which comes out of the item before a phase later and
      // with its output stores just issued, is what the first barrier waits for.
      load_q<T>(p, fresh_lane(), X.it, row_stride_b, X.head_off, X.qrow, qf);
      if (group == 0) load_k_pair_all(0);
    }

    f32x16 o[T::NDB];
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m_ref = -1.0e30f;  // finite: (m_ref - m) * c stays finite
    float l_run = 0.f;
    f32x16 s[2][T::NKB];
    uint32_t pb[2][T::NKB][8];
    int ka[T::NKS], va[T::NDB];  // ka: K buffer the next QK reads; va: V buffer the next PV reads
    fresh_lane().operand_addrs((uint32_t)(uintptr_t)smem, (uint32_t)(uintptr_t)smem, ka, va);
    float alpha1 = 1.f;
    uint64_t grown = 0;

    wait_loads();
    wg_barrier();  // Q and K(P0) of every wave have landed; phase 0 starts
    if (group == 1) {  // group 1 has no matrix work in phase 0: it requests V(P0), awaited behind its QK(P0)
      load_v_pair_all(0);
      wg_barrier();
    }
    pp_stream<T, 0, 2, kPrefetch>(va, ka, pb, qf, o, s, 0, 1.f);  // QK(P0)
#pragma unroll
    for (int ks = 0; ks < T::NKS; ++ks) ka[ks] ^= T::BUF_B;
    if (group == 1) wait_loads();
    wg_barrier();

    if (npairs == 1 && tid == 0) s_item[par] = take_item(p);  // two barriers follow in the last pair
    for (int t = 0; t + 1 < npairs; ++t) {
      // ---- vector phase: softmax of both tiles of pair t (whole tiles)
      // The next index is requested at the start of this phase and put into its slot at the end (visible after the
      // barriers of the last pair): the request takes about a microsecond, which thread 0's wavefront spends on its
      // softmaxes instead of waiting while seven wavefronts wait for it at the barrier.
      const bool ask = t + 2 == npairs && tid == 0;
      uint32_t next_item = 0;
      if (ask) next_item = take_item(p);
      if (group == 1) load_v_pair_all(t + 1);            // read from phase 2t+4 on
      if (group == 0) load_k_pair_all(t + 1);  // read from the next phase on
      tile_softmax<T, false, true>(s[0], 0, TailRows{0, T::BN}, c, pb[0], o, m_ref, l_run);  // no mask: hh unused
      grown = tile_softmax<T, false, true, true>(s[1], 0, TailRows{0, T::BN}, c, pb[1], o, m_ref, l_run, &alpha1);
      if (group == 0) wait_loads();
      if (ask) s_item[par] = next_item;
      wg_barrier();
      // ---- matrix phase: PV(Pt), QK(Pt+1)
      __builtin_amdgcn_s_setprio(1);
      pp_stream<T, 2, 2, kPrefetch>(va, ka, pb, qf, o, s, grown, alpha1);
      l_run = (l_run + row_sum_burst<T>(pb[0])) * alpha1 + row_sum_burst<T>(pb[1]);
      asm volatile("" : "+v"(l_run));  // the sums are taken here, not behind the barrier
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int ks = 0; ks < T::NKS; ++ks) ka[ks] ^= T::BUF_B;
#pragma unroll
      for (int db = 0; db < T::NDB; ++db) va[db] ^= T::BUF_B;
      if (group == 1) wait_loads();  // pair t+1, issued at the start of this group's softmax(Pt)
      wg_barrier();
    }
    // ---- last pair: two tiles or one, the last of them masked; PV only
    if ((nt & 1) == 0) {
      tile_softmax<T, false, true>(s[0], 0, TailRows{0, T::BN}, c, pb[0], o, m_ref, l_run);
      grown = tile_softmax<T, true, true, true>(s[1], fresh_lane().hh, tail_rows<T>(kv_len), c, pb[1], o, m_ref, l_run, &alpha1);
      wg_barrier();
      __builtin_amdgcn_s_setprio(1);
      pp_stream<T, 2, 0, kPrefetch>(va, ka, pb, qf, o, s, grown, alpha1);
      l_run = (l_run + row_sum_burst<T>(pb[0])) * alpha1 + row_sum_burst<T>(pb[1]);
      asm volatile("" : "+v"(l_run));  // the sums are taken here, not behind the barrier
      __builtin_amdgcn_s_setprio(0);
    } else {
      tile_softmax<T, true, true>(s[0], fresh_lane().hh, tail_rows<T>(kv_len), c, pb[0], o, m_ref, l_run);
      wg_barrier();
      __builtin_amdgcn_s_setprio(1);
      pp_stream<T, 1, 0, kPrefetch>(va, ka, pb, qf, o, s, 0, 1.f);
      l_run += row_sum_burst<T>(pb[0]);
      asm volatile("" : "+v"(l_run));
      __builtin_amdgcn_s_setprio(0);
    }
    wg_barrier();

    {
      const Lane<T> L = fresh_lane();
      int qrow = L.wave * 32 + L.l32;  // as in item_ctx
      const bool row_valid = qrow < X.it.q_rows;
      if (!row_valid) qrow = X.it.q_rows - 1;
      // Staging area of the rows.  Group 0 stores while group 1 runs its last matrix phase, which reads V only, and
      // every load of K has been awaited: it takes K buffer 0.  Group 1 stores while group 0 starts the next item and
      // loads its first tiles into both K buffers and V buffer 0: it takes V buffer 1, which is loaded into next by
      // group 1 itself, in the next item's pair loop behind two barriers.
      const uint32_t stage = (uint32_t)(uintptr_t)smem + (group == 0 ? T::K_OFF : T::V_OFF + T::BUF_B) +
                             (uint32_t)(wave & 3) * (32 * T::ROW_B);
      store_out<T>(p, L, X.it, row_stride_b, X.head_off, qrow, row_valid, o, l_run, m_ref, stage);
    }
    if (group == 0) wg_barrier();  // group 0 idles (after its stores) while group 1 runs its last matrix phase
  }
  launch_clock_end(p, clock0);
  if (tid == 0) finish_workgroup(p);
}

// The LDS limit of a kernel is set once per device (its first use there also loads the kernel's code).
template <class T, void (*KERNEL)(AttnParams)>
static hipError_t prepare_t() {
  static bool attr_set[16] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16 || !attr_set[dev]) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(KERNEL), hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 16) attr_set[dev] = true;
  }
  return hipSuccess;
}

template <class T, void (*KERNEL)(AttnParams)>
static hipError_t launch_t(const AttnParams& p, int grid, hipStream_t stream) {
  const hipError_t e = prepare_t<T, KERNEL>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(KERNEL, dim3(grid), dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

hipError_t attn_fwd_prepare() {
  hipError_t e = prepare_t<Tile<128, 8, 64, 2>, attn_fwd_pp_kernel<Tile<128, 8, 64, 2>>>();
  if (e == hipSuccess) e = prepare_t<Tile<64, 8, 64, 2>, attn_fwd_pp_kernel<Tile<64, 8, 64, 2>>>();
  if (e == hipSuccess) e = prepare_t<Tile<128, 4, 64>, attn_fwd_kernel<Tile<128, 4, 64>>>();
  if (e == hipSuccess) e = prepare_t<Tile<64, 4, 64>, attn_fwd_kernel<Tile<64, 4, 64>>>();
  return e;
}

int attn_fwd_block_m(AttnKernel kernel) { return kernel == AttnKernel::kIndependent128 ? 128 : 256; }
int attn_fwd_wgs_per_cu(AttnKernel kernel) { return kernel == AttnKernel::kIndependent128 ? 2 : 1; }

AttnKernel attn_fwd_select(const int32_t* cu_seqlens, const int32_t* cu_seqlens_k, int32_t n_seqs, int32_t n_heads,
                           int n_cus) {
  // Measured on MI355X, head dimension 128 (time of the 128-row kernel over the ping-pong kernel, by 256-row items per
  // compute unit; 4096-token sequences, 6 to 80 heads): 0.38: 0.99;  0.5: 1.03;  0.62: 1.30;  0.75: 1.23;  0.88: 1.18;
  // 1.0: 1.16;  1.25: 0.98;  1.5: 1.01;  1.75: 1.11;  2.0: 1.13;  2.5: 1.09;  3.0: 1.22;  3.5: 1.07;  4 and more:
  // 1.13-1.18; packs of 4352- and 1280-token sequences from 0.94 to 9.6 items per compute unit: 1.07-1.20.  The
  // ping-pong kernel is ahead whenever its items fill the compute units; the 128-row kernel, whose items are half as
  // long, when there is under half a 256-row item per compute unit, or (by 2 %) when a second round of 256-row items
  // would be less than half full.
  // Items with few key tiles (cross-attention against a few hundred text keys) run better on the 128-row kernel, whose
  // workgroups have no idle phase at the ends of an item: 64 keys 0.83, 128: 0.89, 226: 0.96, 256: 0.96, 384: 1.02,
  // 512: 1.04, 768: 1.07, 1024: 1.05, 2048: 1.09.
  // (Comparisons of two kernels must be made on a warm chip: in the first ~20 ms after idle, while the clocks still
  // ramp, whichever kernel runs second looks faster.)
  const int32_t* ck = cu_seqlens_k ? cu_seqlens_k : cu_seqlens;
  int64_t items256 = 0, tiles = 0;
  for (int32_t i = 0; i < n_seqs; ++i) {
    const int64_t lq = cu_seqlens[i + 1] - cu_seqlens[i], lk = ck[i + 1] - ck[i];
    if (lq == 0 || lk == 0) continue;
    const int64_t it = (lq + 255) / 256 * n_heads;
    items256 += it;
    tiles += it * ((lk + 63) / 64);
  }
  if (items256 * 20 < (int64_t)n_cus * 9) return AttnKernel::kIndependent128;
  if (cu_seqlens_k != nullptr && tiles <= 5 * items256) return AttnKernel::kIndependent128;
  const int64_t in_second_round = items256 - n_cus;
  if (in_second_round > 0 && 5 * in_second_round <= 2 * (int64_t)n_cus) return AttnKernel::kIndependent128;
  return AttnKernel::kPingPong256;
}

hipError_t attn_fwd_launch(const AttnParams& p, AttnKernel kernel, int head_dim, int grid, hipStream_t stream) {
  if (kernel != AttnKernel::kIndependent128) {
    if (head_dim == 128) return launch_t<Tile<128, 8, 64, 2>, attn_fwd_pp_kernel<Tile<128, 8, 64, 2>>>(p, grid, stream);
    if (head_dim == 64) return launch_t<Tile<64, 8, 64, 2>, attn_fwd_pp_kernel<Tile<64, 8, 64, 2>>>(p, grid, stream);
  } else {
    if (head_dim == 128) return launch_t<Tile<128, 4, 64>, attn_fwd_kernel<Tile<128, 4, 64>>>(p, grid, stream);
    if (head_dim == 64) return launch_t<Tile<64, 4, 64>, attn_fwd_kernel<Tile<64, 4, 64>>>(p, grid, stream);
  }
  return hipErrorInvalidValue;
}

}  // namespace dit
