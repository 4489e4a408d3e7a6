// DiT denoising-step self-attention forward for gfx950 (MI355X): the "wide" kernel.
//
// 4 wavefronts per workgroup, one per SIMD, one workgroup per compute unit, 64 query rows per wavefront (two
// 32-row halves), 256 per workgroup.  Why: in the other two kernels every MFMA takes a fresh A operand (1 KB per
// wavefront) from LDS, and those reads, not the matrix pipe, set both the cycle count and - through the power they
// draw - the clock the chip sustains.  Here each K / V^T operand read from LDS feeds two MFMAs (one per half), so
// the LDS traffic per flop is halved.  The price is 512 registers per lane (one wavefront per SIMD), so nothing
// hides a wavefront's latencies but its own instruction stream, which is therefore software-pipelined by hand:
//
//   step t (one K/V tile, 64 MFMAs at head_dim 128):
//     MFMA slots  0..31   S(t+1)^T = K(t+1) Q^T               -> scores of the NEXT tile
//     MFMA slots 32..63   O^T     += V(t)^T P(t)^T
//     in the shadow of those MFMAs (the matrix pipe is busy 32 cycles per MFMA, issuing one takes ~8):
//       exponentials, row sums and bf16 packing of tile t, group by group, each group finished before the PV slot
//       that reads it; then the row maxima of tile t+1 (its scores are complete after slot 31); and the direct
//       HBM -> LDS loads of the tiles three steps ahead.
//   Between steps: the cross-lane half of the maxima, the (rare) rescale of O^T and l, one workgroup barrier.
//   The operand ring (reads run 4 operands = 8 MFMAs ahead) carries across the barrier: the last slots of a step
//   already read the first K operands of the next step, so the matrix pipe does not drain at step boundaries.
//
// LDS: four K and four V tile buffers (tile index mod 4).  Step t reads the pair L(t) = {K(t+1), V(t)}, issues the
// loads of L(t+3) (their buffers were last read in step t-1) and, before the barrier that ends it, waits for this
// wavefront's share of L(t+2); so L(t+2) is complete and visible to everyone from step t+1 on, whose last slots
// prefetch from it.  Pairs past the end of the sequence are loaded from the last tile and never used.
//
// Arithmetic is the same, in the same order, as in the other kernels (a row's result does not depend on the kernel).
// The row maximum of the last, partial tile is taken over all 64 score rows: the rows that are masked out of the sums
// are copies of real keys of the same sequence (see tile_first_key), so the maximum over them is a maximum over real
// keys.
#include "attn_device.h"

namespace dit {

template <class T>
struct Wide {
  static_assert(T::NWAVES == 4, "one wavefront per SIMD");
  static constexpr int NBUF = 4;
  static constexpr int BM = T::NWAVES * 64;
  static constexpr int K_OFF = 0;
  static constexpr int V_OFF = NBUF * T::TILE_B;
  static constexpr int ITEM_OFF = 2 * NBUF * T::TILE_B;
  static constexpr int LDS_BYTES = ITEM_OFF + 16;
  static constexpr int LPP = 2 * T::LPT;          // direct loads per wavefront per pair {K tile, V tile}
  static constexpr int NF_QK = T::NKB * T::NKS;   // operand fragments of the first contraction (each feeds 2 MFMAs)
  static constexpr int NF_PV = 2 * T::NKB * T::NDB;
  static constexpr int PD = 4;                    // operand ring depth, in fragments
  static constexpr int NPAIR = 2 * T::NKB * 8;    // pairs of probabilities per lane per tile (both halves)
  static constexpr int NMAX = 2 * T::NKB * 8;     // max3 operations per lane per tile (both halves)
  static_assert(NF_QK % PD == 0 && NF_PV % PD == 0, "the ring position of a fragment must not depend on the step");
};

// Q fragments of one 32-row half (B operand of S^T = K Q^T; lane holds query row l32, d = 16*ks + 8*hh .. +7), loaded
// straight into accumulation registers and awaited here.  (A value that the compiler classes as an ordinary register
// and that an asm operand asks for in an accumulation register is copied in front of every use; these are defined in
// place.  The sign flip for a negative scale is not available on this path: such calls run the ping-pong kernel.)
template <class T>
__device__ __forceinline__ void load_q_acc(const char* qptr, u32x4 (&qf)[T::NKS]) {
  if constexpr (T::NKS == 8) {
    asm volatile(
        "global_load_dwordx4 %0, %8, off\n\t"
        "global_load_dwordx4 %1, %8, off offset:32\n\t"
        "global_load_dwordx4 %2, %8, off offset:64\n\t"
        "global_load_dwordx4 %3, %8, off offset:96\n\t"
        "global_load_dwordx4 %4, %8, off offset:128\n\t"
        "global_load_dwordx4 %5, %8, off offset:160\n\t"
        "global_load_dwordx4 %6, %8, off offset:192\n\t"
        "global_load_dwordx4 %7, %8, off offset:224\n\t"
        "s_waitcnt vmcnt(0)"
        : "=a"(qf[0]), "=a"(qf[1]), "=a"(qf[2]), "=a"(qf[3]), "=a"(qf[4]), "=a"(qf[5]), "=a"(qf[6]), "=a"(qf[7])
        : "v"(qptr)
        : "memory");
  } else {
    static_assert(T::NKS == 4, "head dimension 64 or 128");
    asm volatile(
        "global_load_dwordx4 %0, %4, off\n\t"
        "global_load_dwordx4 %1, %4, off offset:32\n\t"
        "global_load_dwordx4 %2, %4, off offset:64\n\t"
        "global_load_dwordx4 %3, %4, off offset:96\n\t"
        "s_waitcnt vmcnt(0)"
        : "=a"(qf[0]), "=a"(qf[1]), "=a"(qf[2]), "=a"(qf[3])
        : "v"(qptr)
        : "memory");
  }
}

// One pass over the MFMA slots of a tile.
//   DO_QK: nxt[h][kb] = K(ka) Q^T.   DO_PV: o[h][db] += V(va)^T P^T with P = pb.
//   RING_IN: ring already holds the first PD fragments.   RING_OUT: the last slots read the first PD K fragments of
//   the buffer at ka + kstep into the ring.
//   SHADOW: between the MFMAs, exponentials / sums / packing of `cur` into pb and lsum, maxima of `nxt` into mx, and
//   issue_load(i), i in [0, LPP).
template <class T, bool DO_QK, bool DO_PV, bool RING_IN, bool RING_OUT, bool SHADOW, class LoadFn>
__device__ __forceinline__ void wide_stream(int (&va_)[T::NDB], int (&ka_)[T::NKS], int kstep,
                                            bf16x8 (&ring)[Wide<T>::PD], const u32x4 (&qf)[2][T::NKS],
                                            f32x16 (&o)[2][T::NDB], f32x16 (&cur)[2][T::NKB], f32x16 (&nxt)[2][T::NKB],
                                            uint32_t (&pb)[2][T::NKB][8], const float (&mc)[2], float c,
                                            float (&lsum)[2], float (&mx)[2], LoadFn&& issue_load) {
  using W = Wide<T>;
  constexpr int PD = W::PD;
  constexpr int NFQ = DO_QK ? W::NF_QK : 0;
  constexpr int NFP = DO_PV ? W::NF_PV : 0;
  constexpr int NF = NFQ + NFP;            // fragments consumed here
  constexpr int NFR = NF + (RING_OUT ? PD : 0);  // fragments read here (plus PD if !RING_IN, minus none)
  constexpr int NS = 2 * NF;               // MFMA slots
  constexpr int SQ = 2 * NFQ;              // first PV slot

  // fragment F: [0, NFQ) K operand (ks = F / NKB, kb = F % NKB); [NFQ, NF) V^T operand (g = (F-NFQ) / NDB = 2*kb + u,
  // db = (F-NFQ) % NDB); [NF, NF+PD) K operand F-NF of the next buffer.
  auto read_frag = [&](auto fc) {
    constexpr int F = decltype(fc)::value;
    if constexpr (F < NFQ) {
      constexpr int ks = F / T::NKB, kb = F % T::NKB;
      ring[F % PD] = *(lds_bf16x8*)(uintptr_t)(uint32_t)(ka_[ks] + kb * 32 * T::ROW_B);
    } else if constexpr (F < NF) {
      constexpr int g = (F - NFQ) / T::NDB, db = (F - NFQ) % T::NDB;
      lds_char* p0 = (lds_char*)(uintptr_t)(uint32_t)(va_[db] + 16 * g * T::ROW_B);
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
      const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 8 * T::ROW_B));
      ring[F % PD] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
      constexpr int ks = (F - NF) / T::NKB, kb = (F - NF) % T::NKB;
      ring[F % PD] = *(lds_bf16x8*)(uintptr_t)(uint32_t)(ka_[ks] + kstep + kb * 32 * T::ROW_B);
    }
  };
  auto mfma_slot = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    constexpr int F = J / 2, h = J % 2;
    if constexpr (F < NFQ) {
      constexpr int ks = F / T::NKB, kb = F % T::NKB;
      // Written as assembly to pin the register files: scores in ordinary VGPRs (the vector ALU reads them), Q in
      // accumulation registers.  With more than 256 registers per lane the compiler would otherwise put every MFMA
      // result into accumulation registers and copy each score out, one instruction per value.
      // The compiler does not see this instruction's latency: every vector read of these scores is placed at least
      // three MFMA slots (> 96 cycles) after the last MFMA that writes them (the rule is 18 four-cycle wait states).
      if constexpr (ks == 0) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(nxt[h][kb]) : "v"(ring[F % PD]), "a"(qf[h][ks]));
      } else {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(nxt[h][kb]) : "v"(ring[F % PD]), "a"(qf[h][ks]));
      }
    } else {
      constexpr int g = (F - NFQ) / T::NDB, db = (F - NFQ) % T::NDB, kb = g / 2, u = g % 2;
      u32x4 pw = {pb[h][kb][4 * u], pb[h][kb][4 * u + 1], pb[h][kb][4 * u + 2], pb[h][kb][4 * u + 3]};
      o[h][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[F % PD], __builtin_bit_cast(bf16x8, pw), o[h][db], 0, 0, 0);
    }
  };
  // After the second MFMA of fragment F: an empty asm statement that takes the accumulator just written and passes
  // the address register of the next read through, so that the read is not issued earlier; emits nothing.
  auto tie = [&](auto fc) {
    (void)o;
    (void)nxt;
    constexpr int F = decltype(fc)::value;  // fragment just consumed
    constexpr int R = F + PD;               // fragment to read next
    if constexpr (R < NFR) {
      constexpr bool IS_V = R >= NFQ && R < NF;
      constexpr int AI = R < NFQ ? R / T::NKB : (R < NF ? (R - NFQ) % T::NDB : (R - NF) / T::NKB);
      if constexpr (F < NFQ) {
        if constexpr (IS_V) {
          asm volatile("" : "+v"(va_[AI]) : "v"(nxt[1][F % T::NKB]));
        } else {
          asm volatile("" : "+v"(ka_[AI]) : "v"(nxt[1][F % T::NKB]));
        }
      } else {
        if constexpr (IS_V) {
          asm volatile("" : "+v"(va_[AI]) : "a"(o[1][(F - NFQ) % T::NDB]));
        } else {
          asm volatile("" : "+v"(ka_[AI]) : "a"(o[1][(F - NFQ) % T::NDB]));
        }
      }
    }
  };

  // ---- vector work in the shadow of the MFMAs
  // pair n: group g = n / 8 (kb = g / 2, second 8 scores of the block if g odd), half h = (n % 8) / 4, pair n % 4.
  auto exp_pair = [&](auto nc) {
    constexpr int n = decltype(nc)::value;
    constexpr int g = n / 8, h = (n % 8) / 4, kb = g / 2, i = 8 * (g % 2) + 2 * (n % 4);
    const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[h][kb][i], c, -mc[h]));
    const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[h][kb][i + 1], c, -mc[h]));
    pb[h][kb][i >> 1] = pack_bf16x2(p0, p1);
    asm volatile("" : "+v"(pb[h][kb][i >> 1]));
  };
  auto max_op = [&](auto kc) {
    constexpr int k = decltype(kc)::value;
    constexpr int h = k / (W::NMAX / 2), q = k % (W::NMAX / 2), kb = q / 8, i = 2 * (q % 8);
    if constexpr (q == 0) {
      mx[h] = __builtin_fmaxf(nxt[h][kb][i], nxt[h][kb][i + 1]);
    } else {
      mx[h] = __builtin_fmaxf(__builtin_fmaxf(mx[h], nxt[h][kb][i]), nxt[h][kb][i + 1]);
    }
    asm volatile("" : "+v"(mx[h]));
  };
  // Slot after whose MFMA a unit of vector work is issued.  Pairs are spread evenly up to two slots before the
  // last group is read (group g is read from PV slot SQ + 2*NDB*g on); maxima start three slots after the last MFMA of the scores.
  constexpr int kPairSpan = SQ + 6 * T::NDB - 2;
  constexpr int kMaxFirst = SQ + 3, kMaxSpan = NS - SQ - 4;
  auto shadow = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    if constexpr (SHADOW) {
      static_for<0, W::NPAIR>([&](auto nc) {
        constexpr int n = decltype(nc)::value;
        if constexpr (n * kPairSpan / W::NPAIR == J) exp_pair(nc);
      });
      static_for<0, W::NMAX>([&](auto kc) {
        constexpr int k = decltype(kc)::value;
        if constexpr (kMaxFirst + k * kMaxSpan / W::NMAX == J) max_op(kc);
      });
      static_for<0, W::LPP>([&](auto ic) {
        constexpr int i = decltype(ic)::value;
        if constexpr (1 + (NS / W::LPP) * i == J) issue_load(i);
      });
    }
  };

  SCHED_FENCE();
  if constexpr (!RING_IN) {
    static_for<0, PD>([&](auto fc) { read_frag(fc); });
    SCHED_FENCE();
  }
  static_for<0, NS>([&](auto jc) {
    constexpr int J = decltype(jc)::value;
    mfma_slot(jc);
    if constexpr (J % 2 == 1) {
      tie(IC<J / 2>{});
      if constexpr (J / 2 + PD < NFR) read_frag(IC<J / 2 + PD>{});
    }
    shadow(jc);
    SCHED_FENCE();
  });
  SCHED_FENCE();
}

struct NoLoad {
  __device__ __forceinline__ void operator()(int) const {}
};

template <class T>
__global__ void __attribute__((amdgpu_flat_work_group_size(T::NT, T::NT), amdgpu_waves_per_eu(1, 1)))
attn_fwd_wide_kernel(AttnParams p) {
  using W = Wide<T>;
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  lds_char* smem = (lds_char*)smem_generic;
  volatile uint32_t* s_item = reinterpret_cast<volatile uint32_t*>(smem_generic + W::ITEM_OFF);

  const LaunchClock clock0 = launch_clock_begin();
  const int tid = threadIdx.x;
  const int64_t row_stride_b = (int64_t)p.n_heads * T::D * 2;
  const float c = p.c_log2;
  Lane<T> L;
  L.init(tid, row_stride_b);

  if (tid == 0) s_item[0] = blockIdx.x;
  wg_barrier();
  int par = 0;

  for (;;) {
    const uint32_t item_idx = __builtin_amdgcn_readfirstlane(s_item[par]);
    if (item_idx >= p.n_items) break;
    par ^= 1;  // the next index goes to s_item[par] during the item's last step (a barrier follows)
    const ItemU it = fetch_item(p.items, item_idx);
    const int kv_len = it.kv_len;
    const int nt = (kv_len + T::BN - 1) / T::BN;
    const int64_t head_off = (int64_t)it.head * T::D * 2;
    const char* kbase = static_cast<const char*>(p.k) + (int64_t)it.kv_start * row_stride_b + head_off;
    const char* vbase = static_cast<const char*>(p.v) + (int64_t)it.kv_start * row_stride_b + head_off;
    // Half h of this wavefront owns query rows 64*wave + 32*h + lane%32 of the item; halves past the end of a ragged
    // item work on a copy of its last row and store nothing.
    int qrow[2];
    bool row_valid[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      qrow[h] = L.wave * 64 + 32 * h + L.l32;
      row_valid[h] = qrow[h] < it.q_rows;
      if (!row_valid[h]) qrow[h] = it.q_rows - 1;
    }

    // This wave's rows of K(ti) / V(ti) -> buffer ti & 3 (ti clamped to the last tile).
    auto load_k = [&](int ti) {
      const int src = ti < nt ? ti : nt - 1;
      tile_load_one<T>(kbase, row_stride_b, tile_first_key<T>(src, kv_len), kv_len, L.lrow, L.kcol, L.kvoff, smem, W::K_OFF + (ti & 3) * T::TILE_B, L.wave);
    };
    auto load_v = [&](int ti) {
      const int src = ti < nt ? ti : nt - 1;
      tile_load_one<T>(vbase, row_stride_b, tile_first_key<T>(src, kv_len), kv_len, L.lrow, L.vcol, L.vvoff, smem, W::V_OFF + (ti & 3) * T::TILE_B, L.wave);
    };
    load_k(0);
    for (int j = 0; j < 3; ++j) {  // pairs L(0), L(1), L(2)
      load_k(j + 1);
      load_v(j);
    }
    u32x4 qf[2][T::NKS];  // in accumulation registers; the wait inside also covers the tile loads above
#pragma unroll
    for (int h = 0; h < 2; ++h)
      load_q_acc<T>(static_cast<const char*>(p.q) + (int64_t)(it.q_start + qrow[h]) * row_stride_b + head_off + L.hh * 16, qf[h]);

    f32x16 o[2][T::NDB];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int db = 0; db < T::NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[h][db][i] = 0.f;
    float m_ref[2] = {-1.0e30f, -1.0e30f};  // finite, so that (m_ref - m) * 0 is 0 when scale is 0
    float l_run[2] = {0.f, 0.f};
    float mc[2], mx[2], lsum[2] = {0.f, 0.f};
    f32x16 sa[2][T::NKB], sb[2][T::NKB];
    uint32_t pb[2][T::NKB][8];
    bf16x8 ring[W::PD];
    int ka[T::NKS], va[T::NDB];  // ka: K buffer the next QK reads; va: V buffer the next PV reads
    L.operand_addrs((uint32_t)(uintptr_t)smem + W::K_OFF - T::K_OFF, (uint32_t)(uintptr_t)smem + W::V_OFF - T::V_OFF, ka, va);
    int kbuf = 0, vbuf = 0;
    auto k_step = [&]() { return kbuf == W::NBUF - 1 ? -(W::NBUF - 1) * T::TILE_B : T::TILE_B; };
    auto next_k = [&]() {
      const int step = k_step();
      kbuf = kbuf == W::NBUF - 1 ? 0 : kbuf + 1;
#pragma unroll
      for (int ks = 0; ks < T::NKS; ++ks) ka[ks] += step;
    };
    auto next_v = [&]() {
      const int step = vbuf == W::NBUF - 1 ? -(W::NBUF - 1) * T::TILE_B : T::TILE_B;
      vbuf = vbuf == W::NBUF - 1 ? 0 : vbuf + 1;
#pragma unroll
      for (int db = 0; db < T::NDB; ++db) va[db] += step;
    };
    // Row maxima of the tile whose scores are in s are in mx (in-lane part): cross-lane part, then the rescale of
    // O^T and l if some row of the wavefront has a new maximum.
    auto finish_max = [&]() {
      bool grow = false;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        mx[h] = max_with_other_half(mx[h]);
        grow |= (mx[h] - m_ref[h]) * c > kRescaleLog2;
      }
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const float m_new = (mx[h] - m_ref[h]) * c > kRescaleLog2 ? mx[h] : m_ref[h];
          const float alpha = __builtin_amdgcn_exp2f((m_ref[h] - m_new) * c);
          m_ref[h] = m_new;
          l_run[h] *= alpha;
#pragma unroll
          for (int db = 0; db < T::NDB; ++db) {
#pragma unroll
            for (int i = 0; i < 16; ++i) o[h][db][i] *= alpha;
            SCHED_FENCE();  // one block of O^T at a time through the ordinary registers
          }
        }
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) mc[h] = m_ref[h] * c;
    };

    wg_barrier();  // everyone's K(0), L(0), L(1), L(2) have landed
    // S(0), and the first K operands of step 0 into the ring.
    wide_stream<T, true, false, false, true, false>(va, ka, k_step(), ring, qf, o, sb, sa, pb, mc, c, lsum, mx, NoLoad{});
    next_k();
    asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");  // the scores are read at once: see wide_stream
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float m = sa[h][0][0];
#pragma unroll
      for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) m = __builtin_fmaxf(m, sa[h][kb][i]);
      mx[h] = m;
    }
    finish_max();

    // One step: scores of tile t are in `cur`; leaves those of tile t+1 in `nxt`.
    if (nt == 1 && tid == 0) s_item[par] = take_item(p);
    auto step = [&](f32x16 (&cur)[2][T::NKB], f32x16 (&nxt)[2][T::NKB], int t) {
      if (t + 2 == nt && tid == 0) s_item[par] = take_item(p);
      lsum[0] = 0.f;
      lsum[1] = 0.f;
      // Loads of the pair L(t+3) = {K(t+4), V(t+3)}; nt >= 2 here, so every tile is whole.  The tile addresses are
      // formed once per step (scalar instructions also take issue slots of the one wavefront on this SIMD).
      const int tk = t + 4 < nt ? t + 4 : nt - 1, tv = t + 3 < nt ? t + 3 : nt - 1;
      const char* kptr = kbase + (int64_t)tile_first_key<T>(tk, kv_len) * row_stride_b;
      const char* vptr = vbase + (int64_t)tile_first_key<T>(tv, kv_len) * row_stride_b;
      const uint32_t kdst = (uint32_t)(uintptr_t)smem + W::K_OFF + ((t + 4) & 3) * T::TILE_B + L.wave * 1024;
      const uint32_t vdst = (uint32_t)(uintptr_t)smem + W::V_OFF + ((t + 3) & 3) * T::TILE_B + L.wave * 1024;
      const int64_t group_b = (int64_t)T::GROUP * row_stride_b;
      auto issue = [&](int i) {
        if (i < T::LPT) {
          lds_dma_16(kptr, L.kvoff, kdst + i * T::NWAVES * 1024);
          kptr += group_b;
        } else {
          lds_dma_16(vptr, L.vvoff, vdst + (i - T::LPT) * T::NWAVES * 1024);
          vptr += group_b;
        }
      };
      wide_stream<T, true, true, true, true, true>(va, ka, k_step(), ring, qf, o, cur, nxt, pb, mc, c, lsum, mx, issue);
      // Row sums over the packed probabilities, in one burst after the last MFMA has been issued: the dot products share
      // a pipe with the MFMAs, and one between two MFMAs holds both up.
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
          for (int i = 0; i < 8; ++i) lsum[h] = add_prob_pair(lsum[h], pb[h][kb][i]);
        l_run[h] += lsum[h];
      }
      next_k();
      next_v();
      finish_max();
      wait_loads_but<W::LPP>();  // this wave's share of L(t+2); L(t+3), just issued, stays in flight
      phase_barrier();           // the ring reads of the next step's first operands are still outstanding
    };
    // Last tile: masked exponentials, then PV, nothing overlapped.
    auto last = [&](f32x16 (&cur)[2][T::NKB]) {
      const TailRows rows = tail_rows<T>(kv_len);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float ls = 0.f;
#pragma unroll
        for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[h][kb][i], c, -mc[h]));
            float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(cur[h][kb][i + 1], c, -mc[h]));
            const int key = 32 * kb + 8 * (i >> 2) + 4 * L.hh + (i & 3);
            if (key < rows.lo || key >= rows.hi) p0 = 0.f;
            if (key + 1 < rows.lo || key + 1 >= rows.hi) p1 = 0.f;
            pb[h][kb][i >> 1] = pack_bf16x2(p0, p1);
            ls = add_prob_pair(ls, pb[h][kb][i >> 1]);
            asm volatile("" : "+v"(pb[h][kb][i >> 1]), "+v"(ls));  // one pair at a time: keeps the register peak low
            SCHED_FENCE();
          }
        l_run[h] += ls;
      }
      wide_stream<T, false, true, false, false, false>(va, ka, 0, ring, qf, o, cur, cur, pb, mc, c, lsum, mx, NoLoad{});
    };

    // Steps alternate between the two score buffers; the last tile is always finished from sa.
    bool in_sb = false;
    for (int t = 0; t + 1 < nt; t += 2) {
      step(sa, sb, t);
      if (t + 2 >= nt) {
        in_sb = true;
        break;
      }
      step(sb, sa, t + 1);
    }
    if (in_sb) {
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int kb = 0; kb < T::NKB; ++kb) sa[h][kb] = sb[h][kb];
    }
    last(sa);
    wait_loads();  // pairs past the end are never read, but they must not outlive the item
    wg_barrier();  // everyone is done reading: the next item's loads may overwrite the buffers

#pragma unroll
    for (int h = 0; h < 2; ++h) {
      store_out<T>(p, L, it, row_stride_b, head_off, qrow[h], row_valid[h], o[h], l_run[h], m_ref[h]);
      SCHED_FENCE();
    }
  }
  launch_clock_end(p, clock0);
  if (tid == 0) finish_workgroup(p);
}

template <class T>
static hipError_t launch_wide(const AttnParams& p, int grid, hipStream_t stream) {
  static bool attr_set[16] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16 || !attr_set[dev]) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_fwd_wide_kernel<T>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            Wide<T>::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 16) attr_set[dev] = true;
  }
  hipLaunchKernelGGL(attn_fwd_wide_kernel<T>, dim3(grid), dim3(T::NT), Wide<T>::LDS_BYTES, stream, p);
  return hipGetLastError();
}

hipError_t attn_fwd_wide_launch(const AttnParams& p, int head_dim, int grid, hipStream_t stream) {
  if (head_dim == 128) return launch_wide<Tile<128, 4, 64>>(p, grid, stream);
  if (head_dim == 64) return launch_wide<Tile<64, 4, 64>>(p, grid, stream);
  return hipErrorInvalidValue;
}

}  // namespace dit
