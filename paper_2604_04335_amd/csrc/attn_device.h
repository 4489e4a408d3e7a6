// Device-side building blocks shared by the gfx950 (MI355X) attention forward kernels.
//
// DiT denoising-step self-attention forward:
//
// O[r,h,:] = sum_j softmax_j(scale * <Q[r,h,:], K[j,h,:]>) V[j,h,:], j over the
// keys of r's own sequence (paper Sections 4.3 and 5 give the batch; the math is
// plain softmax attention).  bf16 in, fp32 scores/state/accumulators, bf16 out.
//
// Mapping.  A persistent workgroup takes (sequence, head, query tile) items from
// a list through one atomic counter.  Each wavefront owns 32 query rows.  K and V
// tiles of BN keys are copied HBM -> LDS by direct (register-free) loads, double
// buffered.  Both contractions run on the 32x32x16 bf16 MFMA in *transposed* form:
//     S^T[key, query] = K[key, :] . Q[query, :]        A = K (from LDS), B = Q (registers)
//     O^T[d,   query] += V^T[d, key] . P^T[key, query] A = V^T (LDS transpose read), B = P (registers)
// In the MFMA result layout a lane holds one query column and 16 key rows, so the
// row maximum and row sum of the online softmax are in-lane reductions plus one
// exchange with lane^32, and the per-query rescale of O^T is a per-lane scalar.
// The 16 probabilities a lane holds after the softmax are exactly the 2 x 8
// k-slots of the B operand of the second contraction if the V^T operand uses the
// same key order, which two 4-key transpose reads deliver.
//
// LDS layout.  A tile row is the ROW_B bytes of one key of one head, rows are
// contiguous (a direct load writes 64 lanes x 16 B contiguously), and the 16-byte
// chunks of a row are XOR-swizzled so that the 16 rows a b128 read touches per
// pass (K) and the 4 rows x 64 B a transpose read touches per pass (V) fall in
// distinct banks.  The swizzle is applied by choosing which global chunk a lane
// fetches, so it costs nothing.
//
// Epilogue.  In the accumulator layout a lane holds eight bytes of one output row, so the rows are staged through a K
// or V buffer that is free at the end of an item and leave as whole rows (store_out).
//
// Softmax reference.  The value subtracted in the exponent follows a row's running maximum lazily: it moves (and O^T
// and the running sum are rescaled) only in tiles where the row's maximum exceeds it by more than 2^8 in the base-2
// exponent, so probabilities lie in (0, 2^8] rather than (0, 1]; the quotient O / l does not depend on the reference.
// The running sum l is taken over the probabilities as rounded to bf16 for the second contraction, so O / l is a
// convex combination of V rows whatever the rounding did (a row dominated by one key returns that key's V row
// exactly), and the log-sum-exp output carries at most the 2^-8 relative error of the rounded terms:
// |lse - exact| <= ln(1 + 2^-8) = 3.9e-3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_fwd.h"

namespace dit {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

typedef __attribute__((address_space(3))) char lds_char;
// The slot through which a workgroup's wavefronts learn the index of their next item.  Typed as LDS memory on purpose:
// through a generic pointer the read is a flat load, which the hardware counts with the vector-memory operations, and
// the wait for it at the top of an item then also waits for every output store of the item before.
typedef __attribute__((address_space(3))) volatile uint32_t lds_slot;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(1))) const void gptr_void;

// Operand reads of an MFMA stream run this many MFMAs ahead of their use.
constexpr int kPrefetch = 4;
// Full scheduling fence: the compiler's instruction scheduler moves nothing across it.
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// BN keys form one tile: the unit of the softmax (one reference-value decision per row and tile) and of the loads.
// A K or V buffer holds SUBS consecutive tiles; the ping-pong kernel works through SUBS = 2 tiles per phase.
template <int D_, int NWAVES_, int BN_, int SUBS_ = 1>
struct Tile {
  static constexpr int D = D_;
  static constexpr int NWAVES = NWAVES_;
  static constexpr int BN = BN_;
  static constexpr int SUBS = SUBS_;
  static constexpr int NT = NWAVES * 64;           // threads
  static constexpr int BM = NWAVES * 32;           // query rows per workgroup
  static constexpr int ROW_B = D * 2;              // bytes of one K/V row of one head
  static constexpr int TILE_B = BN * ROW_B;        // one K or V tile in LDS
  static constexpr int CPR = ROW_B / 16;           // 16-byte chunks per row
  static constexpr int RPI = 64 / CPR;             // rows one direct-load instruction covers
  static constexpr int GROUP = NWAVES * RPI;       // rows one round of loads (all waves) covers
  static constexpr int LPT = BN / GROUP;           // load instructions per wave per tensor per tile
  static constexpr int NKB = BN / 32;              // 32-key blocks per tile
  static constexpr int NKS = D / 16;               // k-steps of the first contraction
  static constexpr int NDB = D / 32;               // 32-wide d blocks of the output
  static constexpr int NQK = NKB * NKS;            // MFMAs of S^T = K Q^T per tile
  static constexpr int NPV = NKB * 2 * NDB;        // MFMAs of O^T += V^T P^T per tile
  // LDS: [K buffer 0][K buffer 1][V buffer 0][V buffer 1][two item slots], a buffer = SUBS tiles
  static constexpr int BUF_B = SUBS * TILE_B;
  static constexpr int K_OFF = 0;
  static constexpr int V_OFF = 2 * BUF_B;
  static constexpr int ITEM_OFF = 4 * BUF_B;
  static constexpr int LDS_BYTES = 4 * BUF_B + 16;
  static_assert(GROUP % 16 == 0 && BN % GROUP == 0, "load rounds must keep row%16 fixed per lane");
  static_assert(D == 64 || D == 128, "head dimension");

  // Chunk swizzles (XOR on the 16-byte chunk index of a row).
  //   K: the 16 consecutive rows of a b128 pass must land in 16 distinct 16-byte bank groups.
  //   V: the 4 consecutive rows x 4 chunks of a transpose-read pass must land in 4 distinct 64-byte groups.
  __device__ static constexpr int swz_k(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  __device__ static constexpr int swz_v(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);
  return __builtin_bit_cast(uint32_t, h);
}

// acc + both bf16 values of a packed pair (one v_dot2c_f32_bf16 against {1, 1}).  The row sum l is taken over the
// probabilities as rounded for the second contraction, so that O / l is a convex combination of the V rows whatever the
// rounding did (with the lazy reference value the largest probability of a row is no longer the exact value 1).
__device__ __forceinline__ float add_prob_pair(float acc, uint32_t packed) {
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), ones, acc, false);
}

// Per-lane constants of a kernel instance.
template <class T>
struct Lane {
  int lane, wave, l32, hh;
  int lrow;               // row of this lane inside a GROUP-row load round
  int kcol, vcol;         // byte column (swizzled chunk) this lane fetches for K / V
  uint32_t kvoff, vvoff;  // lrow * row_stride + column, the 32-bit per-lane part of a load address

  __device__ __forceinline__ void init(int tid, int64_t row_stride_b) {
    lane = tid & 63;
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    l32 = lane & 31;
    hh = lane >> 5;
    lrow = wave * T::RPI + lane / T::CPR;
    kcol = ((lane % T::CPR) ^ T::swz_k(lrow)) * 16;
    vcol = ((lane % T::CPR) ^ T::swz_v(lrow)) * 16;
    kvoff = (uint32_t)lrow * (uint32_t)row_stride_b + (uint32_t)kcol;
    vvoff = (uint32_t)lrow * (uint32_t)row_stride_b + (uint32_t)vcol;
  }

  // Operand addresses in the K / V buffers at k_base + K_OFF / v_base + V_OFF (recomputed per item: cheaper than
  // keeping a second copy live).
  //   ka[ks]: K operand chunk of k-step ks, 32-key block 0.   va[db]: V transpose read of d-block db, 16-key block 0.
  // V^T operand: lane (d = 32*db + lane%32, half hh) needs keys {k0 .. k0+3} and {k0+8 .. k0+11},
  // k0 = 32*kb + 16*u + 4*hh.  A transpose read returns, to lane i of a 16-lane group, element i%4 of
  // the 8 bytes addressed by lanes i/4 + {0,4,8,12} of the group; so the lane addresses row k0 + (i16/4),
  // columns 16*b + 4*(i16%4) .. +3 of the d-block and receives column 16*b + i16 of rows k0 .. k0+3.
  __device__ __forceinline__ void operand_addrs(uint32_t k_base, uint32_t v_base, int (&ka)[T::NKS], int (&va)[T::NDB]) const {
    const int i16 = lane & 15;
    const int b = (lane >> 4) & 1;
#pragma unroll
    for (int ks = 0; ks < T::NKS; ++ks) ka[ks] = (int)k_base + T::K_OFF + l32 * T::ROW_B + (((2 * ks + hh) ^ T::swz_k(l32)) * 16);
    const int row = 4 * hh + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < T::NDB; ++db) {
      const int chunk = 4 * db + 2 * b + ((i16 & 3) >> 1);
      va[db] = (int)v_base + T::V_OFF + row * T::ROW_B + ((chunk ^ T::swz_v(row)) * 16) + 8 * (i16 & 1);
    }
  }
};

// Direct HBM -> LDS load of this wave's share of one K or V tile into the tile buffer at LDS byte offset dst_off.
// base (start of the sequence's rows for this head), row_stride_b, key0 and kv_len are wave-uniform.  The address of a
// lane is  scalar tile base + 32-bit lane offset;  in the last tile of a sequence rows past the end re-read the last
// key (their scores are masked, and a finite V row times a zero probability adds nothing).
// One direct-load instruction: 64 lanes x 16 bytes from (sbase + voff[lane]) to LDS bytes [lds_addr, lds_addr + 1024).
// Written as inline assembly so that the compiler does not track it: it would otherwise make LDS reads that it
// cannot prove disjoint wait for every outstanding direct load.  Completion is awaited explicitly (wait_loads).
__device__ __forceinline__ void lds_dma_16(const char* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory");
}

// The last tile of a sequence may be partial.  If the sequence has at least BN keys the tile is loaded as the LAST BN
// keys of the sequence (rows [kv_len - BN, kv_len): an ordinary full-tile load, whose first rows repeat keys of the
// tile before and are masked out of the softmax); only a sequence shorter than one tile needs per-lane clamping.
// TailRows gives the valid row range of that last tile for the masks.
struct TailRows {
  int lo, hi;  // rows lo <= r < hi of the last tile are keys that no earlier tile holds
};
template <class T>
__device__ __forceinline__ TailRows tail_rows(int kv_len) {
  const int nt = (kv_len + T::BN - 1) / T::BN;
  const int keys_left = kv_len - (nt - 1) * T::BN;
  TailRows r;
  r.lo = kv_len >= T::BN ? T::BN - keys_left : 0;
  r.hi = kv_len >= T::BN ? T::BN : keys_left;
  return r;
}
// First key of tile ti (ti < number of tiles) as loaded; wave-uniform.
template <class T>
__device__ __forceinline__ int tile_first_key(int ti, int kv_len) {
  const int key0 = ti * T::BN;
  return (key0 + T::BN > kv_len && kv_len >= T::BN) ? kv_len - T::BN : key0;
}

// Rows past the end of a sequence shorter than a tile re-read its last key (their scores are masked, and a finite V
// row times a zero probability adds nothing).
// Load instruction i (0 .. LPT-1) of this wave's share of a tile that is known to be whole (every tile of a sequence
// of at least BN keys): rows i*GROUP + lrow, no branch.
template <class T>
__device__ __forceinline__ void tile_load_part_whole(const char* base, int64_t row_stride_b, int key0, uint32_t voff,
                                                     lds_char* smem, int dst_off, int wave, int i) {
  const char* sbase = base + (int64_t)(key0 + i * T::GROUP) * row_stride_b;  // scalar
  lds_dma_16(sbase, voff, (uint32_t)(uintptr_t)smem + (uint32_t)dst_off + (uint32_t)wave * 1024u + (uint32_t)(i * T::NWAVES * 1024));
}

// This wave's whole share of the tile that starts at key0 = tile_first_key(..): LPT instructions, one test.
template <class T>
__device__ __forceinline__ void tile_load_one(const char* base, int64_t row_stride_b, int key0, int kv_len, int lrow,
                                              int col, uint32_t voff, lds_char* smem, int dst_off, int wave) {
  const char* tbase = base + (int64_t)key0 * row_stride_b;  // scalar
  const uint32_t lds0 = (uint32_t)(uintptr_t)smem + (uint32_t)dst_off + (uint32_t)wave * 1024u;
  if (key0 + T::BN <= kv_len) {
#pragma unroll
    for (int i = 0; i < T::LPT; ++i) {
      const char* sbase = tbase + (int64_t)(i * T::GROUP) * row_stride_b;  // scalar
      lds_dma_16(sbase, voff, lds0 + i * T::NWAVES * 1024);
    }
  } else {
    const int last = kv_len - 1 - key0;  // >= 0
#pragma unroll
    for (int i = 0; i < T::LPT; ++i) {
      int row = i * T::GROUP + lrow;
      row = row < last ? row : last;
      const uint32_t off = (uint32_t)row * (uint32_t)row_stride_b + (uint32_t)col;
      lds_dma_16(tbase, off, lds0 + i * T::NWAVES * 1024);
    }
  }
}

template <int V>
struct IC {
  static constexpr int value = V;
};
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(IC<I>{});
    static_for<I + 1, N>(f);
  }
}

// An MFMA stream: optionally O^T += V^T P^T (V tile addressed by va), then steps [Q0, Q1) of S^T = K Q^T (K tile
// addressed by ka; step q is k-step q / NKB of key block q % NKB, and step 0 of a block starts it from zero).
// Operand reads run PD MFMAs ahead of their use, through a ring of PD operand registers.
// va_ and ka_ pass through the empty asm statements below, so they are taken by reference and stay in their registers
// (working on copies cost one move per address and tile).  Unrolling the tile loop over the buffer parity, with the
// buffer as an immediate offset of the LDS instructions and no address arithmetic per tile at all, was 3 % slower.
template <class T, bool DO_PV, int Q0, int Q1, int PD>
__device__ __forceinline__ void mfma_stream(lds_char* smem, int (&va_)[T::NDB], int (&ka_)[T::NKS],
                                            const uint32_t (&pb)[T::NKB][8], const bf16x8 (&qf)[T::NKS],
                                            f32x16 (&o)[T::NDB], f32x16 (&s)[T::NKB]) {
  constexpr int NPV = DO_PV ? T::NPV : 0;
  constexpr int NQK = Q1 - Q0;
  constexpr int N = NPV + NQK;
  static_assert(Q0 >= 0 && Q0 <= Q1 && Q1 <= T::NQK, "QK step range");
  bf16x8 frag[PD];

  auto load_step = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    if constexpr (J < NPV) {  // PV step J: kb = J / (2*NDB), u = (J / NDB) % 2, db = J % NDB
      constexpr int kb = J / (2 * T::NDB), u = (J / T::NDB) % 2, db = J % T::NDB;
      lds_char* p0 = (lds_char*)(uintptr_t)(uint32_t)(va_[db] + (32 * kb + 16 * u) * T::ROW_B);
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
      const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 8 * T::ROW_B));
      frag[J % PD] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {  // QK step: ks = q / NKB, kb = q % NKB (kb fastest: consecutive MFMAs use different accumulators)
      constexpr int q = Q0 + J - NPV, ks = q / T::NKB, kb = q % T::NKB;
      frag[J % PD] = *(lds_bf16x8*)(uintptr_t)(uint32_t)(ka_[ks] + kb * 32 * T::ROW_B);
    }
  };
  auto mfma_step = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    if constexpr (J < NPV) {
      constexpr int kb = J / (2 * T::NDB), u = (J / T::NDB) % 2, db = J % T::NDB;
      u32x4 pw = {pb[kb][4 * u], pb[kb][4 * u + 1], pb[kb][4 * u + 2], pb[kb][4 * u + 3]};
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[J % PD], __builtin_bit_cast(bf16x8, pw), o[db], 0, 0, 0);
    } else {
      constexpr int q = Q0 + J - NPV, ks = q / T::NKB, kb = q % T::NKB;
      if constexpr (ks == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[J % PD], qf[ks], zero, 0, 0, 0);
      } else {
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[J % PD], qf[ks], s[kb], 0, 0, 0);
      }
    }
  };

  // Order.  The compiler is free to hoist LDS reads far above their MFMAs (it would then hold every operand of the
  // stream in registers at once) and to reorder the two contractions.  An empty asm statement after each MFMA takes
  // the accumulator just written as input and passes the address register of the next read through: the read cannot
  // be issued before that MFMA, and volatile asm statements keep their order.  It emits no instruction.
  auto tie = [&](auto jc) {
    (void)s;
    (void)o;
    constexpr int J = decltype(jc)::value;   // MFMA just issued
    constexpr int R = J + PD;                // read to issue next
    if constexpr (R < N) {
      if constexpr (J < NPV) {
        constexpr int dbj = J % T::NDB;
        if constexpr (R < NPV) {
          asm volatile("" : "+v"(va_[R % T::NDB]) : "v"(o[dbj]));
        } else {
          asm volatile("" : "+v"(ka_[(Q0 + R - NPV) / T::NKB]) : "v"(o[dbj]));
        }
      } else {
        constexpr int kbj = (Q0 + J - NPV) % T::NKB;
        asm volatile("" : "+v"(ka_[(Q0 + R - NPV) / T::NKB]) : "v"(s[kbj]));
      }
    }
  };
  SCHED_FENCE();
  static_for<0, (PD < N ? PD : N)>([&](auto jc) { load_step(jc); });
  SCHED_FENCE();
  static_for<0, N>([&](auto jc) {
    constexpr int J = decltype(jc)::value;
    mfma_step(jc);
    tie(jc);
    if constexpr (J + PD < N) load_step(IC<J + PD>{});
    SCHED_FENCE();  // and the scheduler may not sink that read towards its use either
  });
  SCHED_FENCE();
}

// The MFMA stream of a matrix phase of the ping-pong kernel, which works through a pair of tiles per phase:
// O^T += V^T P^T for NPVS tiles of the V buffer addressed by va_ (tile 0, then tile 1), then S^T = K Q^T for NQKS tiles
// of the K buffer addressed by ka_ (k-step outermost, so a Q fragment serves NQKS * NKB consecutive MFMAs).  Between
// the two tiles' PV MFMAs the rescale that the second tile's softmax deferred is applied (grown != 0: rare), so that
// O^T sees exactly the sequence  (O a0 + P0 V0) a1 + P1 V1  of a tile-by-tile pass.  Operand reads run PD MFMAs ahead
// through a ring of registers, pinned in place as in mfma_stream.
template <class T, int NPVS, int NQKS, int PD>
__device__ __forceinline__ void pp_stream(int (&va_)[T::NDB], int (&ka_)[T::NKS], const uint32_t (&pb)[2][T::NKB][8],
                                          const bf16x8 (&qf)[T::NKS], f32x16 (&o)[T::NDB], f32x16 (&s)[2][T::NKB],
                                          uint64_t grown, float alpha1) {
  static_assert(NPVS >= 0 && NPVS <= 2 && (NQKS == 0 || NQKS == 2), "tiles per phase");
  constexpr int NPV = NPVS * T::NPV;
  constexpr int QW = NQKS * T::NKB;  // score accumulators that a k-step cycles through
  constexpr int N = NPV + NQKS * T::NQK;
  bf16x8 frag[PD];

  auto load_step = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    if constexpr (J < NPV) {
      constexpr int sub = J / T::NPV, j = J % T::NPV, kb = j / (2 * T::NDB), u = (j / T::NDB) % 2, db = j % T::NDB;
      lds_char* p0 = (lds_char*)(uintptr_t)(uint32_t)(va_[db] + sub * T::TILE_B + (32 * kb + 16 * u) * T::ROW_B);
      const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
      const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 8 * T::ROW_B));
      frag[J % PD] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
      constexpr int q = J - NPV, ks = q / QW, sub = (q % QW) / T::NKB, kb = q % T::NKB;
      frag[J % PD] = *(lds_bf16x8*)(uintptr_t)(uint32_t)(ka_[ks] + sub * T::TILE_B + kb * 32 * T::ROW_B);
    }
  };
  auto mfma_step = [&](auto jc) {
    constexpr int J = decltype(jc)::value;
    if constexpr (J < NPV) {
      constexpr int sub = J / T::NPV, j = J % T::NPV, kb = j / (2 * T::NDB), u = (j / T::NDB) % 2, db = j % T::NDB;
      u32x4 pw = {pb[sub][kb][4 * u], pb[sub][kb][4 * u + 1], pb[sub][kb][4 * u + 2], pb[sub][kb][4 * u + 3]};
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[J % PD], __builtin_bit_cast(bf16x8, pw), o[db], 0, 0, 0);
    } else {
      constexpr int q = J - NPV, ks = q / QW, sub = (q % QW) / T::NKB, kb = q % T::NKB;
      if constexpr (ks == 0) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s[sub][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[J % PD], qf[ks], zero, 0, 0, 0);
      } else {
        s[sub][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[J % PD], qf[ks], s[sub][kb], 0, 0, 0);
      }
    }
  };
  // The accumulator of MFMA J goes into an empty asm statement together with the address register of read J + PD, so
  // that the read cannot be issued before that MFMA (see mfma_stream).
  auto tie = [&](auto jc) {
    (void)s;
    (void)o;
    constexpr int J = decltype(jc)::value;
    constexpr int R = J + PD;
    if constexpr (R < N) {
      if constexpr (J < NPV) {
        constexpr int dbj = J % T::NDB;
        if constexpr (R < NPV) {
          asm volatile("" : "+v"(va_[R % T::NDB]) : "v"(o[dbj]));
        } else {
          asm volatile("" : "+v"(ka_[(R - NPV) / QW]) : "v"(o[dbj]));
        }
      } else {
        constexpr int qj = J - NPV;
        asm volatile("" : "+v"(ka_[(R - NPV) / QW]) : "v"(s[(qj % QW) / T::NKB][qj % T::NKB]));
      }
    }
  };
  SCHED_FENCE();
  static_for<0, (PD < N ? PD : N)>([&](auto jc) { load_step(jc); });
  SCHED_FENCE();
  static_for<0, N>([&](auto jc) {
    constexpr int J = decltype(jc)::value;
    mfma_step(jc);
    tie(jc);
    if constexpr (J + PD < N) load_step(IC<J + PD>{});
    SCHED_FENCE();
    if constexpr (NPVS == 2 && J == T::NPV - 1) {
      if (grown != 0) {
#pragma unroll
        for (int db = 0; db < T::NDB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][i] *= alpha1;
      }
      SCHED_FENCE();
    }
  });
  SCHED_FENCE();
}

// max(x[lane], x[lane ^ 32]) without going through LDS.  v_permlane32_swap exchanges the upper half of its first
// register with the lower half of its second: starting from two copies of x, the first ends up with the lower
// half-wave's values in all lanes and the second with the upper half-wave's.  Written as assembly: with the builtin
// the compiler drops the second result when both inputs are the same value.  (The instruction needs two wait states
// after a vector write of its operands.)
__device__ __forceinline__ float max_with_other_half(float x) {
  float lo = x, hi = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\tv_max_f32 %0, %0, %1" : "+v"(lo), "+v"(hi));
  return lo;
}

// How far (in the base-2 exponent) a tile's row maximum may exceed the row's reference value before the reference moves.
constexpr float kRescaleLog2 = 8.0f;

// Online softmax of one tile: scores s -> bf16 probabilities pb (B-operand order), reference max / sum, lazy rescale.
// Element i of block kb is key 32*kb + 8*(i/4) + 4*hh + (i%4) of the tile, for query lane%32.
// PHASED (the ping-pong kernel) leaves two things to the matrix phase that follows: the row sums (row_sum_burst below;
// a v_dot2c shares the matrix pipe and, issued here, would queue behind the MFMA stream that the other wavefront of the
// SIMD runs meanwhile: about 60 cycles each instead of 5), and, with DEFER (the second tile of a pair), the rescale of
// O^T and l, which in a tile-by-tile pass comes after the first tile's PV MFMAs and row sum.  The function returns the
// mask of rows whose reference moved (zero: nothing to do) and, with DEFER, their factors in alpha_out (1 for rows
// that stayed, and for every row when the mask is zero); m_ref is updated here in every variant.
template <class T, bool TAIL, bool PHASED = false, bool DEFER = false>
__device__ __forceinline__ uint64_t tile_softmax(f32x16 (&s)[T::NKB], int hh, TailRows rows, float c,
                                                 uint32_t (&pb)[T::NKB][8], f32x16 (&o)[T::NDB], float& m_ref,
                                                 float& l_run, float* alpha_out = nullptr) {
  static_assert(PHASED || !DEFER, "a deferred rescale needs the phased row sums");
  // Tail mask.  Element i of block kb is key 32 kb + 8 (i / 4) + (i % 4) + 4 hh: the key is dead (not a new key of this
  // tile) unless lo <= key < hi, tested as one unsigned compare of a compile-time constant against two per-lane
  // values.  (With the per-lane part folded into the key instead, the compiler keeps all 32 key indices of a lane
  // in registers across the whole kernel and turns the masking into branches around the exponentials.)
  const int tail_lo = rows.lo - 4 * hh;
  const unsigned tail_n = (unsigned)(rows.hi - rows.lo);
  auto dead = [&](int kb, int i) { return (unsigned)(32 * kb + 8 * (i >> 2) + (i & 3) - tail_lo) >= tail_n; };
  if (TAIL) {
#pragma unroll
    for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[kb][i] = dead(kb, i) ? -__builtin_inff() : s[kb][i];
  }

  // v_max3_f32 written out, one asm statement per block of 16 scores: through fmaxf the compiler first "quiets"
  // every operand it cannot prove canonical with a v_max_f32 x, x, x (MFMA results, asm results), six more
  // instructions per tile; and it pads every asm statement with an s_nop.
  float mx;
#define DIT_S(k, i) "v"(s[k][i])
  asm("v_max3_f32 %0, %1, %2, %3\n\tv_max3_f32 %0, %0, %4, %5\n\tv_max3_f32 %0, %0, %6, %7\n\t"
      "v_max3_f32 %0, %0, %8, %9\n\tv_max3_f32 %0, %0, %10, %11\n\tv_max3_f32 %0, %0, %12, %13\n\t"
      "v_max3_f32 %0, %0, %14, %15\n\tv_max_f32 %0, %0, %16"
      : "=&v"(mx)
      : DIT_S(0, 0), DIT_S(0, 1), DIT_S(0, 2), DIT_S(0, 3), DIT_S(0, 4), DIT_S(0, 5), DIT_S(0, 6), DIT_S(0, 7), DIT_S(0, 8),
        DIT_S(0, 9), DIT_S(0, 10), DIT_S(0, 11), DIT_S(0, 12), DIT_S(0, 13), DIT_S(0, 14), DIT_S(0, 15));
#pragma unroll
  for (int kb = 1; kb < T::NKB; ++kb)
    asm("v_max3_f32 %0, %0, %1, %2\n\tv_max3_f32 %0, %0, %3, %4\n\tv_max3_f32 %0, %0, %5, %6\n\t"
        "v_max3_f32 %0, %0, %7, %8\n\tv_max3_f32 %0, %0, %9, %10\n\tv_max3_f32 %0, %0, %11, %12\n\t"
        "v_max3_f32 %0, %0, %13, %14\n\tv_max3_f32 %0, %0, %15, %16"
        : "+v"(mx)
        : DIT_S(kb, 0), DIT_S(kb, 1), DIT_S(kb, 2), DIT_S(kb, 3), DIT_S(kb, 4), DIT_S(kb, 5), DIT_S(kb, 6), DIT_S(kb, 7),
          DIT_S(kb, 8), DIT_S(kb, 9), DIT_S(kb, 10), DIT_S(kb, 11), DIT_S(kb, 12), DIT_S(kb, 13), DIT_S(kb, 14),
          DIT_S(kb, 15));
#undef DIT_S
  mx = max_with_other_half(mx);

  // The reference value m_ref of a row follows its running maximum lazily: it moves (and O^T and l are rescaled) only
  // when the tile's maximum exceeds it by more than kRescaleLog2 in the exponent, so probabilities lie in
  // (0, 2^kRescaleLog2] instead of (0, 1] — the quotient O / l does not depend on the reference.  The decision is per
  // row (a row that stays has alpha = 1 exactly), so the result does not depend on which rows share a wavefront.
  // (Taking the probabilities first and looking for the maximum only when a sum shows that the reference was too low
  // was measured 3 % slower, although it issues twenty vector instructions fewer per tile.)
  const bool grow = (mx - m_ref) * c > kRescaleLog2;
  const uint64_t grown = __builtin_amdgcn_ballot_w64(grow);
  if constexpr (DEFER) *alpha_out = 1.0f;
  if (grown != 0) {
    const float m_new = grow ? mx : m_ref;
    const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);
    m_ref = m_new;
    if constexpr (DEFER) {
      *alpha_out = alpha;
    } else {
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < T::NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
  }
  const float mc = m_ref * c;

  // Eight scores at a time, with a scheduling fence after each group: the probabilities are packed to bf16 and
  // their fp32 values die before the next group starts, which keeps the register peak of this phase low.
  float lsum = 0.f;
#pragma unroll
  for (int kb = 0; kb < T::NKB; ++kb) {
#pragma unroll
    for (int g = 0; g < 2; ++g) {
#pragma unroll
      for (int i = 8 * g; i < 8 * g + 8; i += 2) {
        float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i], c, -mc));
        float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i + 1], c, -mc));
        pb[kb][i >> 1] = pack_bf16x2(p0, p1);  // a dead key: score -inf, c > 0 (AttnParams::c_log2), probability 0
        if constexpr (!PHASED) lsum = add_prob_pair(lsum, pb[kb][i >> 1]);
      }
      SCHED_FENCE();
    }
  }
  if constexpr (!PHASED) {
    l_run += lsum;
  } else {
    // Everything above is finished here: the compiler otherwise sinks the exponentials of a tile towards their first
    // use, which lies behind a barrier, inside the matrix phase.
#pragma unroll
    for (int kb = 0; kb < T::NKB; ++kb)
      asm volatile("" : "+v"(pb[kb][0]), "+v"(pb[kb][1]), "+v"(pb[kb][2]), "+v"(pb[kb][3]), "+v"(pb[kb][4]), "+v"(pb[kb][5]),
                        "+v"(pb[kb][6]), "+v"(pb[kb][7]));
    asm volatile("" : "+v"(l_run), "+v"(m_ref));
  }
  return grown;
}

// The row sum of one tile's rounded probabilities, in the order tile_softmax adds them: one chain of v_dot2c, issued
// back to back.  The ping-pong kernel calls it at the end of a wavefront's matrix phase, when the matrix pipe of the
// SIMD is this wavefront's own.
template <class T>
__device__ __forceinline__ float row_sum_burst(const uint32_t (&pb)[T::NKB][8]) {
  float lsum = 0.f;
#pragma unroll
  for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
    for (int i = 0; i < 8; ++i) lsum = add_prob_pair(lsum, pb[kb][i]);
  return lsum;
}

// All LDS accesses of this wave are complete, then workgroup barrier.  The "memory" clobber keeps the
// compiler from moving LDS reads or direct loads across it.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// Waits until at most N of this wavefront's vector-memory operations (the youngest N) are outstanding.
template <int N>
__device__ __forceinline__ void wait_loads_but() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
// Workgroup barrier that does not wait for this wave's outstanding LDS reads: for a point where the buffers those
// reads address are not written by anyone before the next barrier.
__device__ __forceinline__ void phase_barrier() { asm volatile("s_barrier" ::: "memory"); }

// Work distribution: workgroup b starts with list index b; further indices come from one atomic counter (thread 0
// of a workgroup), offset by the grid size; indices at or past n_items end the workgroup.  A workgroup asks for its
// next index only towards the end of the current item (two tiles before it ends): asking earlier hides no more latency
// and takes an item away from workgroups that become idle before this one gets to it (with one item per workgroup and
// the request made at the start of an item, the first workgroups to start took two items each and the last none).
__device__ __forceinline__ uint32_t take_item(const AttnParams& p) { return gridDim.x + atomicAdd(&p.sync[0], 1u); }
// After the item loop: the last workgroup to get here clears both words for the next launch.
__device__ __forceinline__ void finish_workgroup(const AttnParams& p) {
  __threadfence();
  const uint32_t done = atomicAdd(&p.sync[1], 1u);
  if (done == gridDim.x - 1) {
    p.sync[0] = 0u;
    p.sync[1] = 0u;
  }
}

// Clock sample of a launch: workgroup 0 (persistent, so it lives about as long as the kernel) reads the shader-cycle
// counter and the constant 100 MHz counter when it starts and when it ends, and leaves the two differences in
// sync[2..5].  Their ratio is the shader clock the chip sustained under this kernel.
struct LaunchClock {
  uint64_t cycles, ticks;
};
__device__ __forceinline__ LaunchClock launch_clock_begin() {
  LaunchClock c;
  c.cycles = __builtin_readcyclecounter();
  c.ticks = __builtin_amdgcn_s_memrealtime();
  return c;
}
__device__ __forceinline__ void launch_clock_end(const AttnParams& p, const LaunchClock& c0) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint64_t* out = reinterpret_cast<uint64_t*>(p.sync + 2);
    out[0] = __builtin_readcyclecounter() - c0.cycles;
    out[1] = __builtin_amdgcn_s_memrealtime() - c0.ticks;
  }
}

// Work item fields, wave-uniform.
struct ItemU {
  int q_start, kv_start, kv_len, head, q_rows, part;
};
// The record comes through a scalar load (idx is the same in every lane): scalar loads are counted apart from the
// vector-memory operations, so the first thing an item does is not a wait for the output stores of the item before it
// (a vector load here cost a wavefront 3 000 to 6 000 cycles per item).  The list is written before the launch (by the
// host or by the kernel before this one on the stream) and never during it.
__device__ __forceinline__ ItemU fetch_item(const WorkItem* items, uint32_t idx) {
  const WorkItem* rec = items + idx;
  u32x4 w;
  asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(w) : "s"(rec) : "memory");
  ItemU u;
  u.q_start = (int)w[0];
  u.kv_start = (int)w[1];
  u.kv_len = (int)w[2];
  const int rh = (int)w[3];
  u.head = rh & 0xFFFF;
  u.q_rows = (rh >> 16) & 0xFFF;
  u.part = (rh >> 28) & 0xF;
  return u;
}

// Q fragments (B operand of S^T = K Q^T): lane holds query row l32 of its wave, d = 16*ks + 8*hh .. +7.
template <class T>
__device__ __forceinline__ void load_q(const AttnParams& p, const Lane<T>& L, const ItemU& it, int64_t row_stride_b,
                                       int64_t head_off, int qrow, bf16x8 (&qf)[T::NKS]) {
  const char* qptr = static_cast<const char*>(p.q) + (int64_t)(it.q_start + qrow) * row_stride_b + head_off + L.hh * 16;
#pragma unroll
  for (int ks = 0; ks < T::NKS; ++ks) {
    u32x4 w = *reinterpret_cast<const u32x4*>(qptr + ks * 32);
    if (p.negate) w ^= u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
    qf[ks] = __builtin_bit_cast(bf16x8, w);
  }
}

// Epilogue: O^T / l -> bf16 -> out, and, if asked for, lse = ln sum_j exp(scale * s_j) = ln 2 * (c * m + log2 l).
// Lane holds d = 32*db + 8*g + 4*hh + j (i = 4*g + j) of query l32: eight bytes of each of 32 rows per store
// instruction if stored from there, 32 partly written cache lines each time, sixteen times per wavefront.  That cost
// 4 % of an item of 4352 keys and 29 % of a cross-attention item of 512 keys (measured by leaving the stores out).  The
// rows therefore go through `stage`, 32 * ROW_B bytes of LDS that belong to this wavefront at this point (the caller
// names a K / V buffer that nobody reads or loads into until the next barrier): written in the accumulator layout,
// 16-byte chunk c of row r at chunk c ^ (r mod chunks per row) so that the 32 rows of a write spread over the banks,
// and read back as whole rows, so that a store instruction writes 1 KB of whole rows (four rows at head dimension 128).
template <class T>
__device__ __forceinline__ void store_out(const AttnParams& p, const Lane<T>& L, const ItemU& it, int64_t row_stride_b,
                                          int64_t head_off, int qrow, bool row_valid, const f32x16 (&o)[T::NDB],
                                          float l_run, float m_ref, uint32_t stage) {
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (p.part_out != nullptr) {
    // split-KV: this item saw one chunk of the keys; its normalised result and lse go to the workspace in fp32
    if (!row_valid) return;
    const float inv = 1.0f / l_tot;
    const int64_t rh = ((int64_t)it.part * p.part_rows + it.q_start + qrow) * p.n_heads + it.head;
    float* optr = p.part_out + rh * T::D + L.hh * 4;
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
        *reinterpret_cast<f32x4*>(optr + 32 * db + 8 * g) =
            f32x4{o[db][4 * g + 0] * inv, o[db][4 * g + 1] * inv, o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv};
      }
    if (L.hh == 0) p.part_lse[rh] = 0.69314718055994530942f * (m_ref * p.c_log2 + __builtin_amdgcn_logf(l_tot));
    return;
  }
  {
    typedef __attribute__((address_space(3))) u32x2 lds_u32x2;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
    constexpr int CH = T::ROW_B / 16;  // 16-byte chunks of a row
    static_assert(4 * T::NDB == CH && 64 % CH == 0, "a row is NDB blocks of four chunks");
    const float inv = 1.0f / l_tot;  // rows past the end of a ragged tile hold a copy of the last row: finite, not stored
    const uint32_t wr = stage + (uint32_t)(L.l32 * T::ROW_B + L.hh * 8);
    const uint32_t wsw = (uint32_t)(L.l32 & (CH - 1)) * 16u;
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 w;
        w[0] = pack_bf16x2(o[db][4 * g + 0] * inv, o[db][4 * g + 1] * inv);
        w[1] = pack_bf16x2(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
        *(lds_u32x2*)(uintptr_t)(wr + ((uint32_t)((4 * db + g) * 16) ^ wsw)) = w;
      }
    // LDS serves a wavefront's instructions in order: the reads below see the writes above, of other lanes too.
    asm volatile("" ::: "memory");
    __builtin_amdgcn_wave_barrier();
    constexpr int RPS = 64 / CH;  // rows per store instruction
    const int ch = L.lane & (CH - 1), r0 = L.lane / CH;
    const int row0 = L.wave * 32 + r0;  // row of the item's query tile
    char* optr = static_cast<char*>(p.out) + (int64_t)(it.q_start + row0) * row_stride_b + head_off + ch * 16;
    u32x4 w[32 / RPS];
#pragma unroll
    for (int i = 0; i < 32 / RPS; ++i) {
      const int r = r0 + i * RPS;
      w[i] = *(lds_u32x4*)(uintptr_t)(stage + (uint32_t)(r * T::ROW_B + ((ch ^ (r & (CH - 1))) * 16)));
    }
#pragma unroll
    for (int i = 0; i < 32 / RPS; ++i) asm volatile("" : "+v"(w[i]));  // all reads are issued before the first store
    const int n_valid = it.q_rows - row0;
#pragma unroll
    for (int i = 0; i < 32 / RPS; ++i)
      if (i * RPS < n_valid)  // streaming stores: the rows are not read again by this call
        __builtin_nontemporal_store(w[i], reinterpret_cast<u32x4*>(optr + (int64_t)(i * RPS) * row_stride_b));
    if (row_valid && p.lse != nullptr && L.hh == 0)
      p.lse[(int64_t)(it.q_start + qrow) * p.n_heads + it.head] = 0.69314718055994530942f * (m_ref * p.c_log2 + __builtin_amdgcn_logf(l_tot));
  }
}

// Per-item state shared by both kernels.
template <class T>
struct ItemCtx {
  ItemU it;
  int nt;
  int64_t head_off;
  const char* kbase;
  const char* vbase;
  int qrow;
  int row_valid;  // 0 or 1 (an int, so that the struct has no padding bytes to copy around)
};

template <class T>
__device__ __forceinline__ ItemCtx<T> item_ctx(const AttnParams& p, const Lane<T>& L, const ItemU& it, int64_t row_stride_b) {
  ItemCtx<T> c;
  c.it = it;
  c.nt = (c.it.kv_len + T::BN - 1) / T::BN;
  c.head_off = (int64_t)c.it.head * T::D * 2;
  c.kbase = static_cast<const char*>(p.k) + (int64_t)c.it.kv_start * row_stride_b + c.head_off;
  c.vbase = static_cast<const char*>(p.v) + (int64_t)c.it.kv_start * row_stride_b + c.head_off;
  // Waves whose 32 rows lie past the end of a ragged query tile work on a copy of the last row and store nothing.
  c.qrow = L.wave * 32 + L.l32;
  c.row_valid = c.qrow < c.it.q_rows;
  if (!c.row_valid) c.qrow = c.it.q_rows - 1;
  return c;
}

template <class T>
__device__ __forceinline__ ItemCtx<T> begin_item(const AttnParams& p, const Lane<T>& L, uint32_t item_idx,
                                                 int64_t row_stride_b) {
  return item_ctx<T>(p, L, fetch_item(p.items, item_idx), row_stride_b);
}

}  // namespace dit
