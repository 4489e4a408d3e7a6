// DiT denoising-step self-attention forward for gfx950 (MI355X).
//
// O[r,h,:] = sum_j softmax_j(scale * <Q[r,h,:], K[j,h,:]>) V[j,h,:], j over the
// keys of r's own sequence (paper Sections 4.3 and 5 give the batch; the math is
// plain softmax attention).  bf16 in, fp32 scores/state/accumulators, bf16 out.
//
// Mapping.  A persistent workgroup of NWAVES wavefronts takes (sequence, head,
// query tile) items from a list through one atomic counter.  Each wavefront owns
// 32 query rows.  K and V tiles of BN keys are copied HBM -> LDS by direct
// (register-free) loads, double buffered, one barrier per tile.  Both
// contractions run on the 32x32x16 bf16 MFMA in *transposed* form:
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
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(1))) const void gptr_void;

// O^T and the running sum are rescaled only in tiles where the maximum of some row of the wavefront
// grows.  The reference maximum is always the true running maximum, so the largest probability of a
// row is exactly 1 and is not perturbed by the bf16 rounding of P (a row dominated by one key then
// returns that key's V row exactly; a stale reference would cost up to 2^-9 relative there).

template <int D_, int NWAVES_, int BN_>
struct Tile {
  static constexpr int D = D_;
  static constexpr int NWAVES = NWAVES_;
  static constexpr int BN = BN_;
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
  static constexpr int LDS_BYTES = 4 * TILE_B + 16;
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

// Issue the direct HBM -> LDS loads of one K tile and one V tile (this wave's share).
// koff / voff: per-lane byte offset of (row lrow, swizzled chunk) relative to a GROUP-row block.
template <class T, bool TAIL>
__device__ __forceinline__ void tile_load(const char* __restrict__ kbase, const char* __restrict__ vbase,
                                          int64_t row_stride_b, int key0, int kv_len, int lrow, int kcol, int vcol,
                                          lds_char* kdst, lds_char* vdst, int wave) {
#pragma unroll
  for (int i = 0; i < T::LPT; ++i) {
    int row = key0 + i * T::GROUP + lrow;
    if (TAIL) row = row < kv_len ? row : kv_len - 1;  // rows past the end re-read the last key; they are masked
    const int64_t roff = (int64_t)row * row_stride_b;
    lds_char* kd = kdst + (i * T::NWAVES + wave) * 1024;
    lds_char* vd = vdst + (i * T::NWAVES + wave) * 1024;
    __builtin_amdgcn_global_load_lds((gptr_void*)(kbase + roff + kcol), (__attribute__((address_space(3))) void*)kd, 16, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr_void*)(vbase + roff + vcol), (__attribute__((address_space(3))) void*)vd, 16, 0, 0);
  }
}

// One K/V tile: S^T = K Q^T, online softmax, O^T += V^T P^T.
// kaddr[ks]: per-lane LDS byte offset of the K operand chunk of k-step ks inside a 32-key block.
// vaddr[db]: per-lane LDS byte offset of the V transpose read of d-block db inside a 16-key block.
template <class T, bool TAIL>
__device__ __forceinline__ void tile_compute(lds_char* kbuf, lds_char* vbuf, int hh, int keys_left, float c,
                                             const int (&kaddr)[T::NKS], const int (&vaddr)[T::NDB],
                                             const bf16x8 (&qf)[T::NKS], f32x16 (&o)[T::NDB], float& m_ref,
                                             float& l_run) {
  f32x16 s[T::NKB];
#pragma unroll
  for (int kb = 0; kb < T::NKB; ++kb) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < T::NKS; ++ks) {
      const bf16x8 a = *(lds_bf16x8*)(kbuf + kaddr[ks] + kb * 32 * T::ROW_B);
      s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[kb], 0, 0, 0);
    }
  }

  // key index inside the tile of element i of block kb: 32*kb + 8*(i/4) + 4*hh + (i%4)
  if (TAIL) {
#pragma unroll
    for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int key = 32 * kb + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (key >= keys_left) s[kb][i] = -__builtin_inff();
      }
  }

  float mx = s[0][0];
#pragma unroll
  for (int kb = 0; kb < T::NKB; ++kb)
#pragma unroll
    for (int i = 0; i < 16; ++i) mx = __builtin_fmaxf(mx, s[kb][i]);
  mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32));

  // Rescale only if the running maximum of some row of this wave grew (rare after the first tiles).
  const bool grow = mx > m_ref;
  if (__builtin_amdgcn_ballot_w64(grow) != 0) {
    const float m_new = __builtin_fmaxf(m_ref, mx);
    const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c);
    m_ref = m_new;
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
  }
  const float mc = m_ref * c;

  float lsum = 0.f;
  uint32_t pb[T::NKB][8];
#pragma unroll
  for (int kb = 0; kb < T::NKB; ++kb) {
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
      float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i], c, -mc));
      float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][i + 1], c, -mc));
      if (TAIL) {
        const int key = 32 * kb + 8 * (i >> 2) + 4 * hh + (i & 3);
        if (key >= keys_left) p0 = 0.f;
        if (key + 1 >= keys_left) p1 = 0.f;
      }
      lsum += p0 + p1;
      pb[kb][i >> 1] = pack_bf16x2(p0, p1);
    }
  }
  l_run += lsum;

  // V^T operand: lane (d = 32*db + lane%32, half hh) needs keys {k0 .. k0+3} and {k0+8 .. k0+11},
  // k0 = 32*kb + 16*u + 4*hh.  A transpose read returns, to lane i of a 16-lane group, element i%4 of
  // the 8 bytes addressed by lanes i/4 + {0,4,8,12} of the group; so the lane addresses row k0 + (i16/4),
  // columns 16*b + 4*(i16%4) .. +3 of the d-block and receives column 16*b + i16 of rows k0 .. k0+3.
#pragma unroll
  for (int kb = 0; kb < T::NKB; ++kb) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      u32x4 pw = {pb[kb][4 * u], pb[kb][4 * u + 1], pb[kb][4 * u + 2], pb[kb][4 * u + 3]};
      const bf16x8 pfrag = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
      for (int db = 0; db < T::NDB; ++db) {
        lds_char* p0 = vbuf + vaddr[db] + (32 * kb + 16 * u) * T::ROW_B;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)(p0 + 8 * T::ROW_B));
        const bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pfrag, o[db], 0, 0, 0);
      }
    }
  }
}

template <class T>
__global__ void __attribute__((amdgpu_flat_work_group_size(T::NT, T::NT), amdgpu_waves_per_eu(2, 2)))
attn_fwd_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(1024))) char smem_generic[];
  // LDS: [K0][V0][K1][V1][item index]
  lds_char* smem = (lds_char*)smem_generic;
  volatile uint32_t* s_item = reinterpret_cast<volatile uint32_t*>(smem_generic + 4 * T::TILE_B);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;
  const int hh = lane >> 5;
  const int i16 = lane & 15;
  const int b = (lane >> 4) & 1;
  const int64_t row_stride_b = (int64_t)p.n_heads * T::D * 2;
  const float c = p.c_log2;

  // Loader lane constants: row inside a GROUP-row round and the global chunk this lane fetches.
  const int lrow = wave * T::RPI + lane / T::CPR;
  const int kcol = ((lane % T::CPR) ^ T::swz_k(lrow)) * 16;
  const int vcol = ((lane % T::CPR) ^ T::swz_v(lrow)) * 16;

  // Reader lane constants.
  int kaddr[T::NKS];
#pragma unroll
  for (int ks = 0; ks < T::NKS; ++ks) kaddr[ks] = l32 * T::ROW_B + (((2 * ks + hh) ^ T::swz_k(l32)) * 16);
  int vaddr[T::NDB];
  {
    const int row = 4 * hh + (i16 >> 2);
#pragma unroll
    for (int db = 0; db < T::NDB; ++db) {
      const int chunk = 4 * db + 2 * b + ((i16 & 3) >> 1);
      vaddr[db] = row * T::ROW_B + ((chunk ^ T::swz_v(row)) * 16) + 8 * (i16 & 1);
    }
  }

  for (;;) {
    if (tid == 0) *s_item = atomicAdd(p.counter, 1u) - p.counter_base;
    __syncthreads();
    const uint32_t item_idx = *s_item;
    if (item_idx >= p.n_items) break;
    const WorkItem it = p.items[item_idx];
    const int head = it.rows_head & 0xFFFF;
    const int q_rows = (it.rows_head >> 16) & 0xFFFF;
    const int kv_len = it.kv_len;
    const int nt = (kv_len + T::BN - 1) / T::BN;
    const int64_t head_off = (int64_t)head * T::D * 2;
    const char* kbase = static_cast<const char*>(p.k) + (int64_t)it.kv_start * row_stride_b + head_off;
    const char* vbase = static_cast<const char*>(p.v) + (int64_t)it.kv_start * row_stride_b + head_off;

    // Tile 0 -> buffer 0 (every wave is past the previous item's last read of it: see the barrier above).
    if (nt == 1) tile_load<T, true>(kbase, vbase, row_stride_b, 0, kv_len, lrow, kcol, vcol, smem, smem + T::TILE_B, wave);
    else tile_load<T, false>(kbase, vbase, row_stride_b, 0, kv_len, lrow, kcol, vcol, smem, smem + T::TILE_B, wave);

    // Q fragments (B operand): lane holds query row l32 of this wave, d = 16*ks + 8*hh .. +7.
    int qrow = wave * 32 + l32;
    const bool row_valid = qrow < q_rows;
    if (!row_valid) qrow = q_rows - 1;
    const char* qptr = static_cast<const char*>(p.q) + (int64_t)(it.q_start + qrow) * row_stride_b + head_off + hh * 16;
    bf16x8 qf[T::NKS];
#pragma unroll
    for (int ks = 0; ks < T::NKS; ++ks) {
      u32x4 w = *reinterpret_cast<const u32x4*>(qptr + ks * 32);
      if (p.negate) w ^= u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
      qf[ks] = __builtin_bit_cast(bf16x8, w);
    }

    f32x16 o[T::NDB];
#pragma unroll
    for (int db = 0; db < T::NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
    float m_ref = -1.0e30f;  // finite, so that (m_ref - m) * 0 is 0 when scale is 0
    float l_run = 0.f;

    const bool wave_active = wave * 32 < q_rows;
    for (int t = 0; t < nt; ++t) {
      lds_char* kcur = smem + (t & 1) * (2 * T::TILE_B);
      lds_char* knxt = smem + ((t & 1) ^ 1) * (2 * T::TILE_B);
      // Tile t has landed (this wave's loads), and after the barrier everyone's; everyone is also done
      // reading the other buffer (tile t-1), so it can be refilled with tile t+1 while tile t is used.
      __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
      __syncthreads();
      if (t + 1 < nt) {
        if (t + 2 == nt) tile_load<T, true>(kbase, vbase, row_stride_b, (t + 1) * T::BN, kv_len, lrow, kcol, vcol, knxt, knxt + T::TILE_B, wave);
        else tile_load<T, false>(kbase, vbase, row_stride_b, (t + 1) * T::BN, kv_len, lrow, kcol, vcol, knxt, knxt + T::TILE_B, wave);
      }
      if (wave_active) {
        const int keys_left = kv_len - t * T::BN;
        if (keys_left >= T::BN) tile_compute<T, false>(kcur, kcur + T::TILE_B, hh, keys_left, c, kaddr, vaddr, qf, o, m_ref, l_run);
        else tile_compute<T, true>(kcur, kcur + T::TILE_B, hh, keys_left, c, kaddr, vaddr, qf, o, m_ref, l_run);
      }
    }

    // Epilogue: O^T / l -> bf16 -> out.  Lane holds d = 32*db + 8*g + 4*hh + j (i = 4*g + j) of query l32.
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    if (row_valid) {
      const float inv = 1.0f / l_tot;
      char* optr = static_cast<char*>(p.out) + (int64_t)(it.q_start + qrow) * row_stride_b + head_off + hh * 8;
#pragma unroll
      for (int db = 0; db < T::NDB; ++db)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          u32x2 w;
          w[0] = pack_bf16x2(o[db][4 * g + 0] * inv, o[db][4 * g + 1] * inv);
          w[1] = pack_bf16x2(o[db][4 * g + 2] * inv, o[db][4 * g + 3] * inv);
          *reinterpret_cast<u32x2*>(optr + (32 * db + 8 * g) * 2) = w;
        }
    }
    // The next item's first loads overwrite buffer 0 and the item slot: wait until every wave has left the tile loop.
    __syncthreads();
  }
}

template <class T>
static hipError_t launch_t(const AttnParams& p, int grid, hipStream_t stream) {
  static bool attr_set[16] = {};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16 || !attr_set[dev]) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<T>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            T::LDS_BYTES);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 16) attr_set[dev] = true;
  }
  hipLaunchKernelGGL(attn_fwd_kernel<T>, dim3(grid), dim3(T::NT), T::LDS_BYTES, stream, p);
  return hipGetLastError();
}

int attn_fwd_block_m(int head_dim) {
  (void)head_dim;
  return 128;
}
int attn_fwd_wgs_per_cu(int head_dim) {
  (void)head_dim;
  return 2;
}

hipError_t attn_fwd_launch(const AttnParams& p, int head_dim, int grid, hipStream_t stream) {
  if (head_dim == 128) return launch_t<Tile<128, 4, 64>>(p, grid, stream);
  if (head_dim == 64) return launch_t<Tile<64, 4, 64>>(p, grid, stream);
  return hipErrorInvalidValue;
}

}  // namespace dit
