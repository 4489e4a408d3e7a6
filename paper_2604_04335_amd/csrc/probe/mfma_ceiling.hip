// What the matrix pipes of this chip deliver, alone and beside the other work of an attention tile: a register-only
// stream of v_mfma_f32_32x32x16_bf16 on every compute unit, operands with the bit activity of the attention kernels'
// data (pseudo-random bf16 of unit scale; all-zero operands would let the chip hold its full clock, which real data
// does not), optionally with the LDS operand reads and the vector instructions that an attention kernel issues per
// MFMA.  The extra work feeds nothing into the MFMAs, so their data activity is the same in every mix, and there are
// no barriers, no loads from memory, no dependent chains and no item boundaries: each mix is an upper bound for a
// kernel of that shape.  The attention numbers are read against these figures as well as against the nominal peak.
//
// This is a measurement aid of bench.py, not part of the attention library: it is built into its own shared object
// (libdit_probe.so) with the one C entry point at the end of this file, and nothing in libdit_attn.so refers to it.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dit {

constexpr int kCeilingMfmaPerIter = 16;            // MFMAs a wavefront issues per loop iteration
constexpr int kCeilingMfmaPerWave = 131072;        // MFMAs per wavefront at two wavefronts per SIMD (twice that at one)
constexpr int kCeilingWavesPerCu = 8;              // two per SIMD, as in the ping-pong attention kernel
constexpr double kCeilingFlopPerMfma = 2.0 * 32 * 32 * 16;
constexpr int kCeilingMixes = 6;                   // mixes 0 .. 5

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kLdsChunks = 4096;  // 64 KB of 16-byte chunks

__device__ __forceinline__ uint32_t mix_bits(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}

// A value in (-2, 2) with a random mantissa.
__device__ __forceinline__ __bf16 unit_scale_value(uint32_t h) {
  return (__bf16)((float)(int32_t)(h & 0xffffu) * (1.0f / 16384.0f) - 2.0f);
}

// Per kCeilingMfmaPerIter MFMAs: LDSN ds_read_b128 (1 KB each per wavefront), VALN v_fma_f32, EXPN v_exp_f32.
template <int LDSN, int VALN, int EXPN>
__global__ void __launch_bounds__(512) mfma_ceiling_kernel(uint64_t* sample, float* sink, int iters) {
  __shared__ u32x4 lds[LDSN ? kLdsChunks : 1];
  if (LDSN) {
    for (int i = threadIdx.x; i < kLdsChunks; i += blockDim.x) {
      const u32x4 t = {mix_bits(i * 4u), mix_bits(i * 4u + 1), mix_bits(i * 4u + 2), mix_bits(i * 4u + 3)};
      lds[i] = t;
    }
    __syncthreads();
  }
  const uint64_t c0 = __builtin_readcyclecounter(), t0 = __builtin_amdgcn_s_memrealtime();
  const uint32_t id = blockIdx.x * 512u + threadIdx.x;
  bf16x8 a[4], b[4];
  for (int r = 0; r < 4; ++r)
    for (int i = 0; i < 8; ++i) {
      a[r][i] = unit_scale_value(mix_bits(id * 64u + r * 8u + i));
      b[r][i] = unit_scale_value(mix_bits(id * 64u + 32u + r * 8u + i));
    }
  f32x16 acc[4] = {};
  float x[8];
  for (int i = 0; i < 8; ++i) x[i] = 0.37f + 0.01f * (float)((id + i) & 63);
  const float m1 = 0.999f + 1e-5f * (float)(id & 15), m2 = 1e-4f;
  // Conflict-free 16-byte reads: lane l takes bytes 16 l .. 16 l + 15 of a 1 KB row; wavefront w starts at row w, the
  // immediate offset adds up to 7 rows, the iteration one of four 16 KB quarters:
  // 3 * 16384 + 7 * 1024 + 7 * 1024 + 1023 < 65536.
  const uint32_t addr = (uint32_t)(uintptr_t)lds + (threadIdx.x & 63) * 16u + (threadIdx.x >> 6) * 1024u;
  for (int it = 0; it < iters; ++it) {
    const uint32_t base = addr + ((uint32_t)it & 3u) * 16384u;
#pragma unroll
    for (int j = 0; j < kCeilingMfmaPerIter; ++j) {
      acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(j >> 2) & 3], b[j & 3], acc[j & 3], 0, 0, 0);
#pragma unroll
      for (int r = j * LDSN / kCeilingMfmaPerIter; r < (j + 1) * LDSN / kCeilingMfmaPerIter; ++r) {
        u32x4 tmp;
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(tmp) : "v"(base), "n"((r & 7) * 1024));
      }
#pragma unroll
      for (int r = j * VALN / kCeilingMfmaPerIter; r < (j + 1) * VALN / kCeilingMfmaPerIter; ++r)
        x[r & 7] = __builtin_fmaf(x[r & 7], m1, m2);
#pragma unroll
      for (int r = j * EXPN / kCeilingMfmaPerIter; r < (j + 1) * EXPN / kCeilingMfmaPerIter; ++r)
        x[r & 7] = __builtin_amdgcn_exp2f(-x[r & 7]);  // x -> 2^-x stays in (0, 1]; the negation is an operand modifier
    }
    if (LDSN) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  float s = 0.f;
  for (int r = 0; r < 4; ++r)
    for (int i = 0; i < 16; ++i) s += acc[r][i];
  for (int i = 0; i < 8; ++i) s += x[i];
  if (s == 123.456f) sink[threadIdx.x & 63] = s;  // never true in practice; keeps the streams from being removed
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    sample[0] = __builtin_readcyclecounter() - c0;
    sample[1] = __builtin_amdgcn_s_memrealtime() - t0;
  }
}

template <int LDSN, int VALN, int EXPN>
void launch(int waves_per_cu, uint64_t* sample, float* sink, int n_cus, hipStream_t stream) {
  const int iters = kCeilingMfmaPerWave / kCeilingMfmaPerIter * (kCeilingWavesPerCu / waves_per_cu);
  hipLaunchKernelGGL((mfma_ceiling_kernel<LDSN, VALN, EXPN>), dim3(n_cus), dim3(waves_per_cu * 64), 0, stream, sample, sink, iters);
}

}  // namespace

// Every compute unit issues kCeilingWavesPerCu * kCeilingMfmaPerWave register-only MFMAs, with the LDS reads and vector
// instructions of `mix` beside them.  sample: device, 2 x uint64, receives the shader-cycle and 100 MHz-counter
// differences over the run of workgroup 0's first wavefront.  sink: device, >= 64 floats (never written in practice;
// it keeps the results alive).
static hipError_t mfma_ceiling_launch(int mix, uint64_t* sample, float* sink, int n_cus, hipStream_t stream) {
  // Per MFMA of a 32-row wavefront the ping-pong attention kernel issues 1 KB of LDS operand reads, 3.25 vector
  // instructions (of its 136 per 32 MFMAs, one fma each here) and one v_exp_f32.
  switch (mix) {
    case 0: launch<0, 0, 0>(8, sample, sink, n_cus, stream); break;     // MFMAs only
    case 1: launch<16, 52, 16>(8, sample, sink, n_cus, stream); break;  // the ping-pong kernel's mix
    case 2: launch<16, 0, 0>(8, sample, sink, n_cus, stream); break;    // its LDS reads only
    case 3: launch<0, 52, 16>(8, sample, sink, n_cus, stream); break;   // its vector instructions only
    case 4: launch<8, 52, 16>(8, sample, sink, n_cus, stream); break;   // 64 query rows per wavefront: half the LDS bytes
    case 5: launch<8, 52, 16>(4, sample, sink, n_cus, stream); break;   // the same with one wavefront per SIMD
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace dit

// What the matrix pipes of device `device_id` deliver, alone and beside the other work of an attention tile.
//   mix            0 MFMAs only (two wavefronts per SIMD); 1 what the ping-pong attention kernel issues per MFMA (1 KB of
//                  LDS operand reads, 3.25 vector instructions, one v_exp_f32); 2 its LDS reads only; 3 its vector
//                  instructions only; 4 like 1 with half the LDS bytes (64 query rows per wavefront); 5 like 4 with one
//                  wavefront per SIMD.
//   warm_launches  0..1000 untimed launches first;  timed_launches 1..1000 launches between two events on the null stream.
//   tflops         out (may be NULL): 2*32*32*16 flop per MFMA over the timed launches.
//   shader_mhz     out (may be NULL): the shader clock sampled inside the last launch.
// Allocates and frees a few hundred bytes of device memory and waits for the launches.
// Returns 0, -1 (argument out of range) or -2 (a HIP call failed).
extern "C" int dit_probe_mfma_ceiling(int device_id, int32_t mix, int32_t warm_launches, int32_t timed_launches, double* tflops,
                                      double* shader_mhz) {
  if (mix < 0 || mix >= dit::kCeilingMixes || warm_launches < 0 || warm_launches > 1000 || timed_launches < 1 ||
      timed_launches > 1000)
    return -1;
  hipDeviceProp_t prop;
  hipError_t e = hipSetDevice(device_id);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, device_id);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return -2;
  }
  const int n_cus = prop.multiProcessorCount;
  char* mem = nullptr;  // [2 x uint64 clock sample][64 floats]
  hipEvent_t ev[2] = {nullptr, nullptr};
  float ms = 0.f;
  uint64_t sample[2] = {0, 0};
  e = hipMalloc(reinterpret_cast<void**>(&mem), 16 + 64 * sizeof(float));
  if (e == hipSuccess) e = hipEventCreate(&ev[0]);
  if (e == hipSuccess) e = hipEventCreate(&ev[1]);
  for (int32_t i = 0; i < warm_launches + timed_launches && e == hipSuccess; ++i) {
    if (i == warm_launches) e = hipEventRecord(ev[0], nullptr);
    if (e == hipSuccess)
      e = dit::mfma_ceiling_launch(mix, reinterpret_cast<uint64_t*>(mem), reinterpret_cast<float*>(mem + 16), n_cus, nullptr);
  }
  if (e == hipSuccess) e = hipEventRecord(ev[1], nullptr);
  if (e == hipSuccess) e = hipEventSynchronize(ev[1]);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[0], ev[1]);
  if (e == hipSuccess) e = hipMemcpy(sample, mem, sizeof(sample), hipMemcpyDeviceToHost);
  if (ev[0]) (void)hipEventDestroy(ev[0]);
  if (ev[1]) (void)hipEventDestroy(ev[1]);
  if (mem) (void)hipFree(mem);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return -2;
  }
  const double flop = static_cast<double>(timed_launches) * n_cus * dit::kCeilingWavesPerCu *
                      static_cast<double>(dit::kCeilingMfmaPerWave) * dit::kCeilingFlopPerMfma;
  if (tflops) *tflops = ms > 0.f ? flop / (static_cast<double>(ms) * 1e-3) * 1e-12 : 0.0;
  if (shader_mhz) *shader_mhz = sample[1] > 0 ? 100.0 * static_cast<double>(sample[0]) / static_cast<double>(sample[1]) : 0.0;
  return 0;
}
