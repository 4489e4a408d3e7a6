// Launch interface of the matrix-pipe ceiling measurements.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dit {

constexpr int kCeilingMfmaPerIter = 16;            // MFMAs a wavefront issues per loop iteration
constexpr int kCeilingMfmaPerWave = 131072;        // MFMAs per wavefront at two wavefronts per SIMD (twice that at one)
constexpr int kCeilingWavesPerCu = 8;              // two per SIMD, as in the ping-pong attention kernel
constexpr double kCeilingFlopPerMfma = 2.0 * 32 * 32 * 16;
constexpr int kCeilingMixes = 6;                   // mixes 0 .. 5, see include/dit_attn.h

// Every compute unit issues kCeilingWavesPerCu * kCeilingMfmaPerWave register-only MFMAs, with the LDS reads and vector
// instructions of `mix` beside them.  sample: device, 2 x uint64, receives the shader-cycle and 100 MHz-counter
// differences over the run of workgroup 0's first wavefront.  sink: device, >= 64 floats (never written in practice;
// it keeps the results alive).  mix must be in 0 .. kCeilingMixes - 1.
hipError_t mfma_ceiling_launch(int mix, uint64_t* sample, float* sink, int n_cus, hipStream_t stream);

}  // namespace dit
