// Launch interface of the matrix-pipe ceiling measurement.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dit {

constexpr int kCeilingMfmaPerIter = 16;            // MFMAs a wavefront issues per loop iteration
constexpr int kCeilingWavesPerCu = 8;              // two per SIMD, as in the ping-pong attention kernel
constexpr double kCeilingFlopPerMfma = 2.0 * 32 * 32 * 16;

// Every wavefront issues iters * kCeilingMfmaPerIter register-only MFMAs.  sample: device, 2 x uint64, receives the
// shader-cycle and 100 MHz-counter differences over workgroup 0's run.  sink: device, >= 64 floats (never written in
// practice; it keeps the accumulators alive).
hipError_t mfma_ceiling_launch(uint64_t* sample, float* sink, int iters, int n_cus, hipStream_t stream);

}  // namespace dit
