// Two calibration kernels for the benchmark: what the chip sustains on a loop of
// nothing but bf16 matrix instructions, and on a plain streaming copy.  They put
// the attention kernels' rates next to measured ceilings (the published peaks
// assume the peak clock, which the power limit does not grant under load).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace svd {

// Every wave runs `iters` rounds of eight independent v_mfma_f32_32x32x16_bf16
// (the instruction of the attention kernels' two products) on pseudo-random bf16
// operands that differ from one instruction to the next; returns the FLOPs of
// the launch through *flops.  out: device floats, 64 per wave (kept so that the
// loop has a use).  work_groups of 512 threads, two waves per SIMD.
hipError_t launch_mfma_probe(float* out, size_t out_floats, int iters, int work_groups, double* flops,
                             hipStream_t stream);
// dst[i] = src[i] over `bytes` bytes (a multiple of 16), 16 bytes per thread and step.
hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream);

}  // namespace svd
