// Calibration kernels of the benchmark (measured ceilings for the roofline).
#include "probe_kernels.h"

namespace svd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kProbeAcc = 8;   // independent accumulators per wave: enough to cover the MFMA latency

// Operand bits from a small integer hash: bf16 values of either sign with exponents around one and
// random mantissas, different in every lane and for every accumulator, so that successive matrix
// instructions see operands that differ (a loop over one constant operand pair toggles no input
// and is granted the full clock; attention operands are not like that).
__device__ __forceinline__ unsigned mix(unsigned x) {
  x ^= x >> 16;
  x *= 0x7feb352du;
  x ^= x >> 15;
  x *= 0x846ca68bu;
  x ^= x >> 16;
  return x;
}
__device__ __forceinline__ __bf16 random_bf16(unsigned seed) {
  const unsigned r = mix(seed);
  const unsigned short bits = (unsigned short)(((r & 1u) << 15) | ((124u + ((r >> 1) & 3u)) << 7) | ((r >> 8) & 0x7fu));
  return __builtin_bit_cast(__bf16, bits);
}

__global__ void __launch_bounds__(512, 2) mfma_probe_kernel(float* __restrict__ out, const int iters) {
  const unsigned id = blockIdx.x * 512u + threadIdx.x;
  bf16x8 a[kProbeAcc], b[kProbeAcc];
#pragma unroll
  for (int j = 0; j < kProbeAcc; ++j)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[j][i] = random_bf16(id * 131u + j * 17u + i);
      b[j][i] = random_bf16(id * 257u + j * 29u + i + 7919u);
    }
  f32x16 acc[kProbeAcc];
#pragma unroll
  for (int j = 0; j < kProbeAcc; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < kProbeAcc; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], b[j], acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < kProbeAcc; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

// Four independent 16-byte loads per thread and step, then the four stores.
__global__ void __launch_bounds__(256) copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                         const size_t n16) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    dst[i] = v0;
    dst[i + stride] = v1;
    dst[i + 2 * stride] = v2;
    dst[i + 3 * stride] = v3;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace

hipError_t launch_mfma_probe(float* out, size_t out_floats, int iters, int work_groups, double* flops,
                             hipStream_t stream) {
  if (!out || iters < 1 || work_groups < 1 || out_floats < (size_t)work_groups * 512) return hipErrorInvalidValue;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(work_groups), dim3(512), 0, stream, out, iters);
  if (flops) *flops = 2.0 * 32 * 32 * 16 * kProbeAcc * (double)iters * 8.0 * work_groups;
  return hipGetLastError();
}

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream) {
  if (!src || !dst || bytes == 0 || bytes % 16) return hipErrorInvalidValue;
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;   // grid-stride beyond 32 work-groups per compute unit
  hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n16);
  return hipGetLastError();
}

}  // namespace svd
