// gfx950 kernel of the token rearrangement (Section 4.1.2): rows of a
// [B, H, L, D] tensor move between frame-major and position-major order.  A
// streaming kernel bound by HBM: every element is read once and written once.
// Work-group (chunk, b * H + h) walks destination rows in order, so writes are
// contiguous; the matching source rows are whole rows of 128 or 256 bytes.
#include <hip/hip_runtime.h>

#include "rearrange_kernels.h"

namespace svd {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kRowsPerGroup = 512;   // destination rows per work-group

__global__ void __launch_bounds__(kThreads) rearrange_tokens_kernel(const __bf16* __restrict__ src,
                                                                    __bf16* __restrict__ dst, const TensorView t,
                                                                    const int first, const int N, const int F,
                                                                    const int inverse) {
  const int bh = blockIdx.y, b = bh / t.H, h = bh % t.H;
  const int64_t base = (int64_t)b * t.stride_b + (int64_t)h * t.stride_h;
  const int cpr = t.D / 8;   // 16-byte pieces per row
  const int r0 = blockIdx.x * kRowsPerGroup;
  const int r1 = r0 + kRowsPerGroup < t.L ? r0 + kRowsPerGroup : t.L;
  const int n_video = N * F;
  auto source_row = [&](const int r) -> int {
    const int v = r - first;
    if (v < 0 || v >= n_video) return r;
    // forward: destination is position-major (v = p*F + f), source frame-major (f*N + p)
    return inverse ? first + (v % N) * F + v / N : first + (v % F) * N + v / F;
  };
  const int total = (r1 - r0) * cpr;
  int g = threadIdx.x;
  for (; g + 3 * kThreads < total; g += 4 * kThreads) {   // four loads in flight per thread
    u32x4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int gg = g + u * kThreads;
      x[u] = *reinterpret_cast<const u32x4*>(src + base + (int64_t)source_row(r0 + gg / cpr) * t.stride_l + (gg % cpr) * 8);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int gg = g + u * kThreads;
      *reinterpret_cast<u32x4*>(dst + base + (int64_t)(r0 + gg / cpr) * t.stride_l + (gg % cpr) * 8) = x[u];
    }
  }
  for (; g < total; g += kThreads) {
    const u32x4 x = *reinterpret_cast<const u32x4*>(src + base + (int64_t)source_row(r0 + g / cpr) * t.stride_l + (g % cpr) * 8);
    *reinterpret_cast<u32x4*>(dst + base + (int64_t)(r0 + g / cpr) * t.stride_l + (g % cpr) * 8) = x;
  }
}

}  // namespace

hipError_t launch_rearrange_tokens(const __bf16* src, __bf16* dst, const TensorView& t, int first, int frame_tokens,
                                   int frames, bool inverse, hipStream_t stream) {
  if (t.L < 1 || t.B * t.H < 1) return hipSuccess;
  const dim3 grid((t.L + kRowsPerGroup - 1) / kRowsPerGroup, t.B * t.H), block(kThreads);
  hipLaunchKernelGGL(rearrange_tokens_kernel, grid, block, 0, stream, src, dst, t, first, frame_tokens, frames,
                     inverse ? 1 : 0);
  return hipGetLastError();
}

}  // namespace svd
