// gfx950 kernels of the offline search step (Section 4.2, Eq. 2, Algorithm 1).
// Both are streaming kernels bound by HBM: the reduction reads two tensors
// once, the selection reads one and writes one.
#include <hip/hip_runtime.h>

#include "search_kernels.h"

namespace svd {
namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMseThreads = 256;
constexpr int kMseChunkBytes = 1 << 18;   // of one tensor, per work-group

__device__ __forceinline__ float bf16_lo(unsigned w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned w) { return __builtin_bit_cast(float, w & 0xffff0000u); }

// Pass 1: work-group (chunk, b * H + h) sums (a - ref)^2 over its share of the
// head's L * D elements, 16 bytes per thread and step.
__global__ void __launch_bounds__(kMseThreads) head_mse_partial_kernel(const __bf16* __restrict__ a,
                                                                       const __bf16* __restrict__ ref,
                                                                       const TensorView t, const int n_chunks,
                                                                       float* __restrict__ partial) {
  const int bh = blockIdx.y, b = bh / t.H, h = bh % t.H;
  const int64_t base = (int64_t)b * t.stride_b + (int64_t)h * t.stride_h;
  const int cpr = t.D / 8;                                  // 16-byte pieces per row
  const int64_t total = (int64_t)t.L * cpr;
  const int64_t per = (total + n_chunks - 1) / n_chunks;
  const int64_t g0 = (int64_t)blockIdx.x * per;
  const int64_t g1 = g0 + per < total ? g0 + per : total;
  float acc = 0.f;
  auto piece = [&](const int64_t g, u32x4* x, u32x4* y) {
    const int64_t off = base + (g / cpr) * t.stride_l + (g % cpr) * 8;
    *x = *reinterpret_cast<const u32x4*>(a + off);
    *y = *reinterpret_cast<const u32x4*>(ref + off);
  };
  auto add = [&](const u32x4& x, const u32x4& y) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float d0 = bf16_lo(x[i]) - bf16_lo(y[i]), d1 = bf16_hi(x[i]) - bf16_hi(y[i]);
      acc = __builtin_fmaf(d0, d0, acc);
      acc = __builtin_fmaf(d1, d1, acc);
    }
  };
  int64_t g = g0 + threadIdx.x;
  for (; g + 3 * kMseThreads < g1; g += 4 * kMseThreads) {   // eight loads in flight per thread
    u32x4 x[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) piece(g + u * kMseThreads, &x[u], &y[u]);
#pragma unroll
    for (int u = 0; u < 4; ++u) add(x[u], y[u]);
  }
  for (; g < g1; g += kMseThreads) {
    u32x4 x, y;
    piece(g, &x, &y);
    add(x, y);
  }
  // wave reduction, then the four waves through LDS, always in the same order
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) acc += __shfl_down(acc, s, 64);
  __shared__ float wave_sum[kMseThreads / 64];
  if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kMseThreads / 64; ++w) s += wave_sum[w];
    partial[(int64_t)bh * n_chunks + blockIdx.x] = s;
  }
}

// Pass 2: one thread per head adds the partial sums of all batch entries and
// chunks in double, in index order.
__global__ void head_mse_final_kernel(const float* __restrict__ partial, const TensorView t, const int n_chunks,
                                      float* __restrict__ mse) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h >= t.H) return;
  double s = 0.0;
  for (int b = 0; b < t.B; ++b)
    for (int c = 0; c < n_chunks; ++c) s += (double)partial[((int64_t)b * t.H + h) * n_chunks + c];
  mse[h] = (float)(s / ((double)t.B * t.L * t.D));
}

struct SelectArgs {
  const __bf16* src[5];
  unsigned char mode[kMaxSelectHeads];
};

// out[:, h] = src[mode[h]][:, h], 16 bytes per thread and step.
__global__ void __launch_bounds__(256) select_heads_kernel(const SelectArgs args, const TensorView sv,
                                                           __bf16* __restrict__ out, const TensorView ov) {
  const int bh = blockIdx.y, b = bh / sv.H, h = bh % sv.H;
  const __bf16* __restrict__ src = args.src[args.mode[h]] + (int64_t)b * sv.stride_b + (int64_t)h * sv.stride_h;
  __bf16* __restrict__ dst = out + (int64_t)b * ov.stride_b + (int64_t)h * ov.stride_h;
  const int cpr = sv.D / 8;
  const int64_t total = (int64_t)sv.L * cpr;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = g / cpr;
    const int c = (int)(g % cpr) * 8;
    *reinterpret_cast<u32x4*>(dst + row * ov.stride_l + c) = *reinterpret_cast<const u32x4*>(src + row * sv.stride_l + c);
  }
}

}  // namespace

int mse_chunks(const TensorView& t) {
  const int64_t bytes = (int64_t)t.L * t.D * 2;
  const int64_t n = (bytes + kMseChunkBytes - 1) / kMseChunkBytes;
  return (int)(n < 1 ? 1 : n);
}

size_t mse_scratch_floats(const TensorView& t) { return (size_t)t.B * t.H * mse_chunks(t); }

hipError_t launch_head_mse(const __bf16* a, const __bf16* ref, const TensorView& t, float* mse, float* scratch,
                           hipStream_t stream) {
  const int n_chunks = mse_chunks(t);
  hipLaunchKernelGGL(head_mse_partial_kernel, dim3(n_chunks, t.B * t.H), dim3(kMseThreads), 0, stream, a, ref, t,
                     n_chunks, scratch);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  hipLaunchKernelGGL(head_mse_final_kernel, dim3((t.H + 63) / 64), dim3(64), 0, stream, scratch, t, n_chunks, mse);
  return hipGetLastError();
}

hipError_t launch_select_heads(const __bf16* const src[5], const TensorView& src_view, const int32_t* mode_of_head,
                               __bf16* out, const TensorView& out_view, hipStream_t stream) {
  if (src_view.H > kMaxSelectHeads) return hipErrorInvalidValue;
  SelectArgs args{};
  for (int m = 0; m < 5; ++m) args.src[m] = src[m];
  for (int h = 0; h < src_view.H; ++h) args.mode[h] = (unsigned char)mode_of_head[h];
  const int64_t total = (int64_t)src_view.L * (src_view.D / 8);
  int bx = (int)((total + 255) / 256);
  if (bx > 1024) bx = 1024;
  hipLaunchKernelGGL(select_heads_kernel, dim3(bx, src_view.B * src_view.H), dim3(256), 0, stream, args, src_view, out,
                     out_view);
  return hipGetLastError();
}

}  // namespace svd
