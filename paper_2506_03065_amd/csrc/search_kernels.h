// Launch interface of the kernels of the offline search step (Section 4.2,
// "Offline Sparse Diffusion Search": Eq. 2 needs MSE(O_i - O_0) per head,
// Algorithm 1 assembles the layer output from the chosen modes).
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace svd {

struct TensorView {
  int B, H, L, D;
  int64_t stride_b, stride_h, stride_l;   // elements; D contiguous
};

// Work-groups per (batch entry, head) of the first reduction pass.
int mse_chunks(const TensorView& t);
// Floats of scratch the reduction needs: one partial sum per (batch, head, chunk).
size_t mse_scratch_floats(const TensorView& t);
// mse[h] = mean over b, l, d of (a - ref)^2; two passes, fixed summation order.
hipError_t launch_head_mse(const __bf16* a, const __bf16* ref, const TensorView& t, float* mse, float* scratch,
                           hipStream_t stream);

constexpr int kMaxSelectHeads = 1024;
// out[:, h] = src[mode_of_head[h]][:, h]; the sources share the layout `src_view`.
hipError_t launch_select_heads(const __bf16* const src[5], const TensorView& src_view, const int32_t* mode_of_head,
                               __bf16* out, const TensorView& out_view, hipStream_t stream);

}  // namespace svd
