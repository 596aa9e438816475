// Launch interface of the token rearrangement (Section 4.1.2, multi-diagonal
// pattern: "by rearranging tokens" the evenly spaced diagonals become one band).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "search_kernels.h"

namespace svd {

// Video block = F frames of N tokens starting at token `first` (frame-major:
// frame f, position p at first + f*N + p).  forward: dst row first + p*F + f =
// src row first + f*N + p; inverse: the opposite; rows outside the block are
// copied in place.  src and dst share the view `t` and must not overlap.
hipError_t launch_rearrange_tokens(const __bf16* src, __bf16* dst, const TensorView& t, int first, int frame_tokens,
                                   int frames, bool inverse, hipStream_t stream);

}  // namespace svd
