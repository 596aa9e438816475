// Launch interface of the FP8 (OCP E4M3) variant of the attention kernels
// (Appendix B: the sparse kernels combined with FP8 quantisation).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "attn_kernels.h"

namespace svd {

// Quantised K and V of every head live in caller-provided scratch:
//   k8   [B][H][Lp][D] bytes        K / 4, one E4M3 byte per element
//   v8t  [B][H][Lp / 64][D][64]     V transposed in groups of 64 keys; inside a
//                                   group, byte 32*h + 16*blk + 4*g + r of row d
//                                   is key 32*blk + 8*g + 4*h + r (the order in
//                                   which the score accumulators of a lane hold
//                                   the keys, so P needs no shuffle)
// Lp = L rounded up to a multiple of 128; keys past the head's key count are
// zero.  For a vertical-stripe head the arrays hold the head's gathered columns
// in list order, so the kernel walks them like a short dense head; for a
// multi-diagonal head in rearranged form they hold the keys in the rearranged order.
struct Fp8Launch {
  AttnLaunch a;          // q, out, shapes, lists, split as for the bf16 kernels (k, v: the bf16 sources of the pre-pass)
  uint8_t* k8;
  uint8_t* v8t;
  int Lp;
  int map_len;           // PBAND: entries of the row map (L rounded up to the key tile)
};

inline int fp8_padded_len(int L) { return (L + 127) / 128 * 128; }
// Bytes of scratch for k8 plus v8t.
inline size_t fp8_scratch_bytes(int B, int H, int L, int D) {
  return 2 * static_cast<size_t>(B) * H * fp8_padded_len(L) * D;
}

// Pre-pass: quantises K and V of the heads of one group (mode as for launch_attention).
hipError_t launch_quantise_kv(const Fp8Launch& p, int mode, hipStream_t stream);
// Attention of one group on the quantised arrays; split dense launches are merged
// with launch_combine of the bf16 kernels (same partial layout).
// small_q as for launch_attention.
hipError_t launch_attention_fp8(const Fp8Launch& p, int mode, hipStream_t stream, bool small_q = false);

}  // namespace svd
