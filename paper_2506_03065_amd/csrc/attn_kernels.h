// Launch interface between the host API and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace svd {

// Kernel-level modes: the five modes of Section 4.2 map to three loop shapes
// (diagonal and multi-diagonal share the banded one) plus the zero fill.
// MODE_PBAND is the banded loop in a rearranged token order (Section 4.1.2): the
// band lists index positions of that order and every row of q, k, v and out is
// reached through the list's row map.
enum { MODE_DENSE = 0, MODE_BAND = 1, MODE_GATHER = 2, MODE_PBAND = 3 };

// Tile shapes the kernels are instantiated for.  Query tile = NW waves x QB
// blocks of 32 rows; key tile = BC keys.
// OCC = waves per SIMD the kernel is compiled for (register budget 512 / OCC).
// Small query tile (half the waves, two work-groups per compute unit) for band
// groups whose bands are narrow: with 128 instead of 256 query rows per tile the
// listed tiles hug the band more closely, which saves more work than the halved
// reuse of a K/V tile costs.  Same key tile, so one plan geometry along the keys.
template <int NW_, int QB_, int BC_, int OCC_>
struct TileShape { static constexpr int NW = NW_, QB = QB_, BC = BC_, OCC = OCC_; };
using Tile128 = TileShape<8, 1, 64, 2>;    // D = 128
using Tile64 = TileShape<8, 1, 128, 2>;    // D = 64
using Tile128s = TileShape<4, 1, 64, 2>;   // D = 128, small query tile
using Tile64s = TileShape<4, 1, 128, 2>;   // D = 64, small query tile
static_assert(Tile128s::BC == Tile128::BC && Tile64s::BC == Tile64::BC, "the small query tile keeps the key tile");

struct AttnLaunch {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  __bf16* out;
  int B, H, L, D;
  int64_t stride_b, stride_h, stride_l;   // elements
  int n_q_blocks;        // query tiles per head
  int n_heads;           // heads in this launch
  int n_items;           // n_q_blocks * n_heads * B
  const int* heads;      // device: head ids of the group, or nullptr = identity
  const int* list_id;    // device: per head of the group, its list
  const int* ws;         // device: workspace base (int32 words)
  int list_table;        // word offset of the group's list records
  float scale_log2e;     // log2(e) / sqrt(D)
  // Key-range split of dense items (split > 1): an item is (query tile, head,
  // batch entry, chunk); chunk c covers key tiles [c*n/split, (c+1)*n/split) and
  // leaves its unnormalised accumulators, reference exponent and row sums in
  // `partial`; a second kernel merges the chunks and writes out.
  int split;             // 1 = off; n_items counts chunks
  float* partial;        // device: partial_floats(...) floats, or nullptr
  // Vertical-stripe groups (MODE_GATHER): the K and V rows of every head's listed
  // columns, gathered by launch_gather_kv ahead of the attention launch, so that
  // the attention loop walks a short dense head: [B * n_heads][2 (K, V)][gather_pad][D],
  // rows past a head's padded list length zero.  gather_pad = the longest padded
  // list of the group (a multiple of the key tile).
  __bf16* gathered;
  int gather_pad;
  // MODE_GATHER: the first skip_q_blocks query tiles of every head belong to another launch (the
  // text rows of a layer with a text prefix, computed densely) and are left alone
  int skip_q_blocks;
};
// Elements of `gathered` for a group of n_heads heads.
inline size_t gathered_elements(int B, int n_heads, int gather_pad, int D) {
  return static_cast<size_t>(B) * n_heads * 2 * gather_pad * D;
}
// Pre-pass of a vertical-stripe group: fills p.gathered from p.k, p.v through the group's column lists.
hipError_t launch_gather_kv(const AttnLaunch& p, hipStream_t stream);

// The whole layer in ONE launch (Section 4.2: heads that share a mode are fused;
// here all groups are): a grid of resident work-groups, two of four waves per
// compute unit, pulls items off eight work queues, one per XCD, heaviest segment
// first.  A segment is one group's items in the order of a grouped launch (query
// tiles of a head consecutive), or the text rows of a sparse group as dense
// items; every segment has eight queues, queue x holding its x-th eighth, so the
// query tiles of a head stay on one XCD.  Segment after segment a work-group
// drains its own XCD's queue, then the other XCDs', and moves on; it leaves after
// the last segment.  Every item runs on the small query tile (128 rows) and
// dense heads are not split: the next segment fills the tail that a launch per
// group pays for.
constexpr int kMaxSegments = 12;
enum { SEG_DENSE = 0, SEG_BAND = 1, SEG_GATHER = 2, SEG_PBAND = 3, SEG_ZERO = 4 };
struct LayerSegment {
  int kind;          // SEG_*
  int n_items;       // n_q_blocks * n_heads * B - first_item
  int n_q_blocks;    // query tiles of 128 rows per head in this segment
  int n_heads;
  int heads;         // word offsets into the plan workspace: head ids of the group,
  int list_id;       //   the list of every head,
  int list_table;    //   the group's list records
  int first_item;    // items below this one are computed elsewhere (the dense head start); n_items counts the rest
};
struct LayerLaunch {
  AttnLaunch a;                      // tensors, shape, strides, scale, ws; the per-group fields are filled per item
  LayerSegment seg[kMaxSegments];    // heaviest first
  int n_segments;
  int* counters;                     // device: kLayerCounterWords queue positions, zeroed by a fill kernel ahead of the layer kernel
};
constexpr int kLayerCounterWords = 8 * kMaxSegments;   // one queue position per (segment, XCD)
// Query rows per item of the single-launch path (the small query tile).
int layer_block_q(int D);
hipError_t launch_layer(const LayerLaunch& p, int n_compute_units, hipStream_t stream);

// Floats of scratch one split launch needs (n_items counts chunks).
size_t partial_floats(int D, int n_items);

void kernel_blocks(int D, int* block_q, int* block_k);
// Query rows of the small tile (band modes only).
int kernel_small_block_q(int D);
// small_q: the launch uses the small query tile (MODE_BAND and MODE_PBAND only;
// n_q_blocks and the lists must have been built for it).
hipError_t launch_attention(const AttnLaunch& p, int mode, hipStream_t stream, bool small_q = false);
hipError_t launch_zero_heads(const AttnLaunch& p, hipStream_t stream);
// Merges the chunks of a split dense launch (same AttnLaunch) into `out`.
hipError_t launch_combine(const AttnLaunch& p, hipStream_t stream);

}  // namespace svd
