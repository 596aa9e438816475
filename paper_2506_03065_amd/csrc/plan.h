// Host-side data model of a compiled layer plan (pattern compiler output).
//
// Section 4.2 of the paper fixes, per layer, one mode per head and fuses heads
// that share a mode.  A plan is that grouping plus, for the sparse modes, the
// block-level description of the kept region of the attention map that the
// kernels iterate over.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "sparse_vdit.h"

namespace svd {

// One distinct band pattern (modes 2, 3): kept diagonals delta = j - i.
struct BandList {
  int32_t half_width = 0;
  std::vector<int32_t> offsets;       // sorted, unique
  std::vector<int32_t> runs;          // 2 * n_runs: inclusive [lo, hi] of merged kept diagonals
  std::vector<int32_t> row_ptr;       // n_q_blocks + 1
  std::vector<int32_t> kv_block_idx;  // per entry
  std::vector<int32_t> flags;         // per entry: 1 = tile needs no mask
  std::vector<int32_t> run_first;     // per entry
  std::vector<int32_t> run_count;     // per entry
  double kept_pairs = 0.0;            // element-level count for one head (text borders included)
  double tile_area = 0.0;             // sum over entries of in-range rows * in-range keys
  // rearranged form (Section 4.1.2): the list above is that of one band in the
  // position-major order; row_map[r] = original row of position r, -1 padded to
  // a multiple of block_k.  Empty for plain lists.
  std::vector<int32_t> row_map;
};

// One distinct column set (mode 4).
struct ColumnList {
  int32_t n_cols = 0;                 // text columns included
  std::vector<int32_t> cols;          // sorted, padded with -1 to a multiple of block_k
};

struct Group {
  int32_t mode = 0;
  bool rearranged = false;            // mode 3 heads in rearranged form (a group of their own)
  // query rows per tile of this group's lists and launches: the plan's block_q,
  // or the small query tile for band groups with narrow bands
  int32_t block_q = 0, n_q_blocks = 0;
  std::vector<int32_t> heads;         // ascending
  std::vector<int32_t> list_id;       // per head of the group
  std::vector<BandList> bands;        // modes 2, 3
  // the same patterns on the small query tile, kept beside `bands` when the group itself runs on the
  // large one: the FP8 kernels run band groups faster on the small tile whatever the band width
  std::vector<BandList> bands_small;
  int32_t n_q_blocks_small = 0;
  std::vector<ColumnList> columns;    // mode 4
  // word offsets into the device workspace (valid when the plan is launchable)
  size_t ws_heads = 0, ws_list_id = 0, ws_list_table = 0;
  size_t ws_list_table_small = 0;     // list records of bands_small (0: none)
};

// Per-list record in the device workspace, 4 int32 words.
//   band list:   {row_ptr offset, entries offset, runs offset, n_runs}
//                rearranged: {row_ptr offset, entries offset, runs offset, row_map offset}
//   column list: {cols offset, padded_len, n_cols, 0}
// Offsets are in int32 words from the workspace base.  A band entry is two
// words {kv_block_idx, meta}, meta = flag | run_first << 1 | run_count << 16.
constexpr int kListRecordWords = 4;
constexpr int32_t kMaxRuns = 32767;

struct Plan {
  svd_tensor_desc desc{};
  int32_t block_q = 0, block_k = 0;
  int32_t n_q_blocks = 0, n_k_blocks = 0;
  // Section 4.1.1: length of the text prefix whose borders (T-T, T-V, V-T) the
  // sparse heads keep whole; 0 = none.  A multiple of block_q and of block_k.
  int32_t text_tokens = 0;
  std::vector<Group> groups;          // ascending mode id
  std::vector<int32_t> ws_image;      // host image of the device workspace
  void* device_workspace = nullptr;   // nullptr: host-only plan
  bool launchable = false;            // block shape matches the kernels and workspace present
};

// Validates the table and parameters and fills plan->groups (lists included)
// and plan->ws_image.  Pure host code, no HIP.
// text_tokens > 0: the band lists of the text query blocks stay empty (their rows
// are computed densely by the caller of the kernels), every other query block
// lists the text key tiles, kept whole, ahead of its band tiles, and the column
// lists gain the text columns.
// block_q_small > 0: band groups (modes 2 and 3) whose lists cover at least 8 %
// less area with that many query rows per tile are compiled for it; with
// always_large none is (the single-launch path runs every item on the large
// query tile) - the small-tile lists are then still kept beside them (bands_small).
svd_status compile_plan(const svd_tensor_desc& desc, const int32_t* strategy_table,
                        const svd_head_params* pattern_params, int32_t block_q, int32_t block_k,
                        int32_t text_tokens, int32_t block_q_small, Plan* plan, bool always_large = false);

svd_status validate_desc(const svd_tensor_desc* desc);

}  // namespace svd
