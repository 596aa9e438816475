// Pattern compiler: per-head strategy table -> fused head groups and block lists.
//
// Section 4.2: after the offline search every head of a layer has a fixed mode,
// heads of a layer with the same mode are fused, and the sparsity of a sparse
// mode is counted in blocks of the attention map.  Section 4.1.2 defines the
// kept regions.  This file turns those definitions into the lists the kernels
// walk, using interval arithmetic on the diagonals delta = j - i (a band pattern
// depends on delta only) - no mask is ever materialised here.
#include <algorithm>
#include <map>
#include <set>
#include <utility>

#include "plan.h"

namespace svd {
namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

using BandKey = std::pair<int32_t, std::vector<int32_t>>;

// Merge the closed intervals [o - w, o + w] into maximal runs of consecutive kept
// diagonals and clip them to the diagonals that exist, [-(L-1), L-1].
std::vector<int32_t> merged_runs(const std::vector<int32_t>& sorted_offsets, int64_t w, int64_t L) {
  std::vector<int32_t> runs;
  bool open = false;
  int64_t lo = 0, hi = 0;
  auto flush = [&]() {
    const int64_t a = std::max<int64_t>(lo, -(L - 1)), b = std::min<int64_t>(hi, L - 1);
    if (a <= b) {
      runs.push_back(static_cast<int32_t>(a));
      runs.push_back(static_cast<int32_t>(b));
    }
  };
  for (int32_t o : sorted_offsets) {
    const int64_t a = static_cast<int64_t>(o) - w, b = static_cast<int64_t>(o) + w;
    if (open && a <= hi + 1) {
      hi = std::max(hi, b);
    } else {
      if (open) flush();
      lo = a;
      hi = b;
      open = true;
    }
  }
  if (open) flush();
  return runs;
}

// Every query row i in [0, L) must keep a key: for run [a, b] the rows with a
// key are those with i + a <= L - 1 and i + b >= 0.
bool every_row_keeps_a_key(const std::vector<int32_t>& runs, int64_t L) {
  std::vector<std::pair<int64_t, int64_t>> rows;
  for (size_t r = 0; r + 1 < runs.size(); r += 2) {
    const int64_t lo = std::max<int64_t>(0, -static_cast<int64_t>(runs[r + 1]));
    const int64_t hi = std::min<int64_t>(L - 1, L - 1 - static_cast<int64_t>(runs[r]));
    if (lo <= hi) rows.emplace_back(lo, hi);
  }
  std::sort(rows.begin(), rows.end());
  int64_t covered = 0;  // rows [0, covered) are known to keep a key
  for (const auto& iv : rows) {
    if (iv.first > covered) return false;
    covered = std::max(covered, iv.second + 1);
  }
  return covered >= L;
}

struct Entry {
  int32_t kb, flag, first, count;
};

// T > 0 (a multiple of bq and bk): text prefix of Section 4.1.1.  Query blocks of
// text rows get no entries; the others list the text tiles first, kept whole.
void build_band_list(BandList* bl, int64_t L, int64_t bq, int64_t bk, int64_t T) {
  const int64_t n_qb = ceil_div(L, bq);
  const size_t n_runs = bl->runs.size() / 2;
  bl->row_ptr.assign(1, 0);
  // element-level pairs: text rows and text columns whole, plus the band inside
  // the video x video square, which has the structure of a sequence of L - T
  const int64_t Lv = L - T;
  bl->kept_pairs = static_cast<double>(T) * L + static_cast<double>(Lv) * T;
  for (size_t r = 0; r < n_runs; ++r) {
    const int64_t a = std::max<int64_t>(bl->runs[2 * r], -(Lv - 1)), b = std::min<int64_t>(bl->runs[2 * r + 1], Lv - 1);
    if (a > b) continue;
    // diagonal delta holds L - |delta| cells: (b - a + 1) * L - sum |delta|
    double pairs = 0.0;
    if (a >= 0) {
      pairs = static_cast<double>(b - a + 1) * Lv - (static_cast<double>(a + b) * (b - a + 1)) / 2.0;
    } else if (b <= 0) {
      pairs = static_cast<double>(b - a + 1) * Lv - (static_cast<double>(-a - b) * (b - a + 1)) / 2.0;
    } else {
      pairs = static_cast<double>(b - a + 1) * Lv - static_cast<double>(b) * (b + 1) / 2.0 -
              static_cast<double>(-a) * (-a + 1) / 2.0;
    }
    bl->kept_pairs += pairs;
  }
  bl->tile_area = 0.0;
  std::vector<Entry> row;
  for (int64_t qb = 0; qb < n_qb; ++qb) {
    const int64_t i0 = qb * bq, i1 = std::min(L, i0 + bq) - 1;
    row.clear();
    if (i0 < T) {   // text rows: dense, not listed
      bl->row_ptr.push_back(static_cast<int32_t>(bl->kv_block_idx.size()));
      continue;
    }
    for (int64_t kb = 0; kb < T / bk; ++kb) row.push_back({static_cast<int32_t>(kb), 1, 0, 0});
    const size_t n_text = row.size();
    for (size_t r = 0; r < n_runs; ++r) {
      const int64_t a = bl->runs[2 * r], b = bl->runs[2 * r + 1];
      const int64_t j_lo = std::max<int64_t>(0, i0 + a), j_hi = std::min<int64_t>(L - 1, i1 + b);
      if (j_lo > j_hi) continue;
      const int64_t kb_lo = j_lo / bk, kb_hi = j_hi / bk;
      // runs ascend, so key-block ranges ascend; a tile may be shared with the
      // tail of the entries already listed for earlier runs
      size_t pos = row.size();
      while (pos > 0 && row[pos - 1].kb >= kb_lo) --pos;
      for (int64_t kb = kb_lo; kb <= kb_hi; ++kb) {
        const int64_t jt0 = kb * bk, jt1 = kb * bk + bk - 1;
        const bool full = jt1 <= L - 1 && a <= jt0 - i1 && jt1 - i0 <= b;
        if (pos < row.size() && row[pos].kb == kb) {
          if (pos < n_text && row[pos].count == 0) row[pos].first = static_cast<int32_t>(r);   // a text tile the band reaches
          row[pos].count += 1;
          row[pos].flag |= full ? 1 : 0;
          ++pos;
        } else {
          row.push_back({static_cast<int32_t>(kb), full ? 1 : 0, static_cast<int32_t>(r), 1});
          pos = row.size();
        }
      }
    }
    for (const Entry& e : row) {
      bl->kv_block_idx.push_back(e.kb);
      bl->flags.push_back(e.flag);
      bl->run_first.push_back(e.first);
      bl->run_count.push_back(e.count);
      const int64_t cols = std::min<int64_t>(L, static_cast<int64_t>(e.kb + 1) * bk) - static_cast<int64_t>(e.kb) * bk;
      bl->tile_area += static_cast<double>(i1 - i0 + 1) * static_cast<double>(cols);
    }
    bl->row_ptr.push_back(static_cast<int32_t>(bl->kv_block_idx.size()));
  }
}

size_t align4(size_t words) { return (words + 3) & ~static_cast<size_t>(3); }

size_t append(std::vector<int32_t>* img, const std::vector<int32_t>& data) {
  const size_t at = align4(img->size());
  img->resize(at, 0);
  img->insert(img->end(), data.begin(), data.end());
  return at;
}

}  // namespace

svd_status validate_desc(const svd_tensor_desc* desc) {
  if (!desc) return SVD_ERR_NULL;
  if (desc->B < 1 || desc->H < 1 || desc->L < 1) return SVD_ERR_SHAPE;
  if (desc->D != 64 && desc->D != 128) return SVD_ERR_SHAPE;
  if (desc->stride_l < desc->D || desc->stride_b < 1 || desc->stride_h < 1) return SVD_ERR_SHAPE;
  if (desc->stride_b % 8 || desc->stride_h % 8 || desc->stride_l % 8) return SVD_ERR_ALIGN;
  // the kernels address the rows of one head with 32-bit byte offsets
  if (static_cast<double>(desc->L) * static_cast<double>(desc->stride_l) * 2.0 >= 4294967296.0)
    return SVD_ERR_UNSUPPORTED;
  // the gather path forms row offsets with a 24-bit multiply: row index and row stride in bytes below 2^24
  if (desc->L >= (1 << 24) || desc->stride_l * 2 >= (1 << 24)) return SVD_ERR_UNSUPPORTED;
  return SVD_OK;
}

svd_status compile_plan(const svd_tensor_desc& desc, const int32_t* strategy_table,
                        const svd_head_params* pattern_params, int32_t block_q, int32_t block_k,
                        int32_t text_tokens, int32_t block_q_small, Plan* plan, bool always_large) {
  if (!strategy_table || !pattern_params || !plan) return SVD_ERR_NULL;
  if (svd_status st = validate_desc(&desc)) return st;
  if (block_q < 1 || block_k < 1) return SVD_ERR_UNSUPPORTED;
  const int64_t L = desc.L;
  const int64_t T = text_tokens;
  if (T < 0 || T >= L) return SVD_ERR_PARAMS;
  if (T % block_q || T % block_k) return SVD_ERR_UNSUPPORTED;
  plan->text_tokens = text_tokens;
  plan->desc = desc;
  plan->block_q = block_q;
  plan->block_k = block_k;
  plan->n_q_blocks = static_cast<int32_t>(ceil_div(L, block_q));
  plan->n_k_blocks = static_cast<int32_t>(ceil_div(L, block_k));
  plan->groups.clear();

  for (int32_t h = 0; h < desc.H; ++h)
    if (strategy_table[h] < SVD_DENSE || strategy_table[h] > SVD_VSTRIPE) return SVD_ERR_MODE;

  // one pass per group: the five modes, and after the plain multi-diagonal heads
  // those in rearranged form (Section 4.1.2), which run another loop shape
  static const int32_t pass_mode[6] = {SVD_DENSE, SVD_SKIP, SVD_DIAG, SVD_MULTIDIAG, SVD_MULTIDIAG, SVD_VSTRIPE};
  static const bool pass_rearranged[6] = {false, false, false, false, true, false};
  for (int pass = 0; pass < 6; ++pass) {
    const int32_t mode = pass_mode[pass];
    Group g;
    g.mode = mode;
    g.rearranged = pass_rearranged[pass];
    std::map<BandKey, int32_t> band_ids;
    std::map<std::vector<int32_t>, int32_t> col_ids;
    for (int32_t h = 0; h < desc.H; ++h) {
      if (strategy_table[h] != mode) continue;
      const svd_head_params& p = pattern_params[h];
      if (mode == SVD_MULTIDIAG && (p.rearr_frames > 0) != g.rearranged) continue;
      int32_t id = 0;
      if (g.rearranged) {
        // one band of half width w in the position-major order of the video block
        if (p.half_width < 0 || p.rearr_first < 0 || p.rearr_frame_tokens < 1) return SVD_ERR_PARAMS;
        const int64_t first = p.rearr_first, N = p.rearr_frame_tokens, F = p.rearr_frames;
        if (first + N * F > L) return SVD_ERR_PARAMS;
        if (T > 0) return SVD_ERR_UNSUPPORTED;
        BandKey key(p.half_width, {p.rearr_first, p.rearr_frame_tokens, p.rearr_frames});
        auto it = band_ids.find(key);
        if (it == band_ids.end()) {
          BandList bl;
          bl.half_width = p.half_width;
          bl.offsets.assign(1, 0);
          bl.runs = merged_runs(bl.offsets, p.half_width, L);
          build_band_list(&bl, L, block_q, block_k, 0);
          bl.row_map.assign(static_cast<size_t>(ceil_div(L, block_k) * block_k), -1);
          for (int64_t i = 0; i < L; ++i) {
            const int64_t v = i - first;
            const int64_t pos = (v < 0 || v >= N * F) ? i : first + (v % N) * F + v / N;
            bl.row_map[static_cast<size_t>(pos)] = static_cast<int32_t>(i);
          }
          id = static_cast<int32_t>(g.bands.size());
          band_ids.emplace(std::move(key), id);
          g.bands.push_back(std::move(bl));
        } else {
          id = it->second;
        }
        g.heads.push_back(h);
        g.list_id.push_back(id);
        continue;
      }
      if (mode == SVD_DIAG || mode == SVD_MULTIDIAG) {
        if (p.half_width < 0) return SVD_ERR_PARAMS;
        std::vector<int32_t> offs;
        if (mode == SVD_DIAG) {
          offs.push_back(0);
        } else {
          if (p.n_offsets < 1) return SVD_ERR_PARAMS;
          if (!p.offsets) return SVD_ERR_NULL;
          offs.assign(p.offsets, p.offsets + p.n_offsets);
          std::sort(offs.begin(), offs.end());
          if (std::adjacent_find(offs.begin(), offs.end()) != offs.end()) return SVD_ERR_PARAMS;
        }
        BandKey key(p.half_width, offs);
        auto it = band_ids.find(key);
        if (it == band_ids.end()) {
          BandList bl;
          bl.half_width = p.half_width;
          bl.offsets = offs;
          bl.runs = merged_runs(offs, p.half_width, L);
          if (bl.runs.size() / 2 > static_cast<size_t>(kMaxRuns)) return SVD_ERR_UNSUPPORTED;
          if (T == 0 && !every_row_keeps_a_key(bl.runs, L)) return SVD_ERR_EMPTY_PATTERN;   // text keys are kept by every row
          build_band_list(&bl, L, block_q, block_k, T);
          id = static_cast<int32_t>(g.bands.size());
          band_ids.emplace(std::move(key), id);
          g.bands.push_back(std::move(bl));
        } else {
          id = it->second;
        }
      } else if (mode == SVD_VSTRIPE) {
        if (p.n_cols < 1) return SVD_ERR_EMPTY_PATTERN;
        if (!p.cols) return SVD_ERR_NULL;
        std::vector<int32_t> cols(p.cols, p.cols + p.n_cols);
        std::sort(cols.begin(), cols.end());
        if (cols.front() < 0 || cols.back() >= L) return SVD_ERR_PARAMS;
        if (std::adjacent_find(cols.begin(), cols.end()) != cols.end()) return SVD_ERR_PARAMS;
        if (T > 0) {   // the text columns belong to every stripe head
          std::vector<int32_t> with_text;
          for (int32_t c = 0; c < T; ++c) with_text.push_back(c);
          for (int32_t c : cols)
            if (c >= T) with_text.push_back(c);
          cols.swap(with_text);
        }
        auto it = col_ids.find(cols);
        if (it == col_ids.end()) {
          ColumnList cl;
          cl.n_cols = static_cast<int32_t>(cols.size());
          cl.cols = cols;
          cl.cols.resize(static_cast<size_t>(ceil_div(cl.n_cols, block_k) * block_k), -1);
          id = static_cast<int32_t>(g.columns.size());
          col_ids.emplace(std::move(cols), id);
          g.columns.push_back(std::move(cl));
        } else {
          id = it->second;
        }
      }
      g.heads.push_back(h);
      g.list_id.push_back(id);
    }
    if (g.heads.empty()) continue;
    g.block_q = block_q;
    if (!g.bands.empty() && block_q_small > 0 && block_q_small < block_q && T % block_q_small == 0) {
      // the same lists on the small query tile: taken when it saves at least 8 % of the listed area.  The
      // 256-row tile reuses a K/V tile in LDS for twice as many rows and runs 6 % (D = 128) to 11 % (D = 64)
      // faster per listed FLOP (measured on the diagonal groups of the benchmark layers, which hold 2-3 %
      // less area on the small tile and are 4-7 % faster on the large one; the multi-diagonal groups, 6-9 %
      // less area, break even)
      std::vector<BandList> alt;
      for (const BandList& bl : g.bands) {
        BandList a;
        a.half_width = bl.half_width;
        a.offsets = bl.offsets;
        a.runs = bl.runs;
        a.row_map = bl.row_map;
        build_band_list(&a, L, block_q_small, block_k, T);
        alt.push_back(std::move(a));
      }
      double area = 0.0, area_small = 0.0;
      for (size_t t = 0; t < g.heads.size(); ++t) {
        area += g.bands[g.list_id[t]].tile_area;
        area_small += alt[g.list_id[t]].tile_area;
      }
      if (!always_large && area_small < 0.92 * area) {
        g.bands.swap(alt);
        g.block_q = block_q_small;
      } else {
        g.bands_small.swap(alt);
        g.n_q_blocks_small = static_cast<int32_t>(ceil_div(L, block_q_small));
      }
    }
    g.n_q_blocks = static_cast<int32_t>(ceil_div(L, g.block_q));
    plan->groups.push_back(std::move(g));
  }

  // Image of the device workspace.
  std::vector<int32_t>& img = plan->ws_image;
  img.clear();
  for (Group& g : plan->groups) {
    g.ws_heads = append(&img, g.heads);
    g.ws_list_id = append(&img, g.list_id);
    const size_t n_lists = g.bands.size() + g.columns.size();
    g.ws_list_table = append(&img, std::vector<int32_t>(n_lists * kListRecordWords, 0));
    auto emit_band_lists = [&img](const std::vector<BandList>& lists, size_t table) {
      for (size_t l = 0; l < lists.size(); ++l) {
        const BandList& bl = lists[l];
        std::vector<int32_t> entries(bl.kv_block_idx.size() * 2);
        for (size_t e = 0; e < bl.kv_block_idx.size(); ++e) {
          entries[2 * e] = bl.kv_block_idx[e];
          entries[2 * e + 1] = bl.flags[e] | (bl.run_first[e] << 1) | (bl.run_count[e] << 16);
        }
        const size_t rp = append(&img, bl.row_ptr), en = append(&img, entries), ru = append(&img, bl.runs);
        int32_t* rec = img.data() + table + l * kListRecordWords;
        rec[0] = static_cast<int32_t>(rp);
        rec[1] = static_cast<int32_t>(en);
        rec[2] = static_cast<int32_t>(ru);
        rec[3] = static_cast<int32_t>(bl.runs.size() / 2);
        if (!bl.row_map.empty()) {
          const size_t rm = append(&img, bl.row_map);
          img[table + l * kListRecordWords + 3] = static_cast<int32_t>(rm);   // append may have moved the image
        }
      }
    };
    emit_band_lists(g.bands, g.ws_list_table);
    if (!g.bands_small.empty()) {
      g.ws_list_table_small = append(&img, std::vector<int32_t>(g.bands_small.size() * kListRecordWords, 0));
      emit_band_lists(g.bands_small, g.ws_list_table_small);
    }
    for (size_t l = 0; l < g.columns.size(); ++l) {
      const ColumnList& cl = g.columns[l];
      const size_t co = append(&img, cl.cols);
      int32_t* rec = img.data() + g.ws_list_table + l * kListRecordWords;
      rec[0] = static_cast<int32_t>(co);
      rec[1] = static_cast<int32_t>(cl.cols.size());
      rec[2] = cl.n_cols;
      rec[3] = 0;
    }
  }
  img.resize(align4(img.size()) + 4, 0);  // never empty, 16-byte multiple
  if (img.size() > static_cast<size_t>(INT32_MAX)) return SVD_ERR_UNSUPPORTED;
  return SVD_OK;
}

}  // namespace svd
