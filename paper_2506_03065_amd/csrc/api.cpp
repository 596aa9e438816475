// C ABI of the library (see include/sparse_vdit.h for the contract).
//
// Host logic only: argument validation, plan life cycle, the copy of the
// compiled lists into the caller's workspace, and the per-layer launch sequence
// of Section 4.2 (one fused launch per mode present in the layer).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "attn_kernels.h"
#include "fp8_kernels.h"
#include "plan.h"
#include "probe_kernels.h"
#include "rearrange_kernels.h"
#include "search_kernels.h"
#include "sparse_vdit.h"
#include "static_scratch.h"

// A launchable plan owns a few side streams and events.  The groups of a layer
// are independent (they write different heads); when the last, partial round of
// work-groups of the heaviest group would leave most compute units idle, the
// forward pass forks the groups onto the side streams and joins them again on
// the caller's stream, so that the lighter groups fill those units.  Otherwise
// the groups run one after the other on the caller's stream.  Streams keep the
// default priority.
constexpr int kSideStreams = 3;
struct svd_plan {
  svd::Plan p;
  hipStream_t side[kSideStreams] = {nullptr, nullptr, nullptr};
  hipEvent_t fork = nullptr;
  hipEvent_t join[kSideStreams] = {nullptr, nullptr, nullptr};
  bool concurrent = false;
  int dense_split = 1;          // key-range chunks per dense item
  size_t partial_offset = 0;    // byte offset of the split scratch in the workspace
  // text prefix (Section 4.1.1): per group, key-range chunks of the dense launch
  // that computes the text rows of its heads, and the byte offset of its scratch
  std::vector<int> text_split;
  std::vector<size_t> text_partial_offset;
  // single launch (plan option): the segments of the layer kernel, heaviest first, and
  // the byte offset of its queue positions in the workspace
  // vertical-stripe group: byte offset of its gathered K/V rows in the workspace, rows per head
  size_t gather_offset = 0;
  int gather_pad = 0;
  bool single_launch = false;
  bool head_start_asked = false;   // form 3, whether or not a whole round of dense items exists
  // dense head start (plan option single_launch = 3): this many 256-row dense items, whole rounds of
  // one work-group per compute unit, run through the dense kernel ahead of the layer kernel
  int dense_head_start = 0;
  const svd::Group* dense_group = nullptr;
  svd::LayerLaunch layer{};
  size_t counters_offset = 0;
  int n_cu = 0;
  ~svd_plan() {
    for (int i = 0; i < kSideStreams; ++i) {
      if (side[i]) (void)hipStreamDestroy(side[i]);
      if (join[i]) (void)hipEventDestroy(join[i]);
    }
    if (fork) (void)hipEventDestroy(fork);
  }
};

namespace {

using svd::Plan;

bool aligned16(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) == 0; }

svd_status resolve_blocks(const svd_tensor_desc& desc, const svd_plan_options* opt, int32_t* bq,
                          int32_t* bk, bool* native) {
  int kq = 0, kk = 0;
  svd::kernel_blocks(desc.D, &kq, &kk);
  *bq = (opt && opt->block_q) ? opt->block_q : kq;
  *bk = (opt && opt->block_k) ? opt->block_k : kk;
  if (*bq < 1 || *bk < 1) return SVD_ERR_UNSUPPORTED;
  if (opt && opt->dense_split < 0) return SVD_ERR_UNSUPPORTED;
  if (opt && opt->text_tokens < 0) return SVD_ERR_PARAMS;
  *native = (*bq == kq && *bk == kk);
  if (opt && (opt->single_launch < 0 || opt->single_launch > 3)) return SVD_ERR_PARAMS;
  if (opt && (opt->single_launch == 1 || opt->single_launch == 3) && !*native) return SVD_ERR_UNSUPPORTED;
  return SVD_OK;
}

// How svd_attn_forward_planned runs the plan: 0 = a launch per group, 1 = the layer kernel alone, 3 = the layer
// kernel after a dense head start.  The library's own choice follows the measurements: the layer kernel saves the
// partly filled last round of every group, 3-5 % of a layer at D = 128 (HunyuanVideo-, Wan2.1-like layers, the
// stack), where the head start brings nothing on top; at D = 64 the grouped launches with their three-way dense
// split stay 2-8 % ahead of both forms.  Grouped launches also whenever the caller forces a dense split, the items
// are short, or there is no device to size the grid from.
int layer_form(const svd_plan_options* opt, const svd_tensor_desc& d, bool native, int n_cu, double tiles_per_item) {
  const int asked = opt ? opt->single_launch : 0;
  if (asked == 1 || asked == 3) return asked;
  if (asked == 2 || !native || n_cu < 1) return 0;
  if (opt && opt->dense_split > 1) return 0;
  // picking an item off a queue costs a few microseconds (an atomic round trip, two barriers): with short items
  // (narrow windows, short sequences) that outweighs the tails (measured: 29 key tiles per item, 8 % slower)
  if (tiles_per_item < 48.0) return 0;
  return d.D == 128 ? 1 : 0;
}

// Key tiles per item of the layer on the 128-row tile, averaged over the heads that compute (what the
// library's choice of the launch form looks at; taken from the table and parameters alone).
double mean_tiles_per_item(const svd_tensor_desc& d, const int32_t* table, const svd_head_params* pp, int block_k,
                           int text_tokens) {
  const double n_kb = std::ceil(static_cast<double>(d.L) / block_k);
  const double rows = svd::layer_block_q(d.D);
  double tiles = 0.0;
  int heads = 0;
  for (int h = 0; h < d.H; ++h) {
    double t = 0.0;
    switch (table[h]) {
      case SVD_DENSE: t = n_kb; break;
      case SVD_DIAG: t = (2.0 * pp[h].half_width + rows) / block_k + 1.0; break;
      case SVD_MULTIDIAG:
        t = (pp[h].rearr_frames > 0 ? 1 : (pp[h].n_offsets > 0 ? pp[h].n_offsets : 1)) * ((2.0 * pp[h].half_width + rows) / block_k + 1.0);
        break;
      case SVD_VSTRIPE: t = std::ceil(static_cast<double>(pp[h].n_cols + text_tokens) / block_k); break;
      default: continue;
    }
    tiles += t < n_kb ? t : n_kb;
    ++heads;
  }
  return heads ? tiles / heads : 0.0;
}

// The small query tile is offered to the band groups only when the caller left
// the block shape to the library (an explicit shape applies to every group).
int32_t small_block_q(const svd_tensor_desc& desc, const svd_plan_options* opt) {
  if (opt && (opt->block_q || opt->block_k)) return 0;
  return svd::kernel_small_block_q(desc.D);
}

// Compute units of the current device, 0 when there is none (host-only use).
int device_compute_units() {
  int dev = 0, n_cu = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
  return n_cu > 0 ? n_cu : 0;
}

constexpr int kMaxDenseSplit = 8;

// Key-range split of the dense group.  A work-group occupies a whole compute
// unit, so n items run in ceil(n / n_cu) rounds and the last round is paid in
// full however few items it holds; with s chunks per item the rounds get s
// times shorter and the last one fuller.  The price is the merge pass over the
// partial results.  Picks the s that minimises a rough time estimate, 1 when
// the gain is small.
int choose_dense_split(const svd_tensor_desc& d, int block_q, int block_k, int n_dense_heads, int n_cu,
                       const svd_plan_options* opt) {
  if (n_dense_heads < 1) return 1;
  const int n_key_tiles = (d.L + block_k - 1) / block_k;
  const int cap = n_key_tiles < kMaxDenseSplit ? n_key_tiles : kMaxDenseSplit;
  if (opt && opt->dense_split > 0) return opt->dense_split < cap ? opt->dense_split : cap;
  if (n_cu < 1) return 1;
  const double n = static_cast<double>((d.L + block_q - 1) / block_q) * n_dense_heads * d.B;
  const double t_item = 4.0 * block_q * d.L * d.D / (d.D == 128 ? 4.6e12 : 4.0e12);   // seconds on one unit
  double best_t = 0.0;
  int best = 1;
  for (int sp = 1; sp <= cap; ++sp) {
    double t = std::ceil(n * sp / n_cu) / sp * t_item * (1.0 + 0.01 * (sp - 1));
    if (sp > 1) t += 15e-6 + 2.0 * 4.0 * static_cast<double>(svd::partial_floats(d.D, static_cast<int>(n) * sp)) / 2.5e12;
    if (sp == 1 || t < best_t * (best == 1 ? 0.97 : 1.0)) {
      best_t = t;
      best = sp;
    }
  }
  return best;
}

int count_dense_heads(const Plan& p) {
  for (const svd::Group& g : p.groups)
    if (g.mode == SVD_DENSE) return static_cast<int>(g.heads.size());
  return 0;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool has_text_rows(const Plan& p, const svd::Group& g) {
  return p.text_tokens > 0 && (g.mode == SVD_DIAG || g.mode == SVD_MULTIDIAG || g.mode == SVD_VSTRIPE);
}

// Key-range chunks of the dense launch over the text rows of one sparse group:
// few query tiles (T / block_q per head) against every key, so the key range is
// cut until about one work-group per compute unit exists, chunks of 8 tiles at least
// (the merge pass walks the chunks one after the other).
int choose_text_split(const Plan& p, const svd::Group& g, int n_cu) {
  if (n_cu < 1) return 1;
  const long long base = static_cast<long long>(p.text_tokens / p.block_q) * g.heads.size() * p.desc.B;
  long long s = n_cu / base;   // rounded down: one more item than compute units would cost a whole second round
  const long long cap = p.n_k_blocks / 8 > 64 ? 64 : p.n_k_blocks / 8;
  if (s > cap) s = cap;
  return s < 1 ? 1 : static_cast<int>(s);
}

// Workspace = [compiled lists | padding to 256 bytes | scratch of the dense split |
// scratch of the text-row launches, one area per sparse group].
// Longest padded column list of the plan's vertical-stripe group (0: no such group).
int stripe_gather_pad(const Plan& p) {
  int pad = 0;
  for (const svd::Group& g : p.groups)
    if (g.mode == SVD_VSTRIPE)
      for (const svd::ColumnList& cl : g.columns) pad = std::max(pad, static_cast<int>(cl.cols.size()));
  return pad;
}

size_t workspace_need(const Plan& p, int dense_split, int n_cu, size_t* partial_offset, std::vector<int>* text_split,
                      std::vector<size_t>* text_offset, bool single_launch = false, size_t* counters_offset = nullptr,
                      size_t* gather_offset = nullptr) {
  size_t end = p.ws_image.size() * sizeof(int32_t);
  if (partial_offset) *partial_offset = 0;
  if (gather_offset) *gather_offset = 0;
  for (const svd::Group& g : p.groups) {
    if (g.mode != SVD_VSTRIPE) continue;
    // the gathered K and V rows of the stripe heads (filled by every forward pass)
    const size_t off = align_up(end, 256);
    if (gather_offset) *gather_offset = off;
    end = off + svd::gathered_elements(p.desc.B, static_cast<int>(g.heads.size()), stripe_gather_pad(p), p.desc.D) * 2;
  }
  if (dense_split > 1) {
    const size_t off = align_up(end, 256);
    if (partial_offset) *partial_offset = off;
    const int items = p.n_q_blocks * count_dense_heads(p) * p.desc.B * dense_split;
    end = off + svd::partial_floats(p.desc.D, items) * sizeof(float);
  }
  if (text_split) text_split->assign(p.groups.size(), 1);
  if (text_offset) text_offset->assign(p.groups.size(), 0);
  for (size_t gi = 0; gi < p.groups.size(); ++gi) {
    const svd::Group& g = p.groups[gi];
    if (!has_text_rows(p, g)) continue;
    const int split = choose_text_split(p, g, n_cu);
    if (text_split) (*text_split)[gi] = split;
    if (split <= 1) continue;
    const size_t off = align_up(end, 256);
    if (text_offset) (*text_offset)[gi] = off;
    const int items = (p.text_tokens / p.block_q) * static_cast<int>(g.heads.size()) * p.desc.B * split;
    end = off + svd::partial_floats(p.desc.D, items) * sizeof(float);
  }
  if (single_launch) {   // the queue positions of the layer kernel come last
    const size_t off = align_up(end, 256);
    if (counters_offset) *counters_offset = off;
    end = off + align_up(svd::kLayerCounterWords * sizeof(int32_t), 256);
  }
  return end;
}

svd::AttnLaunch base_launch(const svd_tensor_desc& d, const void* q, const void* k, const void* v,
                            void* out) {
  svd::AttnLaunch a{};
  a.q = static_cast<const __bf16*>(q);
  a.k = static_cast<const __bf16*>(k);
  a.v = static_cast<const __bf16*>(v);
  a.out = static_cast<__bf16*>(out);
  a.B = d.B;
  a.H = d.H;
  a.L = d.L;
  a.D = d.D;
  a.stride_b = d.stride_b;
  a.stride_h = d.stride_h;
  a.stride_l = d.stride_l;
  a.scale_log2e = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(d.D)));
  a.split = 1;
  return a;
}

svd_status check_tensors(const void* q, const void* k, const void* v, const void* out) {
  if (!q || !k || !v || !out) return SVD_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return SVD_ERR_ALIGN;
  return SVD_OK;
}

// One-shot cache: the plan of the previous sparse_vdit_attn_forward call.
struct OneShot {
  std::mutex mu;
  svd_plan* plan = nullptr;
  svd_tensor_desc desc{};
  std::vector<int32_t> table;
  std::vector<int32_t> flat;   // flattened parameters
  void* workspace = nullptr;
  size_t workspace_bytes = 0;
};
OneShot g_oneshot;

std::vector<int32_t> flatten(const svd_tensor_desc& d, const int32_t* table, const svd_head_params* pp) {
  std::vector<int32_t> f;
  for (int h = 0; h < d.H; ++h) {
    const int mode = table[h];
    f.push_back(mode);
    if (mode == SVD_DIAG || mode == SVD_MULTIDIAG) f.push_back(pp[h].half_width);
    if (mode == SVD_MULTIDIAG && pp[h].rearr_frames > 0) {
      f.push_back(-1);   // marks the rearranged form
      f.push_back(pp[h].rearr_first);
      f.push_back(pp[h].rearr_frame_tokens);
      f.push_back(pp[h].rearr_frames);
      continue;
    }
    if (mode == SVD_MULTIDIAG && pp[h].offsets && pp[h].n_offsets > 0) {
      f.push_back(pp[h].n_offsets);
      f.insert(f.end(), pp[h].offsets, pp[h].offsets + pp[h].n_offsets);
    }
    if (mode == SVD_VSTRIPE && pp[h].cols && pp[h].n_cols > 0) {
      f.push_back(pp[h].n_cols);
      f.insert(f.end(), pp[h].cols, pp[h].cols + pp[h].n_cols);
    }
  }
  return f;
}

}  // namespace

extern "C" {

const char* svd_status_string(svd_status s) {
  switch (s) {
    case SVD_OK: return "ok";
    case SVD_ERR_NULL: return "null pointer";
    case SVD_ERR_SHAPE: return "bad shape";
    case SVD_ERR_DTYPE: return "bad dtype";
    case SVD_ERR_ALIGN: return "misaligned tensor";
    case SVD_ERR_MODE: return "mode id outside 0..4";
    case SVD_ERR_PARAMS: return "bad pattern parameters";
    case SVD_ERR_EMPTY_PATTERN: return "a query row keeps no key";
    case SVD_ERR_WORKSPACE: return "workspace missing or too small";
    case SVD_ERR_UNSUPPORTED: return "unsupported block shape, option combination or tensor size";
    case SVD_ERR_HIP: return "HIP error";
    case SVD_ERR_STATIC_LIMIT: return "the layer's lists need more scratch than the library's static buffer holds";
    default: return "unknown status";
  }
}

svd_status svd_default_blocks(int32_t D, int32_t* block_q, int32_t* block_k) {
  if (!block_q || !block_k) return SVD_ERR_NULL;
  if (D != 64 && D != 128) return SVD_ERR_SHAPE;
  int q = 0, k = 0;
  svd::kernel_blocks(D, &q, &k);
  *block_q = q;
  *block_k = k;
  return SVD_OK;
}

svd_status svd_plan_workspace_bytes(const svd_tensor_desc* desc, const int32_t* strategy_table,
                                    const svd_head_params* pattern_params,
                                    const svd_plan_options* options, size_t* bytes) {
  if (!desc || !strategy_table || !pattern_params || !bytes) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  int32_t bq, bk;
  bool native;
  if (svd_status st = resolve_blocks(*desc, options, &bq, &bk, &native)) return st;
  Plan tmp;
  const int n_cu = device_compute_units();
  const int form = layer_form(options, *desc, native, n_cu,
                              mean_tiles_per_item(*desc, strategy_table, pattern_params, bk, options ? options->text_tokens : 0));
  const bool single = form != 0;
  if (svd_status st = svd::compile_plan(*desc, strategy_table, pattern_params, bq, bk,
                                        options ? options->text_tokens : 0, small_block_q(*desc, options), &tmp, single))
    return st;
  // (the split of the dense heads still serves the grouped launches of such a plan: the FP8 path, the per-group calls)
  const int split = native ? choose_dense_split(*desc, bq, bk, count_dense_heads(tmp), n_cu, options) : 1;
  *bytes = workspace_need(tmp, split, native ? n_cu : 0, nullptr, nullptr, nullptr, single, nullptr);
  return SVD_OK;
}

// The segments of the single-launch path, heaviest items first: the dense group,
// the text rows of the sparse groups (dense items over every key), then the
// sparse groups by their average number of key tiles per item, the zero fill last.
static void build_layer_segments(svd_plan* sp) {
  const Plan& p = sp->p;
  const int bq = svd::layer_block_q(p.desc.D);
  const int n_qb = (p.desc.L + bq - 1) / bq;
  svd::LayerLaunch& lay = sp->layer;
  lay = svd::LayerLaunch{};
  struct Cand {
    svd::LayerSegment seg;
    double cost;
  };
  std::vector<Cand> cands;
  auto segment = [&](const svd::Group& g, int kind, int n_q_blocks) {
    svd::LayerSegment sgm{};
    sgm.kind = kind;
    sgm.n_q_blocks = n_q_blocks;
    sgm.n_heads = static_cast<int>(g.heads.size());
    sgm.n_items = n_q_blocks * sgm.n_heads * p.desc.B;
    sgm.heads = static_cast<int>(g.ws_heads);
    sgm.list_id = static_cast<int>(g.ws_list_id);
    sgm.list_table = static_cast<int>(g.ws_list_table);
    return sgm;
  };
  for (const svd::Group& g : p.groups) {
    if (g.mode == SVD_DENSE) {
      svd::LayerSegment dense = segment(g, svd::SEG_DENSE, n_qb);
      if (sp->dense_head_start > 0) {
        // the head start covers the first items of the (batch, head, 256-row tile) order: whole heads, then
        // the first tiles of one more; a 256-row tile is two 128-row items (one at a ragged end)
        const int heads_done = sp->dense_head_start / p.n_q_blocks, tiles_done = sp->dense_head_start % p.n_q_blocks;
        const int per_tile = p.block_q / bq;   // items of the queues per tile of the head start (1: the same tile)
        const int parts = per_tile * tiles_done < n_qb ? per_tile * tiles_done : n_qb;
        dense.first_item = heads_done * n_qb + parts;
        dense.n_items -= dense.first_item;
        sp->dense_group = &g;
      }
      cands.push_back({dense, 2.0 * p.n_k_blocks + 1.0});
    } else if (g.mode == SVD_SKIP) {
      cands.push_back({segment(g, svd::SEG_ZERO, n_qb), 0.0});
    } else if (g.mode == SVD_VSTRIPE) {
      double tiles = 0.0;
      for (size_t t = 0; t < g.heads.size(); ++t) tiles += static_cast<double>(g.columns[g.list_id[t]].cols.size()) / p.block_k;
      cands.push_back({segment(g, svd::SEG_GATHER, n_qb), tiles / g.heads.size()});
    } else {
      double tiles = 0.0;
      for (size_t t = 0; t < g.heads.size(); ++t) tiles += static_cast<double>(g.bands[g.list_id[t]].kv_block_idx.size());
      cands.push_back({segment(g, g.rearranged ? svd::SEG_PBAND : svd::SEG_BAND, g.n_q_blocks),
                       tiles / g.heads.size() / g.n_q_blocks});
    }
    if (has_text_rows(p, g)) cands.push_back({segment(g, svd::SEG_DENSE, p.text_tokens / bq), 2.0 * p.n_k_blocks});
  }
  std::stable_sort(cands.begin(), cands.end(), [](const Cand& a, const Cand& b) { return a.cost > b.cost; });
  lay.n_segments = 0;
  for (const Cand& c : cands)
    if (lay.n_segments < svd::kMaxSegments) lay.seg[lay.n_segments++] = c.seg;
  lay.counters = reinterpret_cast<int*>(static_cast<char*>(p.device_workspace) + sp->counters_offset);
}

// with_side_streams = false: the plan creates no streams or events of its own and
// runs its groups one after the other on the caller's stream.
static svd_status create_plan(svd_plan** plan, const svd_tensor_desc* desc,
                              const int32_t* strategy_table, const svd_head_params* pattern_params,
                              const svd_plan_options* options, void* device_workspace,
                              size_t workspace_bytes, void* hip_stream, bool with_side_streams) {
  if (!plan || !desc || !strategy_table || !pattern_params) return SVD_ERR_NULL;
  *plan = nullptr;
  if (svd_status st = svd::validate_desc(desc)) return st;
  int32_t bq, bk;
  bool native;
  if (svd_status st = resolve_blocks(*desc, options, &bq, &bk, &native)) return st;
  svd_plan* sp = new (std::nothrow) svd_plan();
  if (!sp) return SVD_ERR_HIP;
  svd_status st = SVD_OK;
  for (int h = 0; h < desc->H; ++h)
    if (strategy_table[h] < SVD_DENSE || strategy_table[h] > SVD_VSTRIPE) {
      delete sp;
      return SVD_ERR_MODE;
    }
  const int form = device_workspace
                       ? layer_form(options, *desc, native, device_compute_units(),
                                    mean_tiles_per_item(*desc, strategy_table, pattern_params, bk, options ? options->text_tokens : 0))
                       : 0;
  if (device_workspace && options && (options->single_launch == 1 || options->single_launch == 3) && device_compute_units() < 1) {
    delete sp;
    return SVD_ERR_HIP;   // the layer kernel is sized from the compute-unit count
  }
  const bool single = form != 0;
  try {
    st = svd::compile_plan(*desc, strategy_table, pattern_params, bq, bk, options ? options->text_tokens : 0,
                           small_block_q(*desc, options), &sp->p, single);
  } catch (...) {
    st = SVD_ERR_UNSUPPORTED;
  }
  if (st != SVD_OK) {
    delete sp;
    return st;
  }
  if (device_workspace) {
    const int n_cu_ws = device_compute_units();
    sp->dense_split = native ? choose_dense_split(*desc, bq, bk, count_dense_heads(sp->p), n_cu_ws, options) : 1;
    const size_t need = workspace_need(sp->p, sp->dense_split, native ? n_cu_ws : 0, &sp->partial_offset,
                                       &sp->text_split, &sp->text_partial_offset, single, &sp->counters_offset,
                                       &sp->gather_offset);
    sp->gather_pad = stripe_gather_pad(sp->p);

    if (workspace_bytes < need || !aligned16(device_workspace)) {
      delete sp;
      return SVD_ERR_WORKSPACE;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(device_workspace, sp->p.ws_image.data(), sp->p.ws_image.size() * sizeof(int32_t),
                       hipMemcpyHostToDevice, stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess) {
      delete sp;
      return SVD_ERR_HIP;
    }
    sp->p.device_workspace = device_workspace;
    sp->p.launchable = native;
    if (single) {
      sp->single_launch = true;
      sp->n_cu = n_cu_ws;
      sp->head_start_asked = form == 3;
      if (form == 3) {
        const long long items = static_cast<long long>(sp->p.n_q_blocks) * count_dense_heads(sp->p) * desc->B;
        sp->dense_head_start = static_cast<int>(items / n_cu_ws * n_cu_ws);
      }
      build_layer_segments(sp);
    }
    if (native && with_side_streams && !single && !(options && options->no_fork)) {
      bool ok = hipEventCreateWithFlags(&sp->fork, hipEventDisableTiming) == hipSuccess;
      for (int i = 0; ok && i < kSideStreams; ++i)
        ok = hipStreamCreateWithFlags(&sp->side[i], hipStreamNonBlocking) == hipSuccess &&
             hipEventCreateWithFlags(&sp->join[i], hipEventDisableTiming) == hipSuccess;
      // Forking pays when the last round of the heaviest group leaves most compute
      // units idle (one work-group occupies a whole unit); otherwise the groups
      // run one after the other, which keeps one head's K/V hot in L2 at a time.
      int dev = 0, n_cu = 0;
      if (ok && hipGetDevice(&dev) == hipSuccess &&
          hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n_cu > 0) {
        const svd::Group* heavy = nullptr;
        static const int order[4] = {SVD_DENSE, SVD_DIAG, SVD_MULTIDIAG, SVD_VSTRIPE};
        for (int mode : order) {
          for (const svd::Group& g : sp->p.groups)
            if (g.mode == mode && !heavy) heavy = &g;
        }
        if (heavy) {
          const long long items = static_cast<long long>(heavy->n_q_blocks) * heavy->heads.size() * desc->B *
                                  (heavy->mode == SVD_DENSE ? sp->dense_split : 1);
          const long long tail = items % n_cu;
          sp->concurrent = tail != 0 && 2 * tail < n_cu;
        }
      }
    }
  }
  *plan = sp;
  return SVD_OK;
}

svd_status svd_plan_create(svd_plan** plan, const svd_tensor_desc* desc,
                           const int32_t* strategy_table, const svd_head_params* pattern_params,
                           const svd_plan_options* options, void* device_workspace,
                           size_t workspace_bytes, void* hip_stream) {
  return create_plan(plan, desc, strategy_table, pattern_params, options, device_workspace, workspace_bytes,
                     hip_stream, true);
}

svd_status svd_plan_destroy(svd_plan* plan) {
  if (!plan) return SVD_ERR_NULL;
  delete plan;
  return SVD_OK;
}

svd_status svd_plan_dense_split(const svd_plan* plan, int32_t* dense_split) {
  if (!plan || !dense_split) return SVD_ERR_NULL;
  *dense_split = plan->dense_split;
  return SVD_OK;
}

svd_status svd_plan_single_launch(const svd_plan* plan, int32_t* single_launch) {
  if (!plan || !single_launch) return SVD_ERR_NULL;
  *single_launch = plan->single_launch ? (plan->dense_head_start > 0 || plan->head_start_asked ? 3 : 1) : 0;
  return SVD_OK;
}

svd_status svd_plan_num_groups(const svd_plan* plan, int32_t* n_groups) {
  if (!plan || !n_groups) return SVD_ERR_NULL;
  *n_groups = static_cast<int32_t>(plan->p.groups.size());
  return SVD_OK;
}

svd_status svd_plan_group_blocks(const svd_plan* plan, int32_t group, int32_t* block_q, int32_t* block_k) {
  if (!plan) return SVD_ERR_NULL;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  if (block_q) *block_q = plan->p.groups[group].block_q;
  if (block_k) *block_k = plan->p.block_k;
  return SVD_OK;
}

svd_status svd_plan_group_rearranged(const svd_plan* plan, int32_t group, int32_t* rearranged) {
  if (!plan || !rearranged) return SVD_ERR_NULL;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  *rearranged = plan->p.groups[group].rearranged ? 1 : 0;
  return SVD_OK;
}

svd_status svd_plan_row_map(const svd_plan* plan, int32_t group, int32_t list, int32_t* padded_len,
                            const int32_t** row_map) {
  if (!plan) return SVD_ERR_NULL;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  const svd::Group& g = plan->p.groups[group];
  if (!g.rearranged || list < 0 || list >= static_cast<int32_t>(g.bands.size())) return SVD_ERR_SHAPE;
  if (padded_len) *padded_len = static_cast<int32_t>(g.bands[list].row_map.size());
  if (row_map) *row_map = g.bands[list].row_map.data();
  return SVD_OK;
}

svd_status svd_plan_group_info(const svd_plan* plan, int32_t group, int32_t* mode, int32_t* n_heads,
                               const int32_t** heads, const int32_t** list_id, int32_t* n_lists) {
  if (!plan) return SVD_ERR_NULL;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  const svd::Group& g = plan->p.groups[group];
  if (mode) *mode = g.mode;
  if (n_heads) *n_heads = static_cast<int32_t>(g.heads.size());
  if (heads) *heads = g.heads.data();
  if (list_id) *list_id = g.list_id.data();
  if (n_lists) *n_lists = static_cast<int32_t>(g.bands.size() + g.columns.size());
  return SVD_OK;
}

svd_status svd_plan_band_list(const svd_plan* plan, int32_t group, int32_t list,
                              int32_t* n_q_blocks, const int32_t** row_ptr,
                              const int32_t** kv_block_idx, const int32_t** flags,
                              const int32_t** run_first, const int32_t** run_count,
                              int32_t* n_runs, const int32_t** runs) {
  if (!plan) return SVD_ERR_NULL;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  const svd::Group& g = plan->p.groups[group];
  if (list < 0 || list >= static_cast<int32_t>(g.bands.size())) return SVD_ERR_SHAPE;
  const svd::BandList& bl = g.bands[list];
  if (n_q_blocks) *n_q_blocks = g.n_q_blocks;
  if (row_ptr) *row_ptr = bl.row_ptr.data();
  if (kv_block_idx) *kv_block_idx = bl.kv_block_idx.data();
  if (flags) *flags = bl.flags.data();
  if (run_first) *run_first = bl.run_first.data();
  if (run_count) *run_count = bl.run_count.data();
  if (n_runs) *n_runs = static_cast<int32_t>(bl.runs.size() / 2);
  if (runs) *runs = bl.runs.data();
  return SVD_OK;
}

svd_status svd_plan_column_list(const svd_plan* plan, int32_t group, int32_t list,
                                int32_t* n_cols, int32_t* padded_len, const int32_t** cols) {
  if (!plan) return SVD_ERR_NULL;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  const svd::Group& g = plan->p.groups[group];
  if (list < 0 || list >= static_cast<int32_t>(g.columns.size())) return SVD_ERR_SHAPE;
  const svd::ColumnList& cl = g.columns[list];
  if (n_cols) *n_cols = cl.n_cols;
  if (padded_len) *padded_len = static_cast<int32_t>(cl.cols.size());
  if (cols) *cols = cl.cols.data();
  return SVD_OK;
}

// fp8: the lists the FP8 path walks (band groups always on the small query tile)
static void group_work(const Plan& p, const svd::Group& g, int64_t* tiles, double* area, double* pairs, bool fp8 = false) {
  const double L = p.desc.L;
  const std::vector<svd::BandList>& bands = fp8 && !g.bands_small.empty() ? g.bands_small : g.bands;
  for (size_t t = 0; t < g.heads.size(); ++t) {
    switch (g.mode) {
      case SVD_DENSE:
        *tiles += static_cast<int64_t>(p.n_q_blocks) * p.n_k_blocks;
        *area += L * L;
        *pairs += L * L;
        break;
      case SVD_DIAG:
      case SVD_MULTIDIAG: {
        const svd::BandList& bl = bands[g.list_id[t]];
        *tiles += static_cast<int64_t>(bl.kv_block_idx.size());
        *area += bl.tile_area;
        *pairs += bl.kept_pairs;   // text borders included
        break;
      }
      case SVD_VSTRIPE: {
        const svd::ColumnList& cl = g.columns[g.list_id[t]];
        *tiles += static_cast<int64_t>(p.n_q_blocks) * static_cast<int64_t>(cl.cols.size() / p.block_k);
        *area += L * cl.n_cols;
        *pairs += L * cl.n_cols + static_cast<double>(p.text_tokens) * (L - cl.n_cols);
        break;
      }
      default:
        break;
    }
    // the text rows of a sparse head are computed densely on top of its list
    if (has_text_rows(p, g)) {
      *tiles += static_cast<int64_t>(p.text_tokens / p.block_q) * p.n_k_blocks;
      *area += static_cast<double>(p.text_tokens) * L;
    }
  }
}

svd_status svd_plan_work(const svd_plan* plan, int64_t* computed_tiles, double* computed_flops,
                         double* kept_pairs) {
  if (!plan) return SVD_ERR_NULL;
  const Plan& p = plan->p;
  int64_t tiles = 0;
  double area = 0.0, pairs = 0.0;
  for (const svd::Group& g : p.groups) group_work(p, g, &tiles, &area, &pairs);
  if (computed_tiles) *computed_tiles = tiles * p.desc.B;
  if (computed_flops) *computed_flops = 4.0 * p.desc.D * area * p.desc.B;
  if (kept_pairs) *kept_pairs = pairs * p.desc.B;
  return SVD_OK;
}

svd_status svd_plan_group_work_fp8(const svd_plan* plan, int32_t group, int64_t* computed_tiles,
                                   double* computed_flops) {
  if (!plan) return SVD_ERR_NULL;
  const Plan& p = plan->p;
  if (group < -1 || group >= static_cast<int32_t>(p.groups.size())) return SVD_ERR_SHAPE;
  int64_t tiles = 0;
  double area = 0.0, pairs = 0.0;
  for (int32_t gi = 0; gi < static_cast<int32_t>(p.groups.size()); ++gi)
    if (group < 0 || gi == group) group_work(p, p.groups[gi], &tiles, &area, &pairs, true);
  if (computed_tiles) *computed_tiles = tiles * p.desc.B;
  if (computed_flops) *computed_flops = 4.0 * p.desc.D * area * p.desc.B;
  return SVD_OK;
}

svd_status svd_plan_group_work(const svd_plan* plan, int32_t group, int64_t* computed_tiles,
                               double* computed_flops, double* kept_pairs) {
  if (!plan) return SVD_ERR_NULL;
  const Plan& p = plan->p;
  if (group < 0 || group >= static_cast<int32_t>(p.groups.size())) return SVD_ERR_SHAPE;
  int64_t tiles = 0;
  double area = 0.0, pairs = 0.0;
  group_work(p, p.groups[group], &tiles, &area, &pairs);
  if (computed_tiles) *computed_tiles = tiles * p.desc.B;
  if (computed_flops) *computed_flops = 4.0 * p.desc.D * area * p.desc.B;
  if (kept_pairs) *kept_pairs = pairs * p.desc.B;
  return SVD_OK;
}

// The dense launch over the text rows of a sparse group, derived from the group's own launch.
static svd::AttnLaunch text_rows_launch(const svd_plan& sp, const svd::Group& g, const svd::AttnLaunch& a) {
  const Plan& p = sp.p;
  const size_t gi = static_cast<size_t>(&g - p.groups.data());
  svd::AttnLaunch d = a;
  d.n_q_blocks = p.text_tokens / p.block_q;
  d.n_items = d.n_q_blocks * d.n_heads * d.B;
  d.split = gi < sp.text_split.size() ? sp.text_split[gi] : 1;
  d.partial = nullptr;
  if (d.split > 1) {
    d.n_items *= d.split;
    d.partial = reinterpret_cast<float*>(static_cast<char*>(p.device_workspace) + sp.text_partial_offset[gi]);
  }
  return d;
}

static svd_status launch_group(const svd_plan& sp, const svd::Group& g, const void* q, const void* k,
                               const void* v, void* out, hipStream_t stream) {
  const Plan& p = sp.p;
  const int* ws = static_cast<const int*>(p.device_workspace);
  svd::AttnLaunch a = base_launch(p.desc, q, k, v, out);
  a.n_q_blocks = g.n_q_blocks;
  a.n_heads = static_cast<int>(g.heads.size());
  a.n_items = a.n_q_blocks * a.n_heads * a.B;
  a.heads = ws + g.ws_heads;
  a.list_id = ws + g.ws_list_id;
  a.ws = ws;
  a.list_table = static_cast<int>(g.ws_list_table);
  const bool small_q = g.block_q != p.block_q;   // band group compiled for the small query tile
  hipError_t err;
  if (g.mode == SVD_SKIP) {
    err = svd::launch_zero_heads(a, stream);
  } else {
    const int kmode = g.mode == SVD_DENSE ? svd::MODE_DENSE
                      : g.mode == SVD_VSTRIPE ? svd::MODE_GATHER
                      : g.rearranged ? svd::MODE_PBAND : svd::MODE_BAND;
    if (g.mode == SVD_DENSE && sp.dense_split > 1) {
      a.split = sp.dense_split;
      a.n_items *= a.split;
      a.partial = reinterpret_cast<float*>(static_cast<char*>(p.device_workspace) + sp.partial_offset);
    }
    if (g.mode == SVD_VSTRIPE) {
      a.gathered = reinterpret_cast<__bf16*>(static_cast<char*>(p.device_workspace) + sp.gather_offset);
      a.gather_pad = sp.gather_pad;
      a.skip_q_blocks = p.text_tokens / p.block_q;   // the text rows come from the dense launch below
      err = svd::launch_gather_kv(a, stream);
      if (err != hipSuccess) return SVD_ERR_HIP;
    }
    err = svd::launch_attention(a, kmode, stream, small_q);
    if (err == hipSuccess && a.split > 1) err = svd::launch_combine(a, stream);
    if (err == hipSuccess && has_text_rows(p, g)) {
      // Section 4.1.1: text queries see every key.  Their rows (the first
      // T / block_q query tiles of every head of the group) are computed by the
      // dense kernel, after the group's own launch on the same stream.
      svd::AttnLaunch d = text_rows_launch(sp, g, a);
      err = svd::launch_attention(d, svd::MODE_DENSE, stream);
      if (err == hipSuccess && d.split > 1) err = svd::launch_combine(d, stream);
    }
  }
  return err == hipSuccess ? SVD_OK : SVD_ERR_HIP;
}

static svd_status check_launchable(const svd_plan* plan, const void* q, const void* k, const void* v,
                                   const void* out, hipStream_t stream) {
  if (!plan) return SVD_ERR_NULL;
  if (svd_status st = check_tensors(q, k, v, out)) return st;
  if (!plan->p.device_workspace) return SVD_ERR_WORKSPACE;
  if (!plan->p.launchable) return SVD_ERR_UNSUPPORTED;
  // A layer with a text prefix is not recorded into a stream capture: a run that
  // captured and replayed such layers ended in a host-side heap abort whose cause
  // is not known; until it is, the combination is refused before anything is enqueued.
  if (plan->p.text_tokens > 0) {
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) return SVD_ERR_HIP;
    if (capture != hipStreamCaptureStatusNone) return SVD_ERR_UNSUPPORTED;
  }
  return SVD_OK;
}

svd_status svd_attn_forward_planned(const svd_plan* plan, const void* q, const void* k, const void* v,
                                    void* out, void* hip_stream) {
  if (svd_status st = check_launchable(plan, q, k, v, out, static_cast<hipStream_t>(hip_stream))) return st;
  const Plan& p = plan->p;
  hipStream_t main_stream = static_cast<hipStream_t>(hip_stream);
  if (plan->single_launch) {
    if (plan->dense_head_start > 0) {
      // whole rounds of the dense kernel on its 256-row tile; what is left of the dense group is in the queues
      const svd::Group& g = *plan->dense_group;
      const int* ws = static_cast<const int*>(p.device_workspace);
      svd::AttnLaunch a = base_launch(p.desc, q, k, v, out);
      a.n_q_blocks = g.n_q_blocks;
      a.n_heads = static_cast<int>(g.heads.size());
      a.n_items = plan->dense_head_start;
      a.heads = ws + g.ws_heads;
      a.list_id = ws + g.ws_list_id;
      a.ws = ws;
      a.list_table = static_cast<int>(g.ws_list_table);
      if (svd::launch_attention(a, svd::MODE_DENSE, main_stream) != hipSuccess) return SVD_ERR_HIP;
    }
    svd::LayerLaunch lay = plan->layer;
    lay.a = base_launch(p.desc, q, k, v, out);
    lay.a.ws = static_cast<const int*>(p.device_workspace);
    for (const svd::Group& g : p.groups) {
      if (g.mode != SVD_VSTRIPE) continue;
      // the stripe heads' K and V rows are gathered ahead of the layer kernel
      svd::AttnLaunch a = lay.a;
      a.n_heads = static_cast<int>(g.heads.size());
      a.heads = lay.a.ws + g.ws_heads;
      a.list_id = lay.a.ws + g.ws_list_id;
      a.list_table = static_cast<int>(g.ws_list_table);
      a.gathered = reinterpret_cast<__bf16*>(static_cast<char*>(p.device_workspace) + plan->gather_offset);
      a.gather_pad = plan->gather_pad;
      if (svd::launch_gather_kv(a, main_stream) != hipSuccess) return SVD_ERR_HIP;
      lay.a.gathered = a.gathered;
      lay.a.gather_pad = a.gather_pad;
      lay.a.skip_q_blocks = p.text_tokens / svd::layer_block_q(p.desc.D);   // text rows are items of the dense kind
    }
    return svd::launch_layer(lay, plan->n_cu, main_stream) == hipSuccess ? SVD_OK : SVD_ERR_HIP;
  }
  // heaviest first: dense, then the band groups, the gathers, and the zero fill
  static const int order[5] = {SVD_DENSE, SVD_DIAG, SVD_MULTIDIAG, SVD_VSTRIPE, SVD_SKIP};
  constexpr int kMaxGroups = 6;   // the five modes plus the rearranged multi-diagonal group
  const svd::Group* seq[kMaxGroups];
  int n = 0;
  for (int mode : order)
    for (const svd::Group& g : p.groups)
      if (g.mode == mode && n < kMaxGroups) seq[n++] = &g;
  if (!plan->concurrent || n < 2) {
    for (int i = 0; i < n; ++i)
      if (svd_status st = launch_group(*plan, *seq[i], q, k, v, out, main_stream)) return st;
    return SVD_OK;
  }
  // fork: the first group stays on the caller's stream, the others go round-robin
  // to the side streams; join: the caller's stream waits for every side stream
  if (hipEventRecord(plan->fork, main_stream) != hipSuccess) return SVD_ERR_HIP;
  bool used[kSideStreams] = {false, false, false};
  svd_status status = SVD_OK;
  for (int i = 0; i < n && status == SVD_OK; ++i) {
    hipStream_t s = main_stream;
    if (i > 0) {
      const int k_side = (i - 1) % kSideStreams;
      s = plan->side[k_side];
      if (!used[k_side]) {
        if (hipStreamWaitEvent(s, plan->fork, 0) != hipSuccess) {
          status = SVD_ERR_HIP;
          break;
        }
        used[k_side] = true;
      }
    }
    status = launch_group(*plan, *seq[i], q, k, v, out, s);
  }
  // joined also after a failed launch, so that whatever was enqueued stays ordered on the caller's stream
  for (int i = 0; i < kSideStreams; ++i) {
    if (!used[i]) continue;
    if (hipEventRecord(plan->join[i], plan->side[i]) != hipSuccess ||
        hipStreamWaitEvent(main_stream, plan->join[i], 0) != hipSuccess)
      status = status == SVD_OK ? SVD_ERR_HIP : status;
  }
  return status;
}

svd_status svd_attn_forward_group(const svd_plan* plan, int32_t group, const void* q, const void* k,
                                  const void* v, void* out, void* hip_stream) {
  if (svd_status st = check_launchable(plan, q, k, v, out, static_cast<hipStream_t>(hip_stream))) return st;
  const Plan& p = plan->p;
  if (group < 0 || group >= static_cast<int32_t>(p.groups.size())) return SVD_ERR_SHAPE;
  return launch_group(*plan, p.groups[group], q, k, v, out, static_cast<hipStream_t>(hip_stream));
}

svd_status svd_dense_attn_forward(const void* q, const void* k, const void* v, void* out,
                                  const svd_tensor_desc* desc, void* hip_stream) {
  if (!desc) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  if (svd_status st = check_tensors(q, k, v, out)) return st;
  int bq = 0, bk = 0;
  svd::kernel_blocks(desc->D, &bq, &bk);
  svd::AttnLaunch a = base_launch(*desc, q, k, v, out);
  a.n_q_blocks = (desc->L + bq - 1) / bq;
  a.n_heads = desc->H;
  a.n_items = a.n_q_blocks * a.n_heads * a.B;
  if (svd::launch_attention(a, svd::MODE_DENSE, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SVD_ERR_HIP;
  return SVD_OK;
}

svd_status sparse_vdit_attn_forward(const void* q, const void* k, const void* v,
                                    const int32_t* strategy_table,
                                    const svd_head_params* pattern_params, void* out,
                                    const svd_tensor_desc* desc, void* device_workspace,
                                    size_t workspace_bytes, void* hip_stream) {
  if (!desc || !strategy_table || !pattern_params) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  if (svd_status st = check_tensors(q, k, v, out)) return st;
  if (!device_workspace) return SVD_ERR_WORKSPACE;
  for (int h = 0; h < desc->H; ++h)
    if (strategy_table[h] < SVD_DENSE || strategy_table[h] > SVD_VSTRIPE) return SVD_ERR_MODE;
  std::lock_guard<std::mutex> lock(g_oneshot.mu);
  std::vector<int32_t> table(strategy_table, strategy_table + desc->H);
  std::vector<int32_t> flat = flatten(*desc, strategy_table, pattern_params);
  const bool hit = g_oneshot.plan && std::memcmp(&g_oneshot.desc, desc, sizeof(*desc)) == 0 &&
                   g_oneshot.table == table && g_oneshot.flat == flat &&
                   g_oneshot.workspace == device_workspace && g_oneshot.workspace_bytes == workspace_bytes;
  if (!hit) {
    svd_plan* fresh = nullptr;
    if (svd_status st = svd_plan_create(&fresh, desc, strategy_table, pattern_params, nullptr,
                                        device_workspace, workspace_bytes, hip_stream))
      return st;
    if (g_oneshot.plan) svd_plan_destroy(g_oneshot.plan);
    g_oneshot.plan = fresh;
    g_oneshot.desc = *desc;
    g_oneshot.table.swap(table);
    g_oneshot.flat.swap(flat);
    g_oneshot.workspace = device_workspace;
    g_oneshot.workspace_bytes = workspace_bytes;
  }
  return svd_attn_forward_planned(g_oneshot.plan, q, k, v, out, hip_stream);
}

// The one-shot call for callers that cannot allocate device memory: the plan's
// workspace is the library's own static buffer of the current device.  The cache
// is per device (each device has its own buffer); no stream, event or device
// memory is created here.
namespace {
constexpr int kMaxStaticDevices = 64;
struct StaticShot {
  svd_plan* plan = nullptr;
  svd_tensor_desc desc{};
  std::vector<int32_t> table, flat;
  hipStream_t last_stream = nullptr;
  bool used = false;
};
std::mutex g_static_mu;
StaticShot g_static[kMaxStaticDevices];
}  // namespace

svd_status sparse_vdit_attn_forward_static(const void* q, const void* k, const void* v,
                                           const int32_t* strategy_table,
                                           const svd_head_params* pattern_params, void* out,
                                           const svd_tensor_desc* desc, void* hip_stream) {
  if (!desc || !strategy_table || !pattern_params) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  if (svd_status st = check_tensors(q, k, v, out)) return st;
  for (int h = 0; h < desc->H; ++h)
    if (strategy_table[h] < SVD_DENSE || strategy_table[h] > SVD_VSTRIPE) return SVD_ERR_MODE;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return SVD_ERR_HIP;
  if (dev < 0 || dev >= kMaxStaticDevices) return SVD_ERR_UNSUPPORTED;
  void* scratch = nullptr;
  size_t scratch_bytes = 0;
  if (svd::static_scratch(&scratch, &scratch_bytes) != hipSuccess) return SVD_ERR_HIP;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  std::lock_guard<std::mutex> lock(g_static_mu);
  StaticShot& c = g_static[dev];
  std::vector<int32_t> table(strategy_table, strategy_table + desc->H);
  std::vector<int32_t> flat = flatten(*desc, strategy_table, pattern_params);
  const bool hit = c.plan && std::memcmp(&c.desc, desc, sizeof(*desc)) == 0 && c.table == table && c.flat == flat;
  if (!hit) {
    // A new plan overwrites the lists in the buffer.  That is a copy and a
    // synchronisation, which a capturing stream cannot record; and whatever the
    // previous call enqueued on another stream must have finished with the buffer.
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) return SVD_ERR_HIP;
    if (capture != hipStreamCaptureStatusNone) return SVD_ERR_UNSUPPORTED;
    if (c.used && c.last_stream != stream && hipDeviceSynchronize() != hipSuccess) return SVD_ERR_HIP;
    // the split of the dense heads is the library's choice unless its partial results
    // do not fit the buffer: then the dense heads run unsplit
    svd_plan_options opt{};
    size_t need = 0;
    if (svd_status st = svd_plan_workspace_bytes(desc, strategy_table, pattern_params, &opt, &need)) return st;
    if (need > scratch_bytes) {
      opt.dense_split = 1;
      if (svd_status st = svd_plan_workspace_bytes(desc, strategy_table, pattern_params, &opt, &need)) return st;
    }
    if (need > scratch_bytes) return SVD_ERR_STATIC_LIMIT;
    svd_plan* fresh = nullptr;
    if (svd_status st = create_plan(&fresh, desc, strategy_table, pattern_params, &opt, scratch, scratch_bytes,
                                    hip_stream, false))
      return st;
    if (c.plan) svd_plan_destroy(c.plan);
    c.plan = fresh;
    c.desc = *desc;
    c.table.swap(table);
    c.flat.swap(flat);
  }
  c.last_stream = stream;
  c.used = true;
  return svd_attn_forward_planned(c.plan, q, k, v, out, hip_stream);
}

// ---------------------------------------------------------------------------
// Offline search step (Section 4.2 "Offline Sparse Diffusion Search", Eq. 2-3,
// Algorithm 1)
// ---------------------------------------------------------------------------

static svd::TensorView view_of(const svd_tensor_desc& d) {
  return svd::TensorView{d.B, d.H, d.L, d.D, d.stride_b, d.stride_h, d.stride_l};
}

static svd_tensor_desc contiguous_desc(const svd_tensor_desc& d) {
  svd_tensor_desc c = d;
  c.stride_l = d.D;
  c.stride_h = static_cast<int64_t>(d.L) * d.D;
  c.stride_b = c.stride_h * d.H;
  return c;
}

svd_status svd_head_mse_workspace_bytes(const svd_tensor_desc* desc, size_t* bytes) {
  if (!desc || !bytes) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  *bytes = svd::mse_scratch_floats(view_of(*desc)) * sizeof(float);
  return SVD_OK;
}

svd_status svd_head_mse(const void* o, const void* o_ref, const svd_tensor_desc* desc, float* mse,
                        void* device_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!o || !o_ref || !desc || !mse) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  if (!aligned16(o) || !aligned16(o_ref)) return SVD_ERR_ALIGN;
  const svd::TensorView t = view_of(*desc);
  if (!device_workspace || workspace_bytes < svd::mse_scratch_floats(t) * sizeof(float) ||
      (reinterpret_cast<uintptr_t>(device_workspace) & 3u))
    return SVD_ERR_WORKSPACE;
  const hipError_t e = svd::launch_head_mse(static_cast<const __bf16*>(o), static_cast<const __bf16*>(o_ref), t, mse,
                                            static_cast<float*>(device_workspace), static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SVD_OK : SVD_ERR_HIP;
}

svd_status svd_plan_head_sparsity(const svd_plan* plan, double* sparsity) {
  if (!plan || !sparsity) return SVD_ERR_NULL;
  const Plan& p = plan->p;
  const double all = static_cast<double>(p.desc.L) * static_cast<double>(p.desc.L);
  for (const svd::Group& g : p.groups) {
    for (size_t t = 0; t < g.heads.size(); ++t) {
      double kept = 0.0;
      if (g.mode == SVD_DENSE) kept = all;
      else if (g.mode == SVD_DIAG || g.mode == SVD_MULTIDIAG) kept = g.bands[g.list_id[t]].kept_pairs;
      else if (g.mode == SVD_VSTRIPE) {
        const double n_cols = g.columns[g.list_id[t]].n_cols;
        kept = n_cols * p.desc.L + static_cast<double>(p.text_tokens) * (p.desc.L - n_cols);
      }
      sparsity[g.heads[t]] = 1.0 - kept / all;
    }
  }
  return SVD_OK;
}

svd_status svd_plan_head_block_sparsity(const svd_plan* plan, double* sparsity) {
  if (!plan || !sparsity) return SVD_ERR_NULL;
  const Plan& p = plan->p;
  for (const svd::Group& g : p.groups) {
    const double all = static_cast<double>(g.n_q_blocks) * p.n_k_blocks;
    const double text_rows = has_text_rows(p, g) ? static_cast<double>(p.text_tokens / g.block_q) * p.n_k_blocks : 0.0;
    for (size_t t = 0; t < g.heads.size(); ++t) {
      double listed = 0.0;
      if (g.mode == SVD_DENSE) listed = all;
      else if (g.mode == SVD_DIAG || g.mode == SVD_MULTIDIAG)
        listed = static_cast<double>(g.bands[g.list_id[t]].kv_block_idx.size()) + text_rows;
      else if (g.mode == SVD_VSTRIPE)
        listed = static_cast<double>(g.n_q_blocks) * static_cast<double>(g.columns[g.list_id[t]].cols.size() / p.block_k) +
                 text_rows;   // the stripe launch covers every query tile; the text rows are then computed densely on top
      sparsity[g.heads[t]] = 1.0 - listed / all;
    }
  }
  return SVD_OK;
}

svd_status svd_search_select(int32_t H, const float* mse, const double* sparsity, double lambda, double epsilon,
                             int32_t* table, double* loss) {
  if (!mse || !sparsity || !table) return SVD_ERR_NULL;
  if (H < 1) return SVD_ERR_SHAPE;
  static const int32_t sparse_modes[4] = {SVD_SKIP, SVD_DIAG, SVD_MULTIDIAG, SVD_VSTRIPE};
  for (int32_t h = 0; h < H; ++h) {
    int above = 0, best = 0;
    double best_loss = 0.0;
    for (int i = 0; i < 4; ++i) {
      const double l = static_cast<double>(mse[i * H + h]) + lambda * (1.0 - sparsity[i * H + h]);   // Eq. 2
      if (loss) loss[i * H + h] = l;
      if (l > epsilon) ++above;
      if (i == 0 || l < best_loss) {   // strict: ties go to the lower mode id
        best_loss = l;
        best = i;
      }
    }
    table[h] = above >= 4 ? SVD_DENSE : sparse_modes[best];   // Eq. 3
  }
  return SVD_OK;
}

svd_status svd_select_heads(const void* const* o_modes, const svd_tensor_desc* src_desc, const int32_t* table,
                            void* out, const svd_tensor_desc* out_desc, void* hip_stream) {
  if (!o_modes || !src_desc || !table || !out || !out_desc) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(src_desc)) return st;
  if (svd_status st = svd::validate_desc(out_desc)) return st;
  if (src_desc->B != out_desc->B || src_desc->H != out_desc->H || src_desc->L != out_desc->L ||
      src_desc->D != out_desc->D)
    return SVD_ERR_SHAPE;
  if (src_desc->H > svd::kMaxSelectHeads) return SVD_ERR_UNSUPPORTED;
  if (!aligned16(out)) return SVD_ERR_ALIGN;
  const __bf16* src[5];
  bool used[5] = {false, false, false, false, false};
  for (int h = 0; h < src_desc->H; ++h) {
    if (table[h] < SVD_DENSE || table[h] > SVD_VSTRIPE) return SVD_ERR_MODE;
    used[table[h]] = true;
  }
  for (int m = 0; m < 5; ++m) {
    if (used[m] && !o_modes[m]) return SVD_ERR_NULL;
    if (o_modes[m] && !aligned16(o_modes[m])) return SVD_ERR_ALIGN;
    src[m] = static_cast<const __bf16*>(o_modes[m]);
  }
  const hipError_t e = svd::launch_select_heads(src, view_of(*src_desc), table, static_cast<__bf16*>(out),
                                                view_of(*out_desc), static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? SVD_OK : SVD_ERR_HIP;
}

// Workspace of svd_search_layer: five contiguous output tensors, the largest
// plan workspace of the five single-mode tables, the reduction scratch, and
// 4 * H floats for the per-head MSEs.
namespace {
struct SearchLayout {
  size_t out_bytes = 0, plan_off = 0, plan_bytes = 0, mse_scratch_off = 0, mse_off = 0, total = 0;
};

svd_status search_layout(const svd_tensor_desc& desc, const svd_head_params* const* params_by_mode, SearchLayout* lay) {
  lay->out_bytes = align_up(static_cast<size_t>(desc.B) * desc.H * desc.L * desc.D * 2, 256);
  std::vector<int32_t> table(desc.H);
  std::vector<svd_head_params> none(desc.H);
  for (int mode = SVD_SKIP; mode <= SVD_VSTRIPE; ++mode) {
    std::fill(table.begin(), table.end(), mode);
    const svd_head_params* pp = (mode >= SVD_DIAG) ? params_by_mode[mode] : none.data();
    if (!pp) return SVD_ERR_NULL;
    size_t bytes = 0;
    const svd_tensor_desc c = contiguous_desc(desc);
    if (svd_status st = svd_plan_workspace_bytes(&c, table.data(), pp, nullptr, &bytes)) return st;
    lay->plan_bytes = bytes > lay->plan_bytes ? bytes : lay->plan_bytes;
  }
  lay->plan_bytes = align_up(lay->plan_bytes, 256);
  lay->plan_off = 5 * lay->out_bytes;
  lay->mse_scratch_off = lay->plan_off + lay->plan_bytes;
  lay->mse_off = lay->mse_scratch_off + align_up(svd::mse_scratch_floats(view_of(desc)) * sizeof(float), 256);
  lay->total = lay->mse_off + align_up(static_cast<size_t>(4) * desc.H * sizeof(float), 256);
  return SVD_OK;
}
}  // namespace

svd_status svd_search_layer_workspace_bytes(const svd_tensor_desc* desc,
                                            const svd_head_params* const* params_by_mode, size_t* bytes) {
  if (!desc || !params_by_mode || !bytes) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  SearchLayout lay;
  if (svd_status st = search_layout(*desc, params_by_mode, &lay)) return st;
  *bytes = lay.total;
  return SVD_OK;
}

svd_status svd_search_layer(const void* q, const void* k, const void* v, const svd_tensor_desc* desc,
                            const svd_head_params* const* params_by_mode, double lambda, double epsilon,
                            int32_t* table, double* loss, void* out, void* device_workspace,
                            size_t workspace_bytes, void* hip_stream) {
  if (!desc || !params_by_mode || !table) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  if (svd_status st = check_tensors(q, k, v, out)) return st;
  if (desc->H > svd::kMaxSelectHeads) return SVD_ERR_UNSUPPORTED;
  SearchLayout lay;
  if (svd_status st = search_layout(*desc, params_by_mode, &lay)) return st;
  if (!device_workspace || workspace_bytes < lay.total || (reinterpret_cast<uintptr_t>(device_workspace) & 255u))
    return SVD_ERR_WORKSPACE;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(device_workspace);
  const int H = desc->H;
  const svd_tensor_desc cdesc = contiguous_desc(*desc);
  void* o_modes[5];
  for (int m = 0; m < 5; ++m) o_modes[m] = ws + m * lay.out_bytes;

  // The single-mode plans read q, k, v with the caller's strides and write the
  // contiguous buffers: the kernels take one descriptor, so a strided input is
  // only accepted when it is already contiguous.
  if (std::memcmp(&cdesc, desc, sizeof(cdesc)) != 0) return SVD_ERR_UNSUPPORTED;

  std::vector<int32_t> mode_table(H);
  std::vector<svd_head_params> none(H);
  std::vector<double> sparsity(static_cast<size_t>(4) * H);
  float* mse_dev = reinterpret_cast<float*>(ws + lay.mse_off);
  for (int mode = SVD_DENSE; mode <= SVD_VSTRIPE; ++mode) {
    std::fill(mode_table.begin(), mode_table.end(), mode);
    const svd_head_params* pp = (mode >= SVD_DIAG) ? params_by_mode[mode] : none.data();
    if (mode == SVD_DENSE) {
      if (svd_status st = svd_dense_attn_forward(q, k, v, o_modes[0], desc, hip_stream)) return st;
      continue;
    }
    svd_plan* plan = nullptr;
    if (svd_status st = svd_plan_create(&plan, desc, mode_table.data(), pp, nullptr, ws + lay.plan_off,
                                        lay.plan_bytes, hip_stream))
      return st;
    svd_status st = svd_attn_forward_planned(plan, q, k, v, o_modes[mode], hip_stream);
    if (st == SVD_OK) st = svd_plan_head_sparsity(plan, sparsity.data() + static_cast<size_t>(mode - 1) * H);
    if (st == SVD_OK)
      st = svd_head_mse(o_modes[mode], o_modes[0], desc, mse_dev + static_cast<size_t>(mode - 1) * H,
                        ws + lay.mse_scratch_off, lay.mse_off - lay.mse_scratch_off, hip_stream);
    // the next plan reuses the list area: everything of this one must have run
    if (st == SVD_OK && hipStreamSynchronize(stream) != hipSuccess) st = SVD_ERR_HIP;
    svd_plan_destroy(plan);
    if (st != SVD_OK) return st;
  }
  std::vector<float> mse(static_cast<size_t>(4) * H);
  if (hipMemcpyAsync(mse.data(), mse_dev, mse.size() * sizeof(float), hipMemcpyDeviceToHost, stream) != hipSuccess ||
      hipStreamSynchronize(stream) != hipSuccess)
    return SVD_ERR_HIP;
  if (svd_status st = svd_search_select(H, mse.data(), sparsity.data(), lambda, epsilon, table, loss)) return st;
  return svd_select_heads(o_modes, &cdesc, table, out, desc, hip_stream);
}

// ---- token rearrangement (Section 4.1.2) ----

svd_status svd_rearrange_tokens(const void* src, void* dst, const svd_tensor_desc* desc, int32_t first_video_token,
                                int32_t frame_tokens, int32_t frames, int32_t inverse, void* hip_stream) {
  if (!src || !dst || !desc) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  if (!aligned16(src) || !aligned16(dst)) return SVD_ERR_ALIGN;
  if (first_video_token < 0 || frame_tokens < 1 || frames < 1) return SVD_ERR_PARAMS;
  if (static_cast<int64_t>(first_video_token) + static_cast<int64_t>(frame_tokens) * frames > desc->L)
    return SVD_ERR_PARAMS;
  if (src == dst) return SVD_ERR_UNSUPPORTED;   // rows move: not an in-place operation
  if (svd::launch_rearrange_tokens(static_cast<const __bf16*>(src), static_cast<__bf16*>(dst), view_of(*desc),
                                   first_video_token, frame_tokens, frames, inverse != 0,
                                   static_cast<hipStream_t>(hip_stream)) != hipSuccess)
    return SVD_ERR_HIP;
  return SVD_OK;
}

// ---- calibration probes of the benchmark ----

svd_status svd_probe_mfma(void* device_scratch, size_t scratch_bytes, int32_t iters, int32_t work_groups,
                          double* flops, void* hip_stream) {
  if (!device_scratch || !flops) return SVD_ERR_NULL;
  if (iters < 1 || work_groups < 1) return SVD_ERR_SHAPE;
  if (scratch_bytes < static_cast<size_t>(work_groups) * 512 * sizeof(float) ||
      (reinterpret_cast<uintptr_t>(device_scratch) & 3u))
    return SVD_ERR_WORKSPACE;
  return svd::launch_mfma_probe(static_cast<float*>(device_scratch), scratch_bytes / sizeof(float), iters, work_groups,
                                flops, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? SVD_OK
             : SVD_ERR_HIP;
}

svd_status svd_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst) return SVD_ERR_NULL;
  if (bytes == 0 || bytes % 16) return SVD_ERR_SHAPE;
  if (!aligned16(src) || !aligned16(dst)) return SVD_ERR_ALIGN;
  return svd::launch_copy_probe(src, dst, bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? SVD_OK
                                                                                                     : SVD_ERR_HIP;
}

// ---- FP8 variant (Appendix B) ----

svd_status svd_fp8_workspace_bytes(const svd_tensor_desc* desc, size_t* bytes) {
  if (!desc || !bytes) return SVD_ERR_NULL;
  if (svd_status st = svd::validate_desc(desc)) return st;
  *bytes = svd::fp8_scratch_bytes(desc->B, desc->H, desc->L, desc->D);
  return SVD_OK;
}

static svd_status check_fp8_workspace(const svd_tensor_desc& d, const void* ws8, size_t bytes) {
  const size_t need = svd::fp8_scratch_bytes(d.B, d.H, d.L, d.D);
  if (!ws8 || bytes < need || (reinterpret_cast<uintptr_t>(ws8) & 255u)) return SVD_ERR_WORKSPACE;
  return SVD_OK;
}

// Pre-pass plus attention of one group on `stream`.
static svd_status launch_group_fp8(const svd_plan& sp, const svd::Group& g, const void* q, const void* k,
                                   const void* v, void* out, void* ws8, hipStream_t stream) {
  const Plan& p = sp.p;
  const svd_tensor_desc& d = p.desc;
  const int* ws = static_cast<const int*>(p.device_workspace);
  svd::Fp8Launch f{};
  svd::AttnLaunch& a = f.a;
  a = base_launch(d, q, k, v, out);
  a.n_q_blocks = g.n_q_blocks;
  a.n_heads = static_cast<int>(g.heads.size());
  a.n_items = a.n_q_blocks * a.n_heads * a.B;
  a.heads = ws + g.ws_heads;
  a.list_id = ws + g.ws_list_id;
  a.ws = ws;
  a.list_table = static_cast<int>(g.ws_list_table);
  if (g.mode == SVD_SKIP) return svd::launch_zero_heads(a, stream) == hipSuccess ? SVD_OK : SVD_ERR_HIP;
  f.Lp = svd::fp8_padded_len(d.L);
  f.map_len = (d.L + p.block_k - 1) / p.block_k * p.block_k;
  f.k8 = static_cast<uint8_t*>(ws8);
  f.v8t = f.k8 + svd::fp8_scratch_bytes(d.B, d.H, d.L, d.D) / 2;
  const int kmode = g.mode == SVD_DENSE ? svd::MODE_DENSE
                    : g.mode == SVD_VSTRIPE ? svd::MODE_GATHER
                    : g.rearranged ? svd::MODE_PBAND : svd::MODE_BAND;
  // the pre-pass of a group runs right before its attention launch, so the
  // quantised arrays of the group are read back while they are fresh in L2
  if (svd::launch_quantise_kv(f, kmode, stream) != hipSuccess) return SVD_ERR_HIP;
  if (g.mode == SVD_DENSE && sp.dense_split > 1) {
    a.split = sp.dense_split;
    a.n_items *= a.split;
    a.partial = reinterpret_cast<float*>(static_cast<char*>(p.device_workspace) + sp.partial_offset);
  }
  bool small_q = g.block_q != p.block_q;
  if (!small_q && !g.bands_small.empty()) {
    // a band group that the bf16 kernels run on the large query tile: the FP8 kernels take the small-tile lists
    small_q = true;
    a.list_table = static_cast<int>(g.ws_list_table_small);
    a.n_q_blocks = g.n_q_blocks_small;
    a.n_items = a.n_q_blocks * a.n_heads * a.B;
  }
  if (g.mode == SVD_VSTRIPE && p.launchable) {
    // a compacted stripe head is walked like a short dense head: no list depends on the query tile, and
    // the FP8 kernel runs faster with two small work-groups per compute unit (measured 6-9 %)
    small_q = true;
    a.n_q_blocks = (d.L + svd::kernel_small_block_q(d.D) - 1) / svd::kernel_small_block_q(d.D);
    a.n_items = a.n_q_blocks * a.n_heads * a.B;
  }
  if (g.mode == SVD_VSTRIPE)   // the text rows come from the dense launch below
    a.skip_q_blocks = p.text_tokens / (small_q ? svd::kernel_small_block_q(d.D) : p.block_q);
  if (svd::launch_attention_fp8(f, kmode, stream, small_q) != hipSuccess) return SVD_ERR_HIP;
  if (a.split > 1 && svd::launch_combine(a, stream) != hipSuccess) return SVD_ERR_HIP;
  if (has_text_rows(p, g)) {
    // text rows: dense over every key; a stripe head's arrays hold its columns
    // only, so they are quantised once more, uncompacted
    a.split = 1;
    a.skip_q_blocks = 0;
    a.n_q_blocks = g.n_q_blocks;
    a.n_items = a.n_q_blocks * a.n_heads * a.B;
    if (g.mode == SVD_VSTRIPE && svd::launch_quantise_kv(f, svd::MODE_DENSE, stream) != hipSuccess) return SVD_ERR_HIP;
    svd::Fp8Launch t = f;
    t.a = text_rows_launch(sp, g, a);
    if (svd::launch_attention_fp8(t, svd::MODE_DENSE, stream) != hipSuccess) return SVD_ERR_HIP;
    if (t.a.split > 1 && svd::launch_combine(t.a, stream) != hipSuccess) return SVD_ERR_HIP;
  }
  return SVD_OK;
}

svd_status svd_attn_forward_fp8(const svd_plan* plan, const void* q, const void* k, const void* v, void* out,
                                void* fp8_workspace, size_t fp8_workspace_bytes, void* hip_stream) {
  if (svd_status st = check_launchable(plan, q, k, v, out, static_cast<hipStream_t>(hip_stream))) return st;
  if (svd_status st = check_fp8_workspace(plan->p.desc, fp8_workspace, fp8_workspace_bytes)) return st;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // heaviest first, all on the caller's stream
  static const int order[5] = {SVD_DENSE, SVD_DIAG, SVD_MULTIDIAG, SVD_VSTRIPE, SVD_SKIP};
  for (int mode : order)
    for (const svd::Group& g : plan->p.groups)
      if (g.mode == mode)
        if (svd_status st = launch_group_fp8(*plan, g, q, k, v, out, fp8_workspace, stream)) return st;
  return SVD_OK;
}

svd_status svd_attn_forward_fp8_group(const svd_plan* plan, int32_t group, const void* q, const void* k,
                                      const void* v, void* out, void* fp8_workspace, size_t fp8_workspace_bytes,
                                      void* hip_stream) {
  if (svd_status st = check_launchable(plan, q, k, v, out, static_cast<hipStream_t>(hip_stream))) return st;
  if (svd_status st = check_fp8_workspace(plan->p.desc, fp8_workspace, fp8_workspace_bytes)) return st;
  if (group < 0 || group >= static_cast<int32_t>(plan->p.groups.size())) return SVD_ERR_SHAPE;
  return launch_group_fp8(*plan, plan->p.groups[group], q, k, v, out, fp8_workspace,
                          static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
