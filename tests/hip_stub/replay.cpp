// Sanitizer harness: drives the library's host code (plan creation, workspace
// sizing, the bf16 and FP8 launch sequences, fork/join, plan destruction) on a
// host model of the HIP runtime, eagerly and under a modelled stream capture.
//
//   replay LAYERS.txt [SHORTFALL_BYTES]
//
// LAYERS.txt, one layer per block:
//   layer <name> B H L D text_tokens dense_split rounds tensors(0|1) compute_units
//   table m_0 .. m_{H-1}
//   head half_width n_offsets o.. n_cols c.. rearr_first rearr_frame_tokens rearr_frames      (H lines)
// SHORTFALL_BYTES > 0 plants a mistake for the test of the harness itself: the plan
// workspace is allocated that much smaller than the library is told.
// Exit status 0 = no model violation (AddressSanitizer aborts on its own).
#include <cstdio>
#include <cstdlib>
#include <fstream>
#include <iostream>
#include <string>
#include <vector>

#include "hip_stub.h"
#include "sparse_vdit.h"

namespace {

struct Layer {
  std::string name;
  int B = 1, H = 1, L = 1, D = 64, text = 0, split = 0, rounds = 1, tensors = 1, cu = 256;
  std::vector<int32_t> table;
  std::vector<std::vector<int32_t>> offsets, cols;
  std::vector<svd_head_params> params;
};

bool read_layer(std::istream& in, Layer* l) {
  std::string word;
  if (!(in >> word)) return false;
  if (word != "layer") {
    std::fprintf(stderr, "expected 'layer', got '%s'\n", word.c_str());
    std::exit(2);
  }
  in >> l->name >> l->B >> l->H >> l->L >> l->D >> l->text >> l->split >> l->rounds >> l->tensors >> l->cu;
  in >> word;   // table
  l->table.resize(l->H);
  for (int h = 0; h < l->H; ++h) in >> l->table[h];
  l->offsets.assign(l->H, {});
  l->cols.assign(l->H, {});
  l->params.assign(l->H, svd_head_params{});
  for (int h = 0; h < l->H; ++h) {
    int n = 0;
    in >> word >> l->params[h].half_width >> n;
    l->offsets[h].resize(n);
    for (int i = 0; i < n; ++i) in >> l->offsets[h][i];
    in >> n;
    l->cols[h].resize(n);
    for (int i = 0; i < n; ++i) in >> l->cols[h][i];
    in >> l->params[h].rearr_first >> l->params[h].rearr_frame_tokens >> l->params[h].rearr_frames;
  }
  for (int h = 0; h < l->H; ++h) {
    l->params[h].n_offsets = static_cast<int32_t>(l->offsets[h].size());
    l->params[h].offsets = l->offsets[h].empty() ? nullptr : l->offsets[h].data();
    l->params[h].n_cols = static_cast<int32_t>(l->cols[h].size());
    l->params[h].cols = l->cols[h].empty() ? nullptr : l->cols[h].data();
  }
  if (!in) {
    std::fprintf(stderr, "truncated layer '%s'\n", l->name.c_str());
    std::exit(2);
  }
  return true;
}

int g_failures = 0;
size_t g_short = 0;   // bytes by which the plan workspace is allocated too small (the library is told the full size)
void expect(bool ok, const Layer& l, const char* what, int status = 0) {
  if (ok) return;
  std::fprintf(stderr, "layer %s: %s (status %d: %s)\n", l.name.c_str(), what, status,
               svd_status_string(static_cast<svd_status>(status)));
  ++g_failures;
}

void run_layer(const Layer& l) {
  stub::set_compute_units(l.cu);
  stub::set_tensor_checks(l.tensors != 0);
  svd_tensor_desc desc{};
  desc.B = l.B;
  desc.H = l.H;
  desc.L = l.L;
  desc.D = l.D;
  desc.stride_l = l.D;
  desc.stride_h = static_cast<int64_t>(l.L) * l.D;
  desc.stride_b = desc.stride_h * l.H;
  const size_t tensor_bytes = l.tensors ? static_cast<size_t>(l.B) * l.H * l.L * l.D * 2 : 256;
  void* q = stub::device_alloc(tensor_bytes);
  void* k = stub::device_alloc(tensor_bytes);
  void* v = stub::device_alloc(tensor_bytes);
  void* out = stub::device_alloc(tensor_bytes);
  size_t bytes8 = 0;
  expect(svd_fp8_workspace_bytes(&desc, &bytes8) == SVD_OK, l, "svd_fp8_workspace_bytes");
  void* ws8 = stub::device_alloc(l.tensors ? bytes8 : 256);
  svd_plan_options opt{};
  opt.dense_split = l.split;
  opt.text_tokens = l.text;
  for (int round = 0; round < l.rounds; ++round) {
    size_t bytes = 0;
    int st = svd_plan_workspace_bytes(&desc, l.table.data(), l.params.data(), &opt, &bytes);
    expect(st == SVD_OK, l, "svd_plan_workspace_bytes", st);
    if (st != SVD_OK) break;
    void* ws = stub::device_alloc(bytes > g_short ? bytes - g_short : 1);   // g_short > 0: a planted shortfall
    svd_plan* plan = nullptr;
    st = svd_plan_create(&plan, &desc, l.table.data(), l.params.data(), &opt, ws, bytes, nullptr);
    expect(st == SVD_OK, l, "svd_plan_create", st);
    if (st != SVD_OK) {
      stub::device_free(ws);
      break;
    }
    for (int fp8 = 0; fp8 < 2; ++fp8) {
      auto call = [&](hipStream_t s) {
        return fp8 ? (l.tensors ? svd_attn_forward_fp8(plan, q, k, v, out, ws8, bytes8, s) : SVD_OK)
                   : svd_attn_forward_planned(plan, q, k, v, out, s);
      };
      stub::new_forward();
      st = call(nullptr);   // eager, default stream
      expect(st == SVD_OK, l, fp8 ? "eager fp8 forward" : "eager forward", st);
      if (l.tensors && st == SVD_OK)
        expect(stub::out_rows_written() == static_cast<size_t>(l.B) * l.H * l.L, l, "every output row stored exactly once");
      stub::new_forward();
      hipStream_t side = stub::create_stream();
      st = call(side);      // warm-up on the capture stream
      expect(st == SVD_OK, l, "forward on a caller stream", st);
      const long nodes_before = stub::captured_nodes();
      stub::new_forward();
      stub::begin_capture(side);
      st = call(side);
      if (l.text > 0 && (l.tensors || !fp8)) {
        // a layer with a text prefix is refused under capture, before anything is enqueued
        expect(st == SVD_ERR_UNSUPPORTED, l, "forward of a text-prefix layer under capture is refused", st);
        expect(stub::captured_nodes() == nodes_before, l, "a refused forward records nothing");
        expect(stub::end_capture(side) == hipSuccess, l, "capture ends");
      } else {
        expect(st == SVD_OK, l, "forward under capture", st);
        expect(stub::end_capture(side) == hipSuccess, l, "capture ends with everything joined");
        expect(!(l.tensors || !fp8) || stub::captured_nodes() > nodes_before, l, "capture recorded launches");
      }
      stub::destroy_stream(side);
    }
    // the per-group entry points address the same workspace
    int32_t n_groups = 0;
    svd_plan_num_groups(plan, &n_groups);
    stub::new_forward();
    for (int32_t g = 0; g < n_groups; ++g) {
      st = svd_attn_forward_group(plan, g, q, k, v, out, nullptr);
      expect(st == SVD_OK, l, "svd_attn_forward_group", st);
    }
    expect(svd_plan_destroy(plan) == SVD_OK, l, "svd_plan_destroy");
    stub::device_free(ws);
  }
  {
    // the same layer as ONE launch (and with the dense head start): eagerly, and under capture (refused with a text prefix)
    for (int form : {1, 3}) {
    svd_plan_options one = opt;
    one.single_launch = form;
    size_t bytes = 0;
    int st = svd_plan_workspace_bytes(&desc, l.table.data(), l.params.data(), &one, &bytes);
    expect(st == SVD_OK, l, "svd_plan_workspace_bytes (single launch)", st);
    void* ws = stub::device_alloc(bytes > g_short ? bytes - g_short : 1);
    svd_plan* plan = nullptr;
    st = svd_plan_create(&plan, &desc, l.table.data(), l.params.data(), &one, ws, bytes, nullptr);
    expect(st == SVD_OK, l, "svd_plan_create (single launch)", st);
    if (st == SVD_OK) {
      int32_t is_single = 0;
      svd_plan_single_launch(plan, &is_single);
      expect(is_single == form, l, "the plan reports its launch form");
      const long before = stub::launches();
      stub::new_forward();
      st = svd_attn_forward_planned(plan, q, k, v, out, nullptr);
      expect(st == SVD_OK, l, "single-launch forward", st);
      if (l.tensors && st == SVD_OK)
        expect(stub::out_rows_written() == static_cast<size_t>(l.B) * l.H * l.L, l, "every output row stored exactly once (layer kernel)");
      stub::new_forward();
      bool stripes = false;
      for (int32_t m : l.table) stripes = stripes || m == SVD_VSTRIPE;
      const long helpers = 1 + (stripes ? 1 : 0);   // the fill of the queue positions, the gather pre-pass of stripe heads
      expect(form == 1 ? stub::launches() == before + 1 + helpers : stub::launches() <= before + 2 + helpers, l,
             "a single-launch forward is the layer kernel plus its helpers (plus the dense head start in that form)");
      hipStream_t side = stub::create_stream();
      stub::begin_capture(side);
      st = svd_attn_forward_planned(plan, q, k, v, out, side);
      expect(l.text > 0 ? st == SVD_ERR_UNSUPPORTED : st == SVD_OK, l, "single-launch forward under capture", st);
      expect(stub::end_capture(side) == hipSuccess, l, "capture ends");
      stub::destroy_stream(side);
      stub::new_forward();
      if (l.tensors) {
        st = svd_attn_forward_fp8(plan, q, k, v, out, ws8, bytes8, nullptr);   // the FP8 path runs such a plan group by group
        expect(st == SVD_OK, l, "fp8 forward with a single-launch plan", st);
      }
      expect(svd_plan_destroy(plan) == SVD_OK, l, "svd_plan_destroy");
    }
    stub::device_free(ws);
    }
  }
  {
    // what the library chooses when the caller leaves the launch form to it
    svd_plan_options own = opt;
    own.dense_split = 0;
    size_t bytes = 0;
    int st = svd_plan_workspace_bytes(&desc, l.table.data(), l.params.data(), &own, &bytes);
    void* ws = stub::device_alloc(bytes ? bytes : 1);
    svd_plan* plan = nullptr;
    if (st == SVD_OK) st = svd_plan_create(&plan, &desc, l.table.data(), l.params.data(), &own, ws, bytes, nullptr);
    expect(st == SVD_OK, l, "plan with the library's choice of the launch form", st);
    if (st == SVD_OK) {
      int32_t form = -1;
      svd_plan_single_launch(plan, &form);
      std::printf("layer %s: the library's launch form is %d\n", l.name.c_str(), form);
      stub::new_forward();
      st = svd_attn_forward_planned(plan, q, k, v, out, nullptr);
      expect(st == SVD_OK, l, "forward with the library's choice of the launch form", st);
      if (l.tensors && st == SVD_OK)
        expect(stub::out_rows_written() == static_cast<size_t>(l.B) * l.H * l.L, l, "every output row stored exactly once (library's choice)");
      svd_plan_destroy(plan);
    }
    stub::device_free(ws);
  }
  if (l.text == 0) {
    // the entry point that allocates nothing: a miss (copy of the lists into the library's buffer),
    // a hit, and a hit under capture; a miss under capture is refused
    stub::new_forward();
    int st = sparse_vdit_attn_forward_static(q, k, v, l.table.data(), l.params.data(), out, &desc, nullptr);
    expect(st == SVD_OK || st == SVD_ERR_STATIC_LIMIT, l, "static one-shot forward", st);
    if (st == SVD_OK) {
      stub::new_forward();
      st = sparse_vdit_attn_forward_static(q, k, v, l.table.data(), l.params.data(), out, &desc, nullptr);
      expect(st == SVD_OK, l, "static one-shot forward, cached plan", st);
      hipStream_t side = stub::create_stream();
      stub::new_forward();
      stub::begin_capture(side);
      st = sparse_vdit_attn_forward_static(q, k, v, l.table.data(), l.params.data(), out, &desc, side);
      expect(st == SVD_OK, l, "static one-shot forward under capture, cached plan", st);
      expect(stub::end_capture(side) == hipSuccess, l, "capture ends");
      if (l.H > 1) {   // another table: a miss, which a capturing stream cannot take
        std::vector<int32_t> other(l.table);
        std::vector<svd_head_params> pp(l.params);
        other[0] = other[0] == SVD_SKIP ? SVD_DENSE : SVD_SKIP;
        stub::begin_capture(side);
        st = sparse_vdit_attn_forward_static(q, k, v, other.data(), pp.data(), out, &desc, side);
        expect(st == SVD_ERR_UNSUPPORTED, l, "static one-shot forward under capture with a new table is refused", st);
        expect(stub::end_capture(side) == hipSuccess, l, "capture ends");
        stub::new_forward();
        st = sparse_vdit_attn_forward_static(q, k, v, other.data(), pp.data(), out, &desc, side);
        expect(st == SVD_OK, l, "static one-shot forward with a new table on another stream", st);
      }
      stub::destroy_stream(side);
    }
  }
  for (void* p : {q, k, v, out, ws8}) stub::device_free(p);
}

}  // namespace

int main(int argc, char** argv) {
  if (argc != 2 && argc != 3) {
    std::fprintf(stderr, "usage: replay LAYERS.txt [SHORTFALL_BYTES]\n");
    return 2;
  }
  if (argc == 3) g_short = static_cast<size_t>(std::atol(argv[2]));
  std::ifstream in(argv[1]);
  if (!in) {
    std::fprintf(stderr, "cannot read %s\n", argv[1]);
    return 2;
  }
  Layer l;
  int n = 0;
  while (read_layer(in, &l)) {
    run_layer(l);
    ++n;
    std::printf("layer %s: %ld launches so far, %ld captured, %d violations, %d failures\n", l.name.c_str(),
                stub::launches(), stub::captured_nodes(), stub::violations(), g_failures);
    std::fflush(stdout);
  }
  std::printf("%d layers replayed\n", n);
  return (stub::violations() || g_failures) ? 1 : 0;
}
