// Host models of the kernel launches behind attn_kernels.h, fp8_kernels.h,
// search_kernels.h and rearrange_kernels.h.  No attention arithmetic here: for
// every work-group a launch would start, the model walks the index arithmetic of
// the kernel (item -> query tile, chunk, head; list records, row pointers,
// entries, runs, columns, row map; partial-result rows) and touches, on the
// host, every word of the plan workspace and every row of q, k, v, out, the
// partial-result scratch and the FP8 arrays that the kernel would address.  All
// of that memory is exact-size heap memory of the test, so an index that leaves
// its buffer is an AddressSanitizer report (and a model violation).
#include <cstdint>
#include <cstring>

#include "attn_kernels.h"
#include "fp8_kernels.h"
#include "hip_stub.h"
#include "probe_kernels.h"
#include "rearrange_kernels.h"
#include "search_kernels.h"
#include "static_scratch.h"

namespace svd {
namespace {

volatile uint64_t g_sink;   // keeps the reads alive

// tensor = true: part of q, k, v, out or the FP8 arrays (skipped when the test could not allocate them)
void touch_read(const void* p, size_t bytes, const char* what, bool tensor = false) {
  if (tensor && !stub::tensor_checks()) return;
  if (!stub::in_device(p, bytes)) {
    stub::violation("%s: read of %zu bytes outside every device allocation", what, bytes);
    return;
  }
  const unsigned char* c = static_cast<const unsigned char*>(p);
  uint64_t s = 0;
  for (size_t i = 0; i < bytes; i += 64) s += c[i];
  if (bytes) s += c[bytes - 1];
  g_sink = g_sink + s;
}
void touch_write(void* p, size_t bytes, const char* what, unsigned char value, bool tensor = false) {
  if (tensor && !stub::tensor_checks()) return;
  if (what[0] == 'o' && what[1] == 'u' && what[2] == 't') stub::note_out_row(p);   // "out row ..."
  if (!stub::in_device(p, bytes)) {
    stub::violation("%s: write of %zu bytes outside every device allocation", what, bytes);
    return;
  }
  std::memset(p, value, bytes);
}
int read_word(const int* p, const char* what) {
  if (!stub::in_device(p, 4)) {
    stub::violation("%s: workspace word outside every device allocation", what);
    return 0;
  }
  return *p;
}

struct Shape { int NW, BC; };
Shape shape_of(int D, bool small_q) {
  if (D == 128) return small_q ? Shape{Tile128s::NW, Tile128s::BC} : Shape{Tile128::NW, Tile128::BC};
  return small_q ? Shape{Tile64s::NW, Tile64s::BC} : Shape{Tile64::NW, Tile64::BC};
}

const __bf16* row_of(const __bf16* t, const AttnLaunch& p, int b, int head, int row) {
  return t + (int64_t)b * p.stride_b + (int64_t)head * p.stride_h + (int64_t)row * p.stride_l;
}

// One work-group of attn_fwd_kernel / attn_fwd_fp8_kernel.  fp8: K and V come from the quantised arrays.
void model_item(const AttnLaunch& p, const Fp8Launch* f8, int mode, bool small_q, int item) {
  const Shape sh = shape_of(p.D, small_q);
  const int BR = sh.NW * 32, BC = sh.BC, DB = p.D / 32;
  const int qblk = item % p.n_q_blocks;
  const int chunk = (item / p.n_q_blocks) % p.split;
  const int hb = item / p.n_q_blocks / p.split;
  const int hg = hb % p.n_heads, b = hb / p.n_heads;
  if (b >= p.B) {
    stub::violation("item %d decodes to batch entry %d of %d", item, b, p.B);
    return;
  }
  const int head = p.heads ? read_word(p.heads + hg, "heads") : hg;
  if (head < 0 || head >= p.H) {
    stub::violation("head id %d outside [0, %d)", head, p.H);
    return;
  }
  const int L = p.L;
  const bool band = mode == MODE_BAND || mode == MODE_PBAND;
  const int* map = nullptr;    // PBAND row map, GATHER column list
  int n_tiles = 0, t_base = 0, e0 = 0;
  const int* entries = nullptr;
  const int* runs = nullptr;
  if (mode == MODE_DENSE) {
    const int n_all = (L + BC - 1) / BC;
    t_base = chunk * n_all / p.split;
    n_tiles = (chunk + 1) * n_all / p.split - t_base;
    if (n_tiles < 1) stub::violation("dense chunk %d of %d holds no key tile", chunk, p.split);
  } else {
    const int* rec = p.ws + p.list_table + 4 * read_word(p.list_id + hg, "list_id");
    touch_read(rec, 16, "list record");
    if (band) {
      const int* row_ptr = p.ws + rec[0];
      e0 = read_word(row_ptr + qblk, "row_ptr");
      const int e1 = read_word(row_ptr + qblk + 1, "row_ptr");
      entries = p.ws + rec[1] + 2 * (int64_t)e0;
      runs = p.ws + rec[2];
      n_tiles = e1 - e0;
      if (n_tiles < 0) stub::violation("row_ptr descends");
      if (n_tiles <= 0) return;
      if (mode == MODE_PBAND) map = p.ws + rec[3];
    } else {
      if (qblk < p.skip_q_blocks) return;
      n_tiles = rec[1] / BC;
      if (rec[1] % BC) stub::violation("column list not padded to the key tile");
      if (!f8 && (!p.gathered || rec[1] > p.gather_pad)) stub::violation("gathered arrays missing or shorter than a padded list");
    }
  }
  // query rows (clamped to L - 1 on load, stored only below L)
  for (int r = 0; r < BR && (stub::tensor_checks() || mode == MODE_PBAND); ++r) {
    int row = qblk * BR + r;
    const bool store = row < L && !(mode == MODE_DENSE && p.split > 1);
    row = row < L ? row : L - 1;
    if (mode == MODE_PBAND) row = read_word(map + row, "row map (query)");
    if (row < 0 || row >= L) {
      stub::violation("query row %d outside [0, %d)", row, L);
      continue;
    }
    touch_read(row_of(p.q, p, b, head, row), (size_t)p.D * 2, "q row", true);
    if (store) touch_write(const_cast<__bf16*>(row_of(p.out, p, b, head, row)), (size_t)p.D * 2, "out row", 0x11, true);
  }
  // key tiles
  const size_t base8 = f8 ? ((size_t)b * p.H + head) * (size_t)f8->Lp * p.D : 0;
  for (int t = 0; t < n_tiles; ++t) {
    int tile = t + t_base;
    if (band) {
      touch_read(entries + 2 * t, 8, "band entry");
      tile = entries[2 * t];
      const int meta = entries[2 * t + 1];
      const int r0 = (meta >> 1) & 0x7fff, rn = meta >> 16;
      if (!(meta & 1))
        for (int r = r0; r < r0 + rn; ++r) touch_read(runs + 2 * r, 8, "run");
      if (tile < 0 || tile * BC >= L) stub::violation("band entry names key tile %d past the sequence", tile);
    }
    if (f8 && mode != MODE_PBAND) {
      // quantised arrays: rows tile*BC .. +BC of the head (compacted for GATHER)
      if ((tile + 1) * BC > f8->Lp) {
        stub::violation("fp8 key tile %d reaches past Lp", tile);
        continue;
      }
      touch_read(f8->k8 + base8 + (size_t)tile * BC * p.D, (size_t)BC * p.D, "k8 tile", true);
      touch_read(f8->v8t + base8 + (size_t)tile * BC * p.D, (size_t)BC * p.D, "v8t tile", true);
      continue;
    }
    if (f8) {   // PBAND in FP8: the arrays are in rearranged order
      touch_read(f8->k8 + base8 + (size_t)tile * BC * p.D, (size_t)BC * p.D, "k8 tile", true);
      touch_read(f8->v8t + base8 + (size_t)tile * BC * p.D, (size_t)BC * p.D, "v8t tile", true);
      continue;
    }
    if (!stub::tensor_checks() && mode != MODE_GATHER && mode != MODE_PBAND) continue;   // no workspace word involved
    if (mode == MODE_GATHER && !f8) {   // the group's gathered rows: a short dense head
      const __bf16* Kg = p.gathered + (size_t)hb * 2 * p.gather_pad * p.D;
      touch_read(Kg + (size_t)tile * BC * p.D, (size_t)BC * p.D * 2, "gathered K tile");
      touch_read(Kg + (size_t)p.gather_pad * p.D + (size_t)tile * BC * p.D, (size_t)BC * p.D * 2, "gathered V tile");
      continue;
    }
    for (int r = 0; r < BC; ++r) {
      int row = tile * BC + r;
      if (mode == MODE_GATHER || mode == MODE_PBAND) {
        row = read_word(map + row, "column list / row map");
        row = row < 0 ? 0 : row;
      } else {
        row = row < L ? row : L - 1;
      }
      if (row >= L) {
        stub::violation("key row %d outside [0, %d)", row, L);
        continue;
      }
      touch_read(row_of(p.k, p, b, head, row), (size_t)p.D * 2, "k row", true);
      touch_read(row_of(p.v, p, b, head, row), (size_t)p.D * 2, "v row", true);
    }
  }
  if (mode == MODE_DENSE && p.split > 1) {
    float* dst = p.partial + (size_t)item * sh.NW * ((DB * 16 + 2) * 64);
    touch_write(dst, (size_t)sh.NW * (DB * 16 + 2) * 64 * sizeof(float), "partial results", 0x22);
  }
}

hipError_t model_attention(const AttnLaunch& p, const Fp8Launch* f8, int mode, hipStream_t stream, bool small_q) {
  if (p.n_items <= 0) return hipSuccess;
  if (p.split < 1 || (p.split > 1 && (mode != MODE_DENSE || !p.partial))) return hipErrorInvalidValue;
  if (p.D != 64 && p.D != 128) return hipErrorInvalidValue;
  if (small_q && !f8 && mode != MODE_BAND && mode != MODE_PBAND) return hipErrorInvalidValue;
  if (small_q && f8 && mode == MODE_DENSE) return hipErrorInvalidValue;
  const int space = p.n_q_blocks * p.n_heads * p.B * p.split;
  if (p.n_items != space && !(mode == MODE_DENSE && p.split == 1 && p.n_items > 0 && p.n_items < space))   // the dense head start
    stub::violation("n_items does not match the item space");
  stub::note_launch(stream, f8 ? "attn_fwd_fp8_kernel" : "attn_fwd_kernel");
  for (int item = 0; item < p.n_items; ++item) model_item(p, f8, mode, small_q, item);
  return hipSuccess;
}

}  // namespace

int kernel_small_block_q(int D) {
  return D == 128 ? Tile128s::NW * Tile128s::QB * 32 : Tile64s::NW * Tile64s::QB * 32;
}

void kernel_blocks(int D, int* block_q, int* block_k) {
  if (D == 128) {
    *block_q = Tile128::NW * Tile128::QB * 32;
    *block_k = Tile128::BC;
  } else {
    *block_q = Tile64::NW * Tile64::QB * 32;
    *block_k = Tile64::BC;
  }
}

size_t partial_floats(int D, int n_items) {
  const int nw = D == 128 ? Tile128::NW : Tile64::NW;
  return (size_t)n_items * nw * ((D / 32 * 16 + 2) * 64);
}

hipError_t launch_attention(const AttnLaunch& p, int mode, hipStream_t stream, bool small_q) {
  return model_attention(p, nullptr, mode, stream, small_q);
}

int layer_block_q(int D) {
  int bq = 0, bk = 0;
  kernel_blocks(D, &bq, &bk);
  return bq;   // the layer kernel runs the kernels' own (large) query tile
}

// The single-launch path: every item of every segment, on the small query tile; the queue positions.
hipError_t launch_layer(const LayerLaunch& p, int n_compute_units, hipStream_t stream) {
  if (p.n_segments < 1) return hipSuccess;
  if (p.n_segments > kMaxSegments || !p.counters || n_compute_units < 1) return hipErrorInvalidValue;
  stub::note_launch(stream, "reset_counters_kernel");
  touch_write(p.counters, kLayerCounterWords * sizeof(int), "queue positions", 0x00);
  stub::note_launch(stream, "attn_layer_kernel");
  const int BR = layer_block_q(p.a.D);
  for (int s = 0; s < p.n_segments; ++s) {
    const LayerSegment& sg = p.seg[s];
    if (sg.kind < SEG_DENSE || sg.kind > SEG_ZERO || sg.n_items < 0) return hipErrorInvalidValue;
    if (s > 0 && sg.kind == SEG_DENSE && p.seg[s - 1].kind != SEG_DENSE)
      stub::violation("segments are not heaviest first: a dense segment follows a lighter one");
    AttnLaunch a = p.a;
    a.n_q_blocks = sg.n_q_blocks;
    a.n_heads = sg.n_heads;
    a.n_items = sg.n_items + sg.first_item;
    a.heads = p.a.ws + sg.heads;
    a.list_id = p.a.ws + sg.list_id;
    a.list_table = sg.list_table;
    a.split = 1;
    a.partial = nullptr;
    if (sg.first_item < 0 || sg.n_items + sg.first_item != sg.n_q_blocks * sg.n_heads * a.B)
      stub::violation("segment %d: first_item + n_items does not match its item space", s);
    if (sg.first_item > 0 && sg.kind != SEG_DENSE) stub::violation("segment %d: only dense segments have a head start", s);
    for (int item = sg.first_item; item < sg.first_item + sg.n_items; ++item) {
      if (sg.kind != SEG_ZERO) {
        const int mode = sg.kind == SEG_DENSE ? MODE_DENSE : sg.kind == SEG_BAND ? MODE_BAND
                         : sg.kind == SEG_GATHER ? MODE_GATHER : MODE_PBAND;
        model_item(a, nullptr, mode, false, item);
        continue;
      }
      const int qblk = item % a.n_q_blocks, hb = item / a.n_q_blocks;
      const int hg = hb % a.n_heads, b = hb / a.n_heads;
      const int head = read_word(a.heads + hg, "heads");
      if (head < 0 || head >= a.H || b >= a.B) {
        stub::violation("zero item %d decodes to head %d, batch entry %d", item, head, b);
        continue;
      }
      for (int r = 0; r < BR; ++r)
        if (qblk * BR + r < a.L)
          touch_write(const_cast<__bf16*>(row_of(a.out, a, b, head, qblk * BR + r)), (size_t)a.D * 2, "out row (zero item)", 0x00, true);
    }
  }
  return hipSuccess;
}

hipError_t launch_gather_kv(const AttnLaunch& p, hipStream_t stream) {
  if (p.n_heads <= 0) return hipSuccess;
  if (!p.gathered || p.gather_pad < 1 || !p.heads || !p.list_id || !p.ws) return hipErrorInvalidValue;
  stub::note_launch(stream, "gather_kv_kernel");
  for (int hb = 0; hb < p.n_heads * p.B; ++hb) {
    const int hg = hb % p.n_heads, b = hb / p.n_heads;
    const int head = read_word(p.heads + hg, "heads");
    if (head < 0 || head >= p.H) {
      stub::violation("gather: head %d", head);
      continue;
    }
    const int* rec = p.ws + p.list_table + 4 * read_word(p.list_id + hg, "list_id");
    touch_read(rec, 16, "list record");
    const int* cols = p.ws + rec[0];
    for (int j = 0; j < rec[1] && j < p.gather_pad; ++j) {
      const int src = read_word(cols + j, "column list (gather)");
      if (src >= p.L) stub::violation("gather: source row %d outside [0, %d)", src, p.L);
      if (src >= 0 && src < p.L) {
        touch_read(row_of(p.k, p, b, head, src), (size_t)p.D * 2, "k row (gather)", true);
        touch_read(row_of(p.v, p, b, head, src), (size_t)p.D * 2, "v row (gather)", true);
      }
    }
    touch_write(p.gathered + (size_t)hb * 2 * p.gather_pad * p.D, (size_t)2 * p.gather_pad * p.D * 2, "gathered rows", 0x00);
  }
  return hipSuccess;
}

hipError_t launch_combine(const AttnLaunch& p, hipStream_t stream) {
  if (p.split <= 1 || p.n_items <= 0) return hipSuccess;
  if (!p.partial) return hipErrorInvalidValue;
  stub::note_launch(stream, "combine_partials_kernel");
  const Shape sh = shape_of(p.D, false);
  const int DB = p.D / 32, BR = sh.NW * 32;
  const int tiles = p.n_items / p.split;
  for (int blk = 0; blk < tiles; ++blk) {
    const int qblk = blk % p.n_q_blocks, hb = blk / p.n_q_blocks;
    const int hg = hb % p.n_heads, b = hb / p.n_heads;
    const int head = p.heads ? read_word(p.heads + hg, "heads") : hg;
    if (head < 0 || head >= p.H || b >= p.B) {
      stub::violation("merge block %d decodes to head %d, batch entry %d", blk, head, b);
      continue;
    }
    for (int c = 0; c < p.split; ++c) {
      const size_t item = ((size_t)hb * p.split + c) * p.n_q_blocks + qblk;
      touch_read(p.partial + item * sh.NW * ((DB * 16 + 2) * 64), (size_t)sh.NW * (DB * 16 + 2) * 64 * sizeof(float),
                 "partial results (merge)");
    }
    for (int r = 0; r < BR; ++r) {
      const int row = qblk * BR + r;
      if (row < p.L) touch_write(const_cast<__bf16*>(row_of(p.out, p, b, head, row)), (size_t)p.D * 2, "out row (merge)", 0x33, true);
    }
  }
  return hipSuccess;
}

hipError_t launch_zero_heads(const AttnLaunch& p, hipStream_t stream) {
  if (p.n_heads <= 0) return hipSuccess;
  stub::note_launch(stream, "zero_heads_kernel");
  for (int hb = 0; hb < p.n_heads * p.B; ++hb) {
    const int hg = hb % p.n_heads, b = hb / p.n_heads;
    const int head = p.heads ? read_word(p.heads + hg, "heads") : hg;
    if (head < 0 || head >= p.H) {
      stub::violation("zero fill of head %d", head);
      continue;
    }
    for (int row = 0; row < p.L; ++row)
      touch_write(const_cast<__bf16*>(row_of(p.out, p, b, head, row)), (size_t)p.D * 2, "out row (zero fill)", 0x00, true);
  }
  return hipSuccess;
}

hipError_t launch_quantise_kv(const Fp8Launch& p, int mode, hipStream_t stream) {
  if (p.a.n_heads <= 0) return hipSuccess;
  if (!p.k8 || !p.v8t || p.Lp != fp8_padded_len(p.a.L)) return hipErrorInvalidValue;
  const int gather = mode == MODE_GATHER ? 1 : mode == MODE_PBAND ? 2 : 0;
  if (gather == 2 && (p.map_len < 1 || p.map_len > p.Lp)) return hipErrorInvalidValue;
  stub::note_launch(stream, "quantise_kv_kernel");
  const AttnLaunch& a = p.a;
  for (int hb = 0; hb < a.n_heads * a.B; ++hb) {
    const int hg = hb % a.n_heads, b = hb / a.n_heads;
    const int head = a.heads ? read_word(a.heads + hg, "heads") : hg;
    if (head < 0 || head >= a.H) {
      stub::violation("quantise: head %d", head);
      continue;
    }
    const int* cols = nullptr;
    int n_pad = p.Lp;
    if (gather) {
      const int* rec = a.ws + a.list_table + 4 * read_word(a.list_id + hg, "list_id");
      touch_read(rec, 16, "list record");
      cols = a.ws + (gather == 1 ? rec[0] : rec[3]);
      n_pad = gather == 1 ? rec[1] : p.map_len;
    }
    const size_t base8 = ((size_t)b * a.H + head) * (size_t)p.Lp * a.D;
    for (int G = 0; G * 64 < n_pad && G < p.Lp / 64; ++G) {
      for (int r = 0; r < 64; ++r) {
        const int key = G * 64 + r;
        const int src = cols ? read_word(cols + key, "column list / row map (quantise)") : (key < a.L ? key : -1);
        if (src >= a.L) stub::violation("quantise: source row %d outside [0, %d)", src, a.L);
        if (src >= 0 && src < a.L) {
          touch_read(row_of(a.k, a, b, head, src), (size_t)a.D * 2, "k row (quantise)", true);
          touch_read(row_of(a.v, a, b, head, src), (size_t)a.D * 2, "v row (quantise)", true);
        }
      }
      touch_write(p.k8 + base8 + (size_t)G * 64 * a.D, (size_t)64 * a.D, "k8 group", 0x44, true);
      touch_write(p.v8t + base8 + (size_t)G * 64 * a.D, (size_t)64 * a.D, "v8t group", 0x55, true);
    }
  }
  return hipSuccess;
}

hipError_t launch_attention_fp8(const Fp8Launch& p, int mode, hipStream_t stream, bool small_q) {
  if (p.a.n_items <= 0) return hipSuccess;
  if (!p.k8 || !p.v8t || p.Lp != fp8_padded_len(p.a.L)) return hipErrorInvalidValue;
  return model_attention(p.a, &p, mode, stream, small_q);
}

// The library's static buffer: here one exact-size "device" allocation for the one modelled device.
hipError_t static_scratch(void** ptr, size_t* bytes) {
  static void* buffer = stub::device_alloc(kStaticScratchBytes);
  *ptr = buffer;
  *bytes = kStaticScratchBytes;
  return hipSuccess;
}

// ---- search step and rearrangement: streaming kernels, ranges only ----

int mse_chunks(const TensorView& t) {
  const int64_t bytes = (int64_t)t.L * t.D * 2;
  const int64_t n = (bytes + (1 << 18) - 1) / (1 << 18);
  return (int)(n < 1 ? 1 : n);
}
size_t mse_scratch_floats(const TensorView& t) { return (size_t)t.B * t.H * mse_chunks(t); }

hipError_t launch_head_mse(const __bf16*, const __bf16*, const TensorView& t, float* mse, float* scratch, hipStream_t stream) {
  stub::note_launch(stream, "head_mse_partial_kernel");
  touch_write(scratch, mse_scratch_floats(t) * sizeof(float), "mse partial sums", 0x66);
  stub::note_launch(stream, "head_mse_final_kernel");
  touch_write(mse, (size_t)t.H * sizeof(float), "mse", 0x00);
  return hipSuccess;
}

hipError_t launch_select_heads(const __bf16* const*, const TensorView& sv, const int32_t*, __bf16*, const TensorView&,
                               hipStream_t stream) {
  if (sv.H > kMaxSelectHeads) return hipErrorInvalidValue;
  stub::note_launch(stream, "select_heads_kernel");
  return hipSuccess;
}

hipError_t launch_mfma_probe(float* out, size_t out_floats, int iters, int work_groups, double* flops, hipStream_t stream) {
  if (!out || iters < 1 || work_groups < 1 || out_floats < (size_t)work_groups * 512) return hipErrorInvalidValue;
  stub::note_launch(stream, "mfma_probe_kernel");
  touch_write(out, (size_t)work_groups * 512 * sizeof(float), "probe output", 0x77);
  if (flops) *flops = 2.0 * 32 * 32 * 16 * 8 * (double)iters * 8.0 * work_groups;
  return hipSuccess;
}

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream) {
  stub::note_launch(stream, "copy_probe_kernel");
  touch_read(src, bytes, "copy source");
  touch_write(dst, bytes, "copy destination", 0x78);
  return hipSuccess;
}

hipError_t launch_rearrange_tokens(const __bf16*, __bf16*, const TensorView&, int, int, int, bool, hipStream_t stream) {
  stub::note_launch(stream, "rearrange_tokens_kernel");
  return hipSuccess;
}

}  // namespace svd
