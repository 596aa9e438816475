// gfx950 (MI355X, CDNA4) kernels of the FP8 variant of the sparse attention
// forward (Appendix B: the sparse kernels of Section 4.2 with FP8 quantisation).
//
// The paper names neither format nor recipe; this build quantises Q, K, V and P
// to OCP E4M3 with fixed power-of-two scales:
//   Q8 = e4m3(q * 4 log2(e) / sqrt(D)),  K8 = e4m3(k / 4),  V8 = e4m3(v),
//   P8 = e4m3(2^(Q8.K8 - m)) with the integer reference m = ceil(row max) - 8,
// and accumulates scores, row sums and the output in fp32.
//
// Two kernels:
//   quantise_kv_kernel   pre-pass of a group of heads: K8 row-major, V8 transposed
//                        in groups of 64 keys with the keys of a group in the
//                        order in which a lane's score accumulators hold them.
//                        A vertical-stripe head (M_4) is compacted here: its
//                        arrays hold the listed key columns only.
//   attn_fwd_fp8_kernel  the loop of the bf16 kernel (transposed scores, lane
//                        owns a query column, one tile of look-ahead between the
//                        two products, lazy reference) on the FP8 matrix
//                        instructions v_mfma_f32_32x32x64_f8f6f4 (both products)
//                        and v_mfma_f32_16x16x128_f8f6f4 (row sums of P).  Modes:
//                        DENSE, BAND, GATHER = the dense loop over a compacted
//                        head, and PBAND = the banded loop of a multi-diagonal
//                        head in rearranged form (Section 4.1.2): the pre-pass
//                        writes K8 and V8 in the rearranged order, Q rows and O
//                        rows go through the list's row map.
// Operand layout of the 32x32x64 instruction: lane l supplies row (column) l % 32
// with the 32 contraction indices 32 * (l / 32) .. + 31 in its 32 bytes; the
// result has the layout of the 32x32 bf16 instructions, so masks, maxima and the
// epilogue are those of the bf16 kernel.  The reference moves in integer steps:
// every rescale is an exact power of two and the rounding of P does not depend
// on the order of the key tiles (outside the subnormal range).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "fp8_kernels.h"

namespace svd {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));

constexpr float kNegInf = -__builtin_inff();
constexpr float kE4M3Max = 448.0f;

// Four floats to four E4M3 bytes, first argument in the lowest byte (round to
// nearest even; the caller keeps the values inside +-448).
__device__ __forceinline__ int pack_e4m3(float a, float b, float c, float d) {
  // the first conversion overwrites the low half of its destination and the second
  // the high half: starting from the bits of `a` (dead afterwards) saves a move
  int w = __builtin_bit_cast(int, a);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, w, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
  return w;
}
__device__ __forceinline__ float sat_e4m3(float x) { return fminf(fmaxf(x, -kE4M3Max), kE4M3Max); }

__device__ __forceinline__ float half_max(float x) {
  const unsigned a = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
  const unsigned r0 = r[0], r1 = r[1];
  return fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
}

// 16-byte chunk swizzle of the K8 tile (row = key, D bytes): a fragment read
// takes 16 bytes per lane with consecutive lanes on consecutive keys.
template <int D>
__device__ __forceinline__ int swz_k8(int row) {
  return D == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

template <int N>
using Int = std::integral_constant<int, N>;

// ---------------------------------------------------------------------------
// Pre-pass.  Work-group = one group of 64 keys of one head.
// ---------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(256) quantise_kv_kernel(const Fp8Launch pp, const int gather) {
  const AttnLaunch& p = pp.a;
  constexpr int SV_STRIDE = D + 8;   // bf16 elements; keeps rows 16-byte aligned
  __shared__ __attribute__((aligned(16))) __bf16 sv[64 * SV_STRIDE];
  const int G = blockIdx.x;
  const int hg = blockIdx.y % p.n_heads;
  const int b = blockIdx.y / p.n_heads;
  const int head = p.heads ? p.heads[hg] : hg;
  const int* cols = nullptr;
  int n_pad = pp.Lp;
  if (gather == 1) {          // vertical-stripe head: its column list
    const int* rec = p.ws + p.list_table + 4 * p.list_id[hg];
    cols = p.ws + rec[0];
    n_pad = rec[1];
  } else if (gather == 2) {   // rearranged head: key j of the arrays is row row_map[j] of the tensors
    const int* rec = p.ws + p.list_table + 4 * p.list_id[hg];
    cols = p.ws + rec[3];
    n_pad = pp.map_len;
  }
  if (G * 64 >= n_pad) return;
  const int64_t base = (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  const __bf16* __restrict__ K = p.k + base;
  const __bf16* __restrict__ V = p.v + base;
  const size_t base8 = ((size_t)b * p.H + head) * (size_t)pp.Lp * D;
  uint8_t* __restrict__ K8 = pp.k8 + base8;
  uint8_t* __restrict__ V8 = pp.v8t + base8;
  const int tid = threadIdx.x;

  auto source_row = [&](int key) -> int {   // -1: no such key (zeros)
    if (cols) return cols[key];
    return key < p.L ? key : -1;
  };

  // K8: 16 elements per step
  constexpr int KCH = D / 16;
  for (int c = tid; c < 64 * KCH; c += 256) {
    const int row = c / KCH, pc = c % KCH;
    const int src = source_row(G * 64 + row);
    i32x4 outw = {0, 0, 0, 0};
    if (src >= 0) {
      const __bf16* s = K + (int64_t)src * p.stride_l + pc * 16;
      const f32x8 lo = __builtin_convertvector(*reinterpret_cast<const bf16x8*>(s), f32x8);
      const f32x8 hi = __builtin_convertvector(*reinterpret_cast<const bf16x8*>(s + 8), f32x8);
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        outw[w] = pack_e4m3(sat_e4m3(lo[4 * w] * 0.25f), sat_e4m3(lo[4 * w + 1] * 0.25f),
                            sat_e4m3(lo[4 * w + 2] * 0.25f), sat_e4m3(lo[4 * w + 3] * 0.25f));
        outw[2 + w] = pack_e4m3(sat_e4m3(hi[4 * w] * 0.25f), sat_e4m3(hi[4 * w + 1] * 0.25f),
                                sat_e4m3(hi[4 * w + 2] * 0.25f), sat_e4m3(hi[4 * w + 3] * 0.25f));
      }
    }
    *reinterpret_cast<i32x4*>(K8 + ((size_t)(G * 64 + row) * D + pc * 16)) = outw;
  }

  // V: the 64 rows of the group through LDS, then one (d, 16 keys) piece per step
  constexpr int VCH = D / 8;
  for (int c = tid; c < 64 * VCH; c += 256) {
    const int row = c / VCH, pc = c % VCH;
    const int src = source_row(G * 64 + row);
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (src >= 0) raw = *reinterpret_cast<const u32x4*>(V + (int64_t)src * p.stride_l + pc * 8);
    *reinterpret_cast<u32x4*>(&sv[row * SV_STRIDE + pc * 8]) = raw;
  }
  __syncthreads();
  for (int c = tid; c < D * 4; c += 256) {
    const int d = c >> 2, piece = c & 3;
    const int h = piece >> 1, blk = piece & 1;
    i32x4 outw;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float x[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) x[r] = sat_e4m3((float)sv[(32 * blk + 8 * g + 4 * h + r) * SV_STRIDE + d]);
      outw[g] = pack_e4m3(x[0], x[1], x[2], x[3]);
    }
    *reinterpret_cast<i32x4*>(V8 + (((size_t)G * D + d) * 64 + piece * 16)) = outw;
  }
}

// ---------------------------------------------------------------------------
// Attention on the quantised arrays.
// ---------------------------------------------------------------------------
template <int D, int NW, int BC, int OCC, int MODE>
__global__ void __launch_bounds__(NW * 64, OCC) attn_fwd_fp8_kernel(const Fp8Launch pp) {
  const AttnLaunch& p = pp.a;
  constexpr bool kBand = MODE == MODE_BAND || MODE == MODE_PBAND;   // walks a CSR list of key tiles
  constexpr int BR = NW * 32;        // query rows per work-group (one 32-row block per wave)
  constexpr int KB2 = BC / 32;       // 32-key blocks per tile
  constexpr int G64 = BC / 64;       // 64-key contraction steps of the second product
  constexpr int KS = D / 64;         // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;         // 32-row blocks of O^T
  constexpr int TILE_BYTES = BC * D;
  constexpr bool DEEP = D == 128 && MODE == MODE_DENSE;   // pipeline shape, see the stages below
  constexpr int LPT = TILE_BYTES / (NW * 1024);   // load instructions per wave, tile and matrix
  static_assert(TILE_BYTES % (NW * 1024) == 0 && LPT >= 1, "tile must split evenly over the waves");
  static_assert(BC % 64 == 0, "key tiles are whole groups of 64");

  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * TILE_BYTES];
  unsigned char* const sK = smem;                    // [2][BC][D] bytes, swizzled
  unsigned char* const sV = smem + 2 * TILE_BYTES;   // [2][G64][DB][2 halves][2][32 d][16 keys]

  // ---- which tile of which head (XCD-aware: consecutive items share an XCD) ----
  const int per_xcd = (p.n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (item >= p.n_items) return;
  const int qblk = item % p.n_q_blocks;
  const int chunk = (item / p.n_q_blocks) % p.split;
  const int hb = item / p.n_q_blocks / p.split;
  const int hg = hb % p.n_heads;
  const int b = hb / p.n_heads;
  const int head = p.heads ? p.heads[hg] : hg;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;
  const int half = lane >> 5;

  const int64_t base = (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  const __bf16* __restrict__ Q = p.q + base;
  __bf16* __restrict__ O = p.out + base;
  const size_t base8 = ((size_t)b * p.H + head) * (size_t)pp.Lp * D;
  const int L = p.L;

  // ---- the list this head walks ----
  int n_tiles = 0;
  int t_base = 0;     // DENSE: first key tile of this item's chunk
  int n_keys = L;     // DENSE, GATHER: keys of the head's arrays
  typedef const i32x2 __attribute__((address_space(4)))* const_int2_ptr;
  const_int2_ptr entries = nullptr;   // BAND
  const_int2_ptr runs = nullptr;      // BAND
  const int* __restrict__ row_map = nullptr;   // PBAND: row of the tensors for every position of the rearranged order
  if (MODE == MODE_DENSE) {
    const int n_all = (L + BC - 1) / BC;
    t_base = chunk * n_all / p.split;
    n_tiles = (chunk + 1) * n_all / p.split - t_base;
  } else {
    const int* rec = p.ws + p.list_table + 4 * p.list_id[hg];
    if (kBand) {
      const int* row_ptr = p.ws + rec[0];
      const int e0 = row_ptr[qblk], e1 = row_ptr[qblk + 1];
      entries = (const_int2_ptr)(uintptr_t)(p.ws + rec[1]) + e0;
      runs = (const_int2_ptr)(uintptr_t)(p.ws + rec[2]);
      n_tiles = e1 - e0;
      if (n_tiles == 0) return;   // rows that another launch computes (text rows of a layer with a text prefix)
      if (MODE == MODE_PBAND) row_map = p.ws + rec[3];
    } else {
      if (qblk < p.skip_q_blocks) return;   // text rows: another launch computes them
      n_tiles = rec[1] / BC;
      n_keys = rec[2];
    }
  }

  // ---- Q fragments: B operand of S^T = K Q^T (lane: query l32, d = 64 ks + 32 half + 0..31) ----
  const float c_scale = p.scale_log2e * 4.0f;
  const int q0 = qblk * BR + wave * 32;
  i32x8 qf[KS];
  {
    int row = q0 + l32;
    row = row < L ? row : L - 1;
    if (MODE == MODE_PBAND) row = row_map[row];   // the pre-pass moved K and V; Q and O go through the map
    const __bf16* src = Q + (int64_t)row * p.stride_l + half * 32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bf16x8 raw = *reinterpret_cast<const bf16x8*>(src + ks * 64 + j * 8);
        const f32x8 x = __builtin_convertvector(raw, f32x8) * c_scale;
        qf[ks][2 * j] = pack_e4m3(sat_e4m3(x[0]), sat_e4m3(x[1]), sat_e4m3(x[2]), sat_e4m3(x[3]));
        qf[ks][2 * j + 1] = pack_e4m3(sat_e4m3(x[4]), sat_e4m3(x[5]), sat_e4m3(x[6]), sat_e4m3(x[7]));
      }
    }
  }

  // Softmax state.  Scores are kept relative to an INTEGER reference exponent:
  // the score accumulators start from nm = -reference, so exp2 applies to the
  // MFMA result as it is.  thr: -inf until the lane has seen its first kept key,
  // afterwards 8 (the largest relative score the reference allows: P <= 256).
  constexpr float kHeadroom = 8.0f;
  f32x16 o[DB], nm;
  f32x4 l4;
  float thr = kNegInf, mx_raw = kNegInf;
#pragma unroll
  for (int i = 0; i < 4; ++i) l4[i] = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) nm[i] = 0.f;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

  // A operand of the row-sum MFMA (16x16x128): fed with a P fragment of the
  // 32x32x64 product (lane: query l32, the 32 keys of half `half`), the unit sees
  // column l % 16 and the quarter l / 16 of its contraction range in lane l.
  // Rows 0 and 8 of A are one over the even quarters, rows 4 and 12 over the odd
  // ones, the other rows are zero: element 0 of the result (row 4 * (l / 16),
  // column l % 16) is the sum over the 64 keys of the lane's own query.
  i32x8 sum_a;
  {
    const int m16 = lane & 15, g16 = lane >> 4;
    const bool on = ((m16 & 7) == 0 && (g16 & 1) == 0) || ((m16 & 7) == 4 && (g16 & 1) == 1);
#pragma unroll
    for (int i = 0; i < 8; ++i) sum_a[i] = on ? 0x38383838 : 0;   // 0x38 = 1.0
  }

  // ---- tile loader: buffer loads straight into LDS, 16 bytes per lane, a wave
  // instruction fills 1 KB of LDS linearly.  K8: the XOR swizzle is applied on the
  // global side.  V8: the lane that fills LDS chunk (group, db, half, j, d) fetches
  // bytes 32 half + 16 j .. of row d of the group. ----
  typedef __attribute__((address_space(3))) void* lds_ptr;
  unsigned g_k[LPT], g_v[LPT];
#pragma unroll
  for (int u = 0; u < LPT; ++u) {
    const int n = (wave * LPT + u) * 64 + lane;   // 16-byte chunk of the tile in LDS
    const int r = n * 16 / D, slot = (n * 16 % D) >> 4;
    g_k[u] = (unsigned)(r * D + ((slot ^ swz_k8<D>(r)) << 4));
    const int dd = n & 31, j = (n >> 5) & 1, hh = (n >> 6) & 1, db = (n >> 7) % DB, g = (n >> 7) / DB;
    g_v[u] = (unsigned)(((g * D + db * 32 + dd) << 6) + ((2 * hh + j) << 4));
  }
  const unsigned head_bytes8 = (unsigned)pp.Lp * (unsigned)D;
  const __amdgpu_buffer_rsrc_t rsrc_k =
      __builtin_amdgcn_make_buffer_rsrc((void*)(pp.k8 + base8), 0, (int)head_bytes8, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_v =
      __builtin_amdgcn_make_buffer_rsrc((void*)(pp.v8t + base8), 0, (int)head_bytes8, 0x00020000);
  auto load_tile = [&](auto is_k_tag, const int buf, const int t) {
    constexpr bool IS_K = decltype(is_k_tag)::value != 0;
    const __amdgpu_buffer_rsrc_t rsrc = IS_K ? rsrc_k : rsrc_v;
    unsigned char* dst = (IS_K ? sK : sV) + buf * TILE_BYTES + wave * (LPT * 1024);
    const int tile = kBand ? entries[t].x : t + t_base;
#pragma unroll
    for (int u = 0; u < LPT; ++u)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(dst + u * 1024), 16, (int)(IS_K ? g_k[u] : g_v[u]),
                                               (int)((unsigned)tile * (unsigned)TILE_BYTES), 0, 0);
  };

  // per-lane LDS read offsets (everything else is an immediate)
  int k_off[KS][2];   // K fragment: key l32 of a 32-key block, chunks 4 ks + 2 half + {0, 1}
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int j = 0; j < 2; ++j) k_off[ks][j] = l32 * D + (((4 * ks + 2 * half + j) ^ swz_k8<D>(l32)) << 4);
  const int v_off = half * 1024 + l32 * 16;   // V fragment: row l32 of a 32-row block of d, half `half`

  // ---- S^T = K Q^T for the tile held in K buffer BUF ----
  auto scores = [&](auto buf_tag, f32x16 (&s)[KB2]) {
    constexpr int BUF = decltype(buf_tag)::value;
    const unsigned char* kbase = sK + BUF * TILE_BYTES;
#pragma unroll
    for (int kb2 = 0; kb2 < KB2; ++kb2) s[kb2] = nm;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2) {
        const i32x4 a0 = *reinterpret_cast<const i32x4*>(kbase + kb2 * 32 * D + k_off[ks][0]);
        const i32x4 a1 = *reinterpret_cast<const i32x4*>(kbase + kb2 * 32 * D + k_off[ks][1]);
        const i32x8 a = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        s[kb2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, qf[ks], s[kb2], 0, 0, 0, 0, 0, 0);
      }
    }
  };

  // ---- masks: element (kb2, i) of a lane is key kb2*32 + (i/4)*8 + half*4 + i%4 ----
  // Returns false when nothing was changed.  Band tiles: a wave first classifies
  // each of its 32 x 32 blocks against the run with wave-uniform arithmetic; only
  // blocks that a band edge (or the end of the sequence) crosses are masked
  // element by element.
  auto apply_mask = [&](f32x16 (&s)[KB2], const int t) -> bool {
    bool changed = false;
    if (kBand) {
      const i32x2 ent = entries[t];
      const int kv0 = ent.x * BC;
      const int r0 = (ent.y >> 1) & 0x7fff, rn = ent.y >> 16;
      const int qw0 = __builtin_amdgcn_readfirstlane(q0);
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2) {
        const int jb0 = kv0 + kb2 * 32;
        const int dmin = jb0 - qw0 - 31, dmax = dmin + 62;
        if (rn == 1) {
          const i32x2 run = runs[r0];
          if (dmin >= run.x && dmax <= run.y && jb0 + 31 < L) continue;
          changed = true;
          if (dmax < run.x || dmin > run.y || jb0 >= L) {
#pragma unroll
            for (int i = 0; i < 16; ++i) s[kb2][i] = kNegInf;
            continue;
          }
        }
        changed = true;
        const int iq = q0 + l32;
        const int jb = jb0 + half * 4;
        f32x16 kept;
#pragma unroll
        for (int i = 0; i < 16; ++i) kept[i] = kNegInf;
        for (int r = r0; r < r0 + rn; ++r) {
          const i32x2 run = runs[r];
          int hi = run.y;
          hi = hi < L - 1 - iq ? hi : L - 1 - iq;
          const int t0 = jb - iq - run.x;
          const unsigned span = (unsigned)(hi - run.x);
          if (hi >= run.x) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const unsigned d = (unsigned)(t0 + (i / 4) * 8 + (i % 4));
              kept[i] = d <= span ? s[kb2][i] : kept[i];
            }
          }
        }
        s[kb2] = kept;
      }
    } else {
      const int limit = n_keys - (t + t_base) * BC - half * 4;
      changed = true;
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          s[kb2][i] = kb2 * 32 + (i / 4) * 8 + (i % 4) < limit ? s[kb2][i] : kNegInf;
    }
    return changed;
  };

  auto tile_max = [&](const f32x16 (&s)[KB2]) {
    float a = kNegInf, bq = kNegInf;   // two chains of v_max3
#pragma unroll
    for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
      for (int i = 0; i < 8; i += 2) {
        a = fmaxf(fmaxf(a, s[kb2][i]), s[kb2][i + 1]);
        bq = fmaxf(fmaxf(bq, s[kb2][8 + i]), s[kb2][8 + i + 1]);
      }
    mx_raw = fmaxf(a, bq);
  };

  // ---- reference update.  When a tile exceeds the reference by more than 8 the
  // reference moves to ceil(row max) - 8, an integer: the scores already
  // computed and the accumulator seed shift by it, l and O scale by an exact
  // power of two.  The branch is wave-uniform and rarely taken.  `flush` runs
  // first inside the branch: it adds what is still waiting to be accumulated
  // under the old reference. ----
  auto settle_max = [&](f32x16 (&s)[KB2], auto&& flush) {
    const float mx = half_max(mx_raw);
    const bool grow = mx > thr;   // false when the lane's tile is fully masked
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      flush();
      const float step = __builtin_ceilf(mx) - kHeadroom;
      const float delta = grow ? step : 0.f;
      const float alpha = (grow && thr != kNegInf) ? __builtin_amdgcn_exp2f(-step) : 1.0f;
      thr = grow ? kHeadroom : thr;
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb2][i] -= delta;
#pragma unroll
      for (int i = 0; i < 16; ++i) nm[i] -= delta;
      l4[0] *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
  };

  // ---- P = exp2(relative score) as E4M3, in the B-operand layout of the second
  // product: byte 16 blk + i of the lane = element i of block 2 g64 + blk ----
  auto exponentiate = [&](const f32x16 (&s)[KB2], i32x8 (&pf)[G64]) {
#pragma unroll
    for (int g64 = 0; g64 < G64; ++g64)
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x16& sv = s[g64 * 2 + blk];
          pf[g64][blk * 4 + g] =
              pack_e4m3(__builtin_amdgcn_exp2f(sv[4 * g]), __builtin_amdgcn_exp2f(sv[4 * g + 1]),
                        __builtin_amdgcn_exp2f(sv[4 * g + 2]), __builtin_amdgcn_exp2f(sv[4 * g + 3]));
        }
  };

  // ---- O^T += V^T P^T and l += rowsum(P) for the tile held in V buffer BUF ----
  auto accumulate = [&](auto buf_tag, const i32x8 (&pf)[G64]) {
    constexpr int BUF = decltype(buf_tag)::value;
    const unsigned char* vbase = sV + BUF * TILE_BYTES + v_off;
#pragma unroll
    for (int g64 = 0; g64 < G64; ++g64) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const unsigned char* src = vbase + (g64 * DB + db) * 2048;
        const i32x4 a0 = *reinterpret_cast<const i32x4*>(src);
        const i32x4 a1 = *reinterpret_cast<const i32x4*>(src + 512);
        const i32x8 a = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        o[db] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, pf[g64], o[db], 0, 0, 0, 0, 0, 0);
      }
      l4 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(sum_a, pf[g64], l4, 0, 0, 0, 0, 0, 0);
    }
  };

  // Two pipeline shapes.  FLAT (two tiles deep, the shape of the bf16 kernel): a
  // stage turns the scores of tile t into P and accumulates P V of the same tile.
  // The FP8 product takes the probabilities of 64 keys at once, so its first
  // instruction waits for the whole tile's exponentials and the matrix pipe of
  // the wave idles meanwhile (the other wave of the SIMD fills in).  DEEP (three
  // tiles deep): P of tile t is consumed one stage later, nothing in a stage
  // waits for anything else in it; it costs one more stage per list and eight
  // more registers per 64 keys of tile, and pays only for long dense lists at
  // D = 128.
  f32x16 s_a[KB2], s_b[KB2];
  if (!DEEP) {
    if (n_tiles > 0) {
      load_tile(Int<1>{}, 0, 0);
      load_tile(Int<0>{}, 0, 0);
      if (n_tiles > 1) load_tile(Int<1>{}, 1, 1);
    }
    __syncthreads();
    if (n_tiles > 0) {
      scores(Int<0>{}, s_a);
      tile_max(s_a);
    }
    __syncthreads();   // K(0) has been read by every wave before the first stage requests K(2) into its buffer

    // One pipeline stage (see the bf16 kernel): on entry s_cur holds the raw scores
    // of tile t; LDS holds K(t+1) and V(t); K(t+2) and V(t+1) are requested here.
    // INNER: t + 2 is not the last tile of the list, so outside band lists nothing
    // of tile t can be masked.
    auto flat_stage = [&](auto par_tag, auto next_tag, auto inner_tag, const int t, f32x16 (&s_cur)[KB2],
                     f32x16 (&s_next)[KB2]) {
      constexpr int PAR = decltype(par_tag)::value;
      constexpr bool has1 = decltype(next_tag)::value != 0;
      constexpr bool INNER = decltype(inner_tag)::value != 0;
      const bool has2 = INNER || t + 2 < n_tiles;
      if (has2) load_tile(Int<1>{}, PAR, t + 2);
      if (has1) load_tile(Int<0>{}, PAR ^ 1, t + 1);
      bool masked;
      if (kBand) masked = !(entries[t].y & 1);
      else if (INNER) masked = false;
      else masked = (t + t_base + 1) * BC > n_keys;
      if (masked && apply_mask(s_cur, t)) tile_max(s_cur);
      settle_max(s_cur, []() {});
      i32x8 pf[G64];
      if (has1) scores(Int<PAR ^ 1>{}, s_next);
      exponentiate(s_cur, pf);
      if (has1) tile_max(s_next);
      accumulate(Int<PAR>{}, pf);
      if (has1) {
        // Issue order: one MFMA, the LDS reads that feed the MFMAs two steps later,
        // then a share of the vector work (0x008 MFMA, 0x100 DS read, 0x002 VALU, 0x400 TRANS).
        constexpr int N_QK = KS * KB2, N_PV = G64 * DB, N_SUM = G64;
        constexpr int N_KRD = N_QK * 2, N_VRD = N_PV * 2;
        // per score element: one exp2, half a conversion, half a max3
        constexpr int VALU_PER = (KB2 * 16 * 2 + N_QK + N_PV + N_SUM - 1) / (N_QK + N_PV + N_SUM);
        constexpr int AHEAD = 4;   // reads issued ahead of the MFMA that needs them (two MFMAs' worth)
        __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
        for (int i = 0; i < N_QK; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (2 * i + AHEAD < N_KRD + N_VRD) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
        }
#pragma unroll
        for (int g = 0; g < G64; ++g) {
#pragma unroll
          for (int j = 0; j < DB; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (2 * (N_QK + g * DB + j) + AHEAD < N_KRD + N_VRD) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
        }
      }
      if (has1) asm volatile("" : "+v"(mx_raw));   // keeps the maximum chain of the next tile inside this block
      __syncthreads();
    };

    int t = 0;
    for (; t + 5 <= n_tiles; t += 2) {
      flat_stage(Int<0>{}, Int<1>{}, Int<1>{}, t, s_a, s_b);
      flat_stage(Int<1>{}, Int<1>{}, Int<1>{}, t + 1, s_b, s_a);
    }
    for (; t + 2 < n_tiles; t += 2) {
      flat_stage(Int<0>{}, Int<1>{}, Int<0>{}, t, s_a, s_b);
      flat_stage(Int<1>{}, Int<1>{}, Int<0>{}, t + 1, s_b, s_a);
    }
    if (t + 1 < n_tiles) {
      flat_stage(Int<0>{}, Int<1>{}, Int<0>{}, t, s_a, s_b);
      flat_stage(Int<1>{}, Int<0>{}, Int<0>{}, t + 1, s_b, s_a);
    } else if (t < n_tiles) {
      flat_stage(Int<0>{}, Int<0>{}, Int<0>{}, t, s_a, s_b);
    }
  } else {
    i32x8 pf_a[G64], pf_b[G64];
    if (n_tiles > 0) {
      load_tile(Int<1>{}, 0, 0);
      if (n_tiles > 1) load_tile(Int<1>{}, 1, 1);
    }
    __syncthreads();
    if (n_tiles > 0) {
      scores(Int<0>{}, s_a);
      tile_max(s_a);
    }
    __syncthreads();   // K(0) has been read by every wave before the first stage requests K(2) into its buffer

    // One pipeline stage, three tiles deep.  On entry s_cur holds the raw scores of
    // tile t and pf_prev the probabilities of tile t - 1; LDS holds K(t+1) and
    // V(t-1); K(t+2) and V(t) are requested here.  The block then contains the
    // scores of tile t + 1 and O += P V of tile t - 1 on the matrix pipe, and the
    // exponentials of tile t plus the maximum of tile t + 1 on the vector pipe:
    // nothing in it waits for anything else in it.  (The FP8 product takes the
    // probabilities of 64 keys at once, so P of a tile cannot be consumed in the
    // stage that produces it without stalling the matrix pipe.)
    // FIRST: t = 0, nothing to accumulate yet.  NEXT: a tile t + 1 exists.
    // INNER: t + 2 is not the last tile of the list, so outside band lists nothing
    // of tile t can be masked.
    auto deep_stage = [&](auto par_tag, auto first_tag, auto next_tag, auto inner_tag, const int t, f32x16 (&s_cur)[KB2],
                     f32x16 (&s_next)[KB2], i32x8 (&pf_prev)[G64], i32x8 (&pf_cur)[G64]) {
      constexpr int PAR = decltype(par_tag)::value;     // t & 1
      constexpr bool FIRST = decltype(first_tag)::value != 0;
      constexpr bool has1 = decltype(next_tag)::value != 0;
      constexpr bool INNER = decltype(inner_tag)::value != 0;
      const bool has2 = INNER || t + 2 < n_tiles;
      if (has2) load_tile(Int<1>{}, PAR, t + 2);   // K(t+2) takes the place of K(t), read in the last stage
      load_tile(Int<0>{}, PAR, t);                 // V(t) takes the place of V(t-2)
      bool masked;
      if (kBand) masked = !(entries[t].y & 1);
      else if (INNER) masked = false;
      else masked = (t + t_base + 1) * BC > n_keys;
      if (masked && apply_mask(s_cur, t)) tile_max(s_cur);
      settle_max(s_cur, [&]() {
        if (!FIRST) {
          accumulate(Int<PAR ^ 1>{}, pf_prev);
#pragma unroll
          for (int g64 = 0; g64 < G64; ++g64)
#pragma unroll
            for (int i = 0; i < 8; ++i) pf_prev[g64][i] = 0;   // the block below adds it once more: zeros now
        }
      });
      if (has1) scores(Int<PAR ^ 1>{}, s_next);
      if (!FIRST) accumulate(Int<PAR ^ 1>{}, pf_prev);
      exponentiate(s_cur, pf_cur);
      if (has1) tile_max(s_next);
      if (has1 && !FIRST) {
        // Issue order: one MFMA, the LDS reads that feed the MFMAs two steps later,
        // then a share of the vector work (0x008 MFMA, 0x100 DS read, 0x002 VALU, 0x400 TRANS).
        constexpr int N_QK = KS * KB2, N_PV = G64 * DB, N_SUM = G64;
        constexpr int N_RD = (N_QK + N_PV) * 2;
        // per score element: one exp2, half a conversion, half a max3
        constexpr int VALU_PER = (KB2 * 16 * 2 + N_QK + N_PV + N_SUM - 1) / (N_QK + N_PV + N_SUM);
        constexpr int AHEAD = 4;   // reads issued ahead of the MFMA that needs them (two MFMAs' worth)
        __builtin_amdgcn_sched_group_barrier(0x100, AHEAD, 0);
#pragma unroll
        for (int i = 0; i < N_QK; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if (2 * i + AHEAD < N_RD) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
        }
#pragma unroll
        for (int g = 0; g < G64; ++g) {
#pragma unroll
          for (int j = 0; j < DB; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (2 * (N_QK + g * DB + j) + AHEAD < N_RD) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
        }
      }
      if (has1) asm volatile("" : "+v"(mx_raw));   // keeps the maximum chain of the next tile inside this block
      // the loads issued at the top of the stage must have landed before anyone reads them
      __syncthreads();
    };

    // Tile 0 alone, then two stages per trip (odd tile first) so that buffer indices
    // and register sets stay static; after the last stage the probabilities of the
    // last tile are still to be accumulated.
    if (n_tiles > 1) {
      deep_stage(Int<0>{}, Int<1>{}, Int<1>{}, Int<0>{}, 0, s_a, s_b, pf_b, pf_a);
      int t = 1;
      for (; t + 5 <= n_tiles; t += 2) {
        deep_stage(Int<1>{}, Int<0>{}, Int<1>{}, Int<1>{}, t, s_b, s_a, pf_a, pf_b);
        deep_stage(Int<0>{}, Int<0>{}, Int<1>{}, Int<1>{}, t + 1, s_a, s_b, pf_b, pf_a);
      }
      for (; t + 2 < n_tiles; t += 2) {
        deep_stage(Int<1>{}, Int<0>{}, Int<1>{}, Int<0>{}, t, s_b, s_a, pf_a, pf_b);
        deep_stage(Int<0>{}, Int<0>{}, Int<1>{}, Int<0>{}, t + 1, s_a, s_b, pf_b, pf_a);
      }
      if (t + 1 < n_tiles) {
        deep_stage(Int<1>{}, Int<0>{}, Int<1>{}, Int<0>{}, t, s_b, s_a, pf_a, pf_b);
        deep_stage(Int<0>{}, Int<0>{}, Int<0>{}, Int<0>{}, t + 1, s_a, s_b, pf_b, pf_a);
        accumulate(Int<0>{}, pf_a);
      } else {
        deep_stage(Int<1>{}, Int<0>{}, Int<0>{}, Int<0>{}, t, s_b, s_a, pf_a, pf_b);
        accumulate(Int<1>{}, pf_b);
      }
    } else if (n_tiles == 1) {
      deep_stage(Int<0>{}, Int<1>{}, Int<0>{}, Int<0>{}, 0, s_a, s_b, pf_b, pf_a);
      accumulate(Int<0>{}, pf_a);
    }
  }

  // ---- split launch: leave the chunk's state for the merge kernel (layout of the bf16 kernel) ----
  if (MODE == MODE_DENSE && p.split > 1) {
    float* dst = p.partial + ((size_t)item * NW + wave) * ((DB * 16 + 2) * 64) + lane;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[(db * 16 + i) * 64] = o[db][i];
    dst[(DB * 16) * 64] = -nm[0];
    dst[(DB * 16 + 1) * 64] = l4[0];
    return;
  }

  // ---- epilogue: O = O^T / l, bf16, lane owns query l32: 4 consecutive d per store ----
  const float inv = 1.0f / l4[0];
  const int row = q0 + l32;
  if (row < L) {
    __bf16* dst = O + (int64_t)(MODE == MODE_PBAND ? row_map[row] : row) * p.stride_l;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x2 a01 = {o[db][g * 4 + 0] * inv, o[db][g * 4 + 1] * inv};
        const f32x2 a23 = {o[db][g * 4 + 2] * inv, o[db][g * 4 + 3] * inv};
        const bf16x2 b01 = __builtin_convertvector(a01, bf16x2);
        const bf16x2 b23 = __builtin_convertvector(a23, bf16x2);
        const bf16x4 out4 = {b01[0], b01[1], b23[0], b23[1]};
        *reinterpret_cast<bf16x4*>(dst + db * 32 + g * 8 + half * 4) = out4;
      }
    }
  }
}

template <int D, int NW, int BC, int OCC>
hipError_t launch_mode_fp8(const Fp8Launch& p, int mode, hipStream_t stream) {
  const int per_xcd = (p.a.n_items + 7) / 8;
  const dim3 grid(per_xcd * 8), block(NW * 64);
  switch (mode) {
    case MODE_DENSE:
      hipLaunchKernelGGL((attn_fwd_fp8_kernel<D, NW, BC, OCC, MODE_DENSE>), grid, block, 0, stream, p);
      break;
    case MODE_BAND:
      hipLaunchKernelGGL((attn_fwd_fp8_kernel<D, NW, BC, OCC, MODE_BAND>), grid, block, 0, stream, p);
      break;
    case MODE_GATHER:
      hipLaunchKernelGGL((attn_fwd_fp8_kernel<D, NW, BC, OCC, MODE_GATHER>), grid, block, 0, stream, p);
      break;
    case MODE_PBAND:
      hipLaunchKernelGGL((attn_fwd_fp8_kernel<D, NW, BC, OCC, MODE_PBAND>), grid, block, 0, stream, p);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_quantise_kv(const Fp8Launch& p, int mode, hipStream_t stream) {
  if (p.a.n_heads <= 0) return hipSuccess;
  if (!p.k8 || !p.v8t || p.Lp != fp8_padded_len(p.a.L)) return hipErrorInvalidValue;
  const dim3 grid(p.Lp / 64, p.a.n_heads * p.a.B), block(256);
  const int gather = mode == MODE_GATHER ? 1 : mode == MODE_PBAND ? 2 : 0;
  if (gather == 2 && (p.map_len < 1 || p.map_len > p.Lp)) return hipErrorInvalidValue;
  if (p.a.D == 128) hipLaunchKernelGGL(quantise_kv_kernel<128>, grid, block, 0, stream, p, gather);
  else if (p.a.D == 64) hipLaunchKernelGGL(quantise_kv_kernel<64>, grid, block, 0, stream, p, gather);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_attention_fp8(const Fp8Launch& p, int mode, hipStream_t stream, bool small_q) {
  if (p.a.n_items <= 0) return hipSuccess;
  if (!p.k8 || !p.v8t || p.Lp != fp8_padded_len(p.a.L)) return hipErrorInvalidValue;
  if (p.a.split < 1 || (p.a.split > 1 && (mode != MODE_DENSE || !p.a.partial))) return hipErrorInvalidValue;
  if (small_q) {   // small query tile: the band modes, and the compacted stripe heads (no list depends on it)
    if (mode != MODE_BAND && mode != MODE_PBAND && mode != MODE_GATHER) return hipErrorInvalidValue;
    const int per_xcd = (p.a.n_items + 7) / 8;
    const dim3 grid(per_xcd * 8);
    if (p.a.D == 128) {
      using T = Tile128s;
      if (mode == MODE_BAND) hipLaunchKernelGGL((attn_fwd_fp8_kernel<128, T::NW, T::BC, T::OCC, MODE_BAND>), grid, dim3(T::NW * 64), 0, stream, p);
      else if (mode == MODE_PBAND) hipLaunchKernelGGL((attn_fwd_fp8_kernel<128, T::NW, T::BC, T::OCC, MODE_PBAND>), grid, dim3(T::NW * 64), 0, stream, p);
      else hipLaunchKernelGGL((attn_fwd_fp8_kernel<128, T::NW, T::BC, T::OCC, MODE_GATHER>), grid, dim3(T::NW * 64), 0, stream, p);
    } else if (p.a.D == 64) {
      using T = Tile64s;
      if (mode == MODE_BAND) hipLaunchKernelGGL((attn_fwd_fp8_kernel<64, T::NW, T::BC, T::OCC, MODE_BAND>), grid, dim3(T::NW * 64), 0, stream, p);
      else if (mode == MODE_PBAND) hipLaunchKernelGGL((attn_fwd_fp8_kernel<64, T::NW, T::BC, T::OCC, MODE_PBAND>), grid, dim3(T::NW * 64), 0, stream, p);
      else hipLaunchKernelGGL((attn_fwd_fp8_kernel<64, T::NW, T::BC, T::OCC, MODE_GATHER>), grid, dim3(T::NW * 64), 0, stream, p);
    } else {
      return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  // the tiles are those of the bf16 kernels, so one plan serves both
  static_assert(Tile128::QB == 1 && Tile64::QB == 1, "the FP8 kernel keeps one 32-row block per wave");
  if (p.a.D == 128) return launch_mode_fp8<128, Tile128::NW, Tile128::BC, Tile128::OCC>(p, mode, stream);
  if (p.a.D == 64) return launch_mode_fp8<64, Tile64::NW, Tile64::BC, Tile64::OCC>(p, mode, stream);
  return hipErrorInvalidValue;
}

}  // namespace svd
