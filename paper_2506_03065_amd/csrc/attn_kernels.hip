// gfx950 (MI355X, CDNA4) kernels of the sparse attention forward.
//
// One kernel template serves the three computing modes of Section 4.2:
//   DENSE   M_0, Eq. 1 over every key block
//   BAND    M_2 / M_3 (Section 4.1.2 diagonal and multi-diagonal patterns):
//           key blocks come from a CSR list, partially kept tiles are masked
//           element-wise against the runs of kept diagonals
//   GATHER  M_4 (vertical-stripe pattern): key rows are gathered through the
//           head's sorted column list
// plus a fill kernel for M_1 (skipped heads, zeros).  A launch covers all heads
// of a group (Section 4.2: heads sharing a mode are fused).
//
// Per work-group: one tile of BR query rows of one head.  Online-softmax
// recurrence over the listed key tiles; scores are computed TRANSPOSED,
// S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so that a lane owns one query
// column: the row maximum is a per-lane scalar (one cross-half exchange), and
// the exponentiated scores already sit in the operand layout of the second
// product O^T += V^T P^T.  V^T fragments come from the row-major V tile in LDS
// through the transposing LDS read (ds_read_b64_tr_b16).  Accumulation, scores
// and softmax are fp32; P is rounded to bf16 for the second product, and its
// row sums are taken on the matrix pipe.
//
// K and V tiles travel global -> LDS directly (buffer loads with the LDS bit),
// one tile ahead of their use.  The loop is software-pipelined inside each
// wave: while the VALU turns the scores of tile t into P, the matrix pipe
// already computes the scores of tile t + 1; K therefore runs one tile ahead of
// V through the LDS buffers.  The vector work per score is one exp2, half a
// conversion and half a max3: Q carries log2(e) / sqrt(D), and the score
// accumulators are seeded with minus the reference exponent.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "attn_kernels.h"

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
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr float kNegInf = -__builtin_inff();

// Exchange between the two half-waves (lanes l and l ^ 32) with
// v_permlane32_swap: given (a, b) it returns {a.lower | b.lower moved up,
// a.upper moved down | b.upper}; with a == b == x every lane gets the value of
// the lower-half lane of its pair and that of the upper-half lane.
__device__ __forceinline__ void half_pair(float x, float* own_lo, float* own_hi) {
  const unsigned a = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
  const unsigned r0 = r[0], r1 = r[1];   // scalars first: bit_cast of a vector element misreads lane 0
  *own_lo = __builtin_bit_cast(float, r0);
  *own_hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float half_max(float x) {
  float lo, hi;
  half_pair(x, &lo, &hi);
  return fmaxf(lo, hi);
}

// 16-byte chunk swizzles of the LDS tiles (row = key, chunk = 8 bf16 of D).
// K is read 16 bytes per lane with consecutive lanes on consecutive keys; V is
// read through the transposing read, 4 keys x 64 bytes per half-wave.  Both
// depend only on row bits that are lane bits at the reading side.
template <int D>
__device__ __forceinline__ int swz_k(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int swz_v(int row) {
  return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

template <int N>
using Int = std::integral_constant<int, N>;

// Uniform values held in vector registers (arguments of a non-inlined function, words loaded
// through a vector load) moved to scalar registers; a no-op on values that already are scalar.
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
// (Every pointer that goes through here points into global memory.  Rebuilt from two integers it
// would be a pointer of unknown address space and every access through it a FLAT access, which is
// slower and shares the LDS counter; the detour through the global address space keeps them global.)
template <typename T>
__device__ __forceinline__ T* uni(T* ptr) {
  const unsigned long long u = (unsigned long long)ptr;
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)u);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(u >> 32));
  typedef T __attribute__((address_space(1)))* global_ptr;
  return (T*)(global_ptr)(uintptr_t)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ int64_t uni(int64_t x) {
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(unsigned long long)x);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)x >> 32));
  return (int64_t)(((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ float uni(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}
// a pointer into the constant address space (the plan's lists), made scalar
template <typename T>
__device__ __forceinline__ const T __attribute__((address_space(4)))* uni_const(const T __attribute__((address_space(4)))* ptr) {
  const unsigned long long u = (unsigned long long)(uintptr_t)ptr;
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)u);
  const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(u >> 32));
  return (const T __attribute__((address_space(4)))*)(uintptr_t)(((unsigned long long)hi << 32) | lo);
}

// One item = one tile of BR query rows of one head (and, for split dense launches,
// one chunk of the key range): everything a work-group does between picking the
// item and storing its rows.  smem: 4 * BC * D * 2 bytes of LDS, 16-byte aligned.
// Every wave of the work-group calls it with the same item; a return leaves no
// wave behind at a barrier (all returns are work-group uniform).
template <int D, int NW, int QB, int BC, int OCC, int MODE>
__device__ __forceinline__ void attn_item(const AttnLaunch& p, const int item, unsigned char* const smem) {
  constexpr bool kBand = MODE == MODE_BAND || MODE == MODE_PBAND;        // walks a CSR list of key tiles
  constexpr bool kIndirect = MODE == MODE_PBAND;   // key rows come through an index list (the row map)
  constexpr bool kGathered = MODE == MODE_GATHER;  // K and V are the group's gathered rows: a short dense head
  constexpr int NT = NW * 64;
  constexpr int QW = QB * 32;       // query rows per wave
  constexpr int BR = NW * QW;       // query rows per work-group
  constexpr int CH = D / 8;         // 16-byte chunks per row
  constexpr int KB2 = BC / 32;      // 32-key blocks per tile
  constexpr int KS = D / 16;        // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;        // 32-row blocks of O^T
  constexpr int NCH = BC * CH / NT; // chunks per thread and tile (K and V each)
  static_assert(BC * CH % NT == 0, "tile must split evenly over the threads");
  constexpr int TILE_BYTES = BC * D * 2;
  constexpr int ROW_BYTES = D * 2;

  unsigned char* const sK = smem;                    // [2][BC][D] bf16, swizzled
  unsigned char* const sV = smem + 2 * TILE_BYTES;   // [2][BC][D] bf16, swizzled

  const int qblk = item % p.n_q_blocks;
  const int chunk = (item / p.n_q_blocks) % p.split;   // key-range chunk (dense launches only)
  const int hb = item / p.n_q_blocks / p.split;
  const int hg = hb % p.n_heads;
  const int b = hb / p.n_heads;
  const int head = uni(p.heads ? p.heads[hg] : hg);   // scalar: the buffer resources of K and V are built from it

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps everything derived from it in scalar registers
  const int l32 = lane & 31;
  const int half = lane >> 5;

  const int64_t base = (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  const __bf16* __restrict__ Q = p.q + base;
  const __bf16* __restrict__ K = kGathered ? p.gathered + (size_t)hb * 2 * p.gather_pad * D : p.k + base;
  const __bf16* __restrict__ V = kGathered ? K + (size_t)p.gather_pad * D : p.v + base;
  __bf16* __restrict__ O = p.out + base;
  const int L = p.L;

  // ---- the list this head walks ----
  int n_tiles = 0;
  int t_base = 0;                               // DENSE: first key tile of this item's chunk
  // The band lists are read through the constant address space: the plan's
  // workspace is never written by a kernel, and loads with a uniform address
  // from that space are scalar loads, which neither queue behind nor wait for
  // the tile loads in flight.
  typedef const i32x2 __attribute__((address_space(4)))* const_int2_ptr;
  const_int2_ptr entries = nullptr;   // BAND
  const_int2_ptr runs = nullptr;      // BAND
  const int* __restrict__ cols = nullptr;      // PBAND: the row map
  int n_cols = 0;                              // GATHER: the head's columns (the keys of its gathered arrays)
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
      if (MODE == MODE_PBAND) cols = p.ws + rec[3];
    } else {
      if (qblk < p.skip_q_blocks) return;   // text rows: another launch computes them
      n_tiles = rec[1] / BC;
      n_cols = rec[2];
    }
  }

  // The list pointers and counts are uniform but may have been loaded through the vector
  // memory path: as scalars, the list reads in the loop are scalar loads, which neither
  // queue behind nor wait for the tile loads in flight.
  entries = uni_const(entries);
  runs = uni_const(runs);
  cols = uni(cols);
  n_tiles = uni(n_tiles);
  n_cols = uni(n_cols);
  t_base = uni(t_base);

  // ---- Q fragments: B operand of S^T = K Q^T (lane: query l32, 8 of 16 d) ----
  // Q is multiplied by log2(e) / sqrt(D) here, once, and rounded back to bf16:
  // the scores then come out of the matrix pipe in the exponent domain of exp2
  // and need no per-element scaling.
  const float c_scale = p.scale_log2e;
  const int q0 = qblk * BR + wave * QW;
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int row = q0 + qb * 32 + l32;
    row = row < L ? row : L - 1;
    if (MODE == MODE_PBAND) row = cols[row];   // position of the rearranged order -> row of the tensor
    const __bf16* src = Q + (int64_t)row * p.stride_l + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 raw = *reinterpret_cast<const bf16x8*>(src + ks * 16);
      const f32x8 scaled = __builtin_convertvector(raw, f32x8) * c_scale;
      qf[qb][ks] = __builtin_convertvector(scaled, bf16x8);
    }
  }

  // Softmax state per 32-row block.  Scores are kept RELATIVE to a reference
  // exponent: the score accumulators start from nm = -reference (16 copies, the
  // C operand of the first MFMA of a block), so exp2 applies to the MFMA result
  // as it is.  thr is the excess over the reference that makes the lane move
  // it: -inf until the lane has seen its first kept key, kLazyLog2 afterwards.
  // The row sums accumulate in element 0 of l4 through a small MFMA.
  constexpr float kLazyLog2 = 8.0f;
  f32x16 o[DB][QB], nm[QB];
  f32x4 l4[QB];
  float thr[QB], mx_raw[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    thr[qb] = kNegInf;
    mx_raw[qb] = kNegInf;
#pragma unroll
    for (int i = 0; i < 4; ++i) l4[qb][i] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) nm[qb][i] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][qb][i] = 0.f;
  }
  // A operand of the row-sum MFMA (16x16x32): fed with a P fragment laid out for
  // the 32x32x16 product (lane: query l32, 8 keys of half `half`), the 16x16x32
  // unit sees query l%16 + 16*((l/16)&1) and keys 8*(l/32).. in lane l.  Rows 0
  // and 8 of A select the lanes of the even 16-lane blocks, rows 4 and 12 those
  // of the odd ones, all other rows are zero: element 0 of the result (row
  // 4*(l/16), column l%16) is then the sum over the 16 keys of the lane's own
  // query, in every lane.
  bf16x8 sum_a;
  {
    const int m16 = lane & 15, g16 = lane >> 4;
    const bool on = ((m16 & 7) == 0 && (g16 & 1) == 0) || ((m16 & 7) == 4 && (g16 & 1) == 1);
    const __bf16 v = on ? (__bf16)1.0f : (__bf16)0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) sum_a[i] = v;
  }

  // ---- tile loader: direct global -> LDS loads (global_load_lds_dwordx4: 16 bytes
  // per lane, a wave instruction fills 1 KB of LDS linearly from a uniform base,
  // no staging registers).  Wave w fills the slabs w*LPT .. w*LPT+LPT-1 of a tile.
  // The XOR swizzle is applied on the global side: the lane that fills chunk
  // slot c' of row r fetches chunk c' ^ swz(r) of that key row, so K and V use
  // different per-lane offsets.  A tile is addressed as a uniform base (scalar
  // registers) plus those 32-bit offsets; only a ragged last tile recomputes
  // them with the row clamped to L - 1 (those rows are masked later). ----
  constexpr int LPT = TILE_BYTES / (NW * 1024);   // load instructions per wave, tile and matrix
  static_assert(TILE_BYTES % (NW * 1024) == 0, "tile must split evenly over the waves");
  typedef __attribute__((address_space(3))) void* lds_ptr;
  typedef __attribute__((address_space(1))) const void* glb_ptr;
  const unsigned stride_bytes = kGathered ? (unsigned)ROW_BYTES : (unsigned)p.stride_l * 2u;   // of a key row
  unsigned g_k[LPT], g_v[LPT];   // DENSE, BAND, GATHER: byte offset inside the tile; PBAND: chunk offset inside the row
  unsigned g_r[LPT];             // PBAND: 4 * row of the slab's lane inside the tile
#pragma unroll
  for (int u = 0; u < LPT; ++u) {
    const int byte = (wave * LPT + u) * 1024 + lane * 16;
    const int r = byte / ROW_BYTES, slot = (byte % ROW_BYTES) >> 4;
    const unsigned ck = (unsigned)(slot ^ swz_k<D>(r)) * 16u, cv = (unsigned)(slot ^ swz_v<D>(r)) * 16u;
    g_r[u] = (unsigned)r * 4u;
    g_k[u] = kIndirect ? ck : (unsigned)r * stride_bytes + ck;
    g_v[u] = kIndirect ? cv : (unsigned)r * stride_bytes + cv;
  }
  // buffer resources of this head's K and V (raw buffers: base, byte range, no swizzle)
  const unsigned head_bytes = kGathered ? (unsigned)p.gather_pad * (unsigned)ROW_BYTES
                                        : (unsigned)(L - 1) * stride_bytes + (unsigned)ROW_BYTES;
  const __amdgpu_buffer_rsrc_t rsrc_k = __builtin_amdgcn_make_buffer_rsrc((void*)K, 0, (int)head_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrc_v = __builtin_amdgcn_make_buffer_rsrc((void*)V, 0, (int)head_bytes, 0x00020000);
  // INNER: the tile is known to lie inside [0, L) (anything but the last tile of a list)
  auto load_tile = [&](auto is_k_tag, auto inner_tag, const int buf, const int t) {
    constexpr bool IS_K = decltype(is_k_tag)::value != 0;
    constexpr bool INNER = decltype(inner_tag)::value != 0;
    const char* src_b = reinterpret_cast<const char*>(IS_K ? K : V);
    const __amdgpu_buffer_rsrc_t rsrc = IS_K ? rsrc_k : rsrc_v;
    unsigned char* dst = (IS_K ? sK : sV) + buf * TILE_BYTES + wave * (LPT * 1024);
    if (kIndirect) {
      // key rows come from the row map at the tile the band list names (-1 = padding: any valid row, masked later)
      const char* list = reinterpret_cast<const char*>(cols + entries[t].x * BC);
#pragma unroll
      for (int u = 0; u < LPT; ++u) {
        int c = *reinterpret_cast<const int*>(list + g_r[u]);
        c = c < 0 ? 0 : c;
        const unsigned off = __umul24((unsigned)c, stride_bytes) + (IS_K ? g_k[u] : g_v[u]);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(dst + u * 1024), 16, (int)off, 0, 0, 0);
      }
    } else {
      const int row0 = (kBand ? entries[t].x : t + t_base) * BC;
      const char* base_b = src_b + (unsigned)row0 * stride_bytes;
      if (INNER || kGathered || row0 + BC <= L) {   // gathered arrays are padded to whole tiles
#pragma unroll
        for (int u = 0; u < LPT; ++u)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(dst + u * 1024), 16, (int)(IS_K ? g_k[u] : g_v[u]),
                                                   (int)((unsigned)row0 * stride_bytes), 0, 0);
      } else {
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
          const int byte = (wave * LPT + u) * 1024 + lane * 16;
          int r = byte / ROW_BYTES;
          const int slot = (byte % ROW_BYTES) >> 4;
          const unsigned c = (unsigned)(slot ^ (IS_K ? swz_k<D>(r) : swz_v<D>(r))) * 16u;
          r = r < L - 1 - row0 ? r : L - 1 - row0;
          __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_ptr)(dst + u * 1024), 16,
                                                   (int)((unsigned)r * stride_bytes + c),
                                                   (int)((unsigned)row0 * stride_bytes), 0, 0);
        }
      }
    }
  };

  // per-lane LDS read offsets (everything else is an immediate)
  int k_off[KS];   // K fragment: key l32 of a 32-key block, chunk 2 * ks + half
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) k_off[ks] = l32 * ROW_BYTES + (((2 * ks + half) ^ swz_k<D>(l32)) << 4);
  const int ti = lane & 15;           // lane inside its block of 16
  const int dsel = (lane >> 4) & 1;   // which 16 of the 32 d rows
  int v_off[DB];   // V^T fragment: key row half*4 + ti/4 of a 16-key step, 4 d from db*32 + dsel*16 + (ti%4)*4
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    const int r = half * 4 + (ti >> 2);
    const int c = db * 4 + 2 * dsel + ((ti & 3) >> 1);
    v_off[db] = r * ROW_BYTES + ((c ^ swz_v<D>(r)) << 4) + ((ti & 1) << 3);
  }

  // ---- S^T = K Q^T for the tile held in K buffer BUF ----
  auto scores = [&](auto buf_tag, f32x16 (&s)[KB2][QB]) {
    constexpr int BUF = decltype(buf_tag)::value;
    const unsigned char* kbase = sK + BUF * TILE_BYTES;
#pragma unroll
    for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) s[kb2][qb] = nm[qb];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(kbase + kb2 * 32 * ROW_BYTES + k_off[ks]);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          s[kb2][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[kb2][qb], 0, 0, 0);
      }
    }
  };

  // ---- masks: element (kb2, i) of a lane is key kb2*32 + (i/4)*8 + half*4 + i%4 ----
  // Returns false when nothing was changed (the wave's part of the tile is kept
  // as a whole).  Band tiles: a wave first classifies each of its 32 x 32 blocks
  // against the run with wave-uniform arithmetic; only blocks that a band edge
  // (or the end of the sequence) actually crosses are masked element by element.
  auto apply_mask = [&](f32x16 (&s)[KB2][QB], const int t) -> bool {
    bool changed = false;
    if (kBand) {
      const i32x2 ent = entries[t];
      const int kv0 = ent.x * BC;
      const int r0 = (ent.y >> 1) & 0x7fff, rn = ent.y >> 16;
      const int qw0 = __builtin_amdgcn_readfirstlane(q0);
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const int jb0 = kv0 + kb2 * 32;                      // first key of the block
          const int dmin = jb0 - (qw0 + qb * 32) - 31, dmax = dmin + 62;   // diagonals the block touches
          if (rn == 1) {
            const i32x2 run = runs[r0];
            if (dmin >= run.x && dmax <= run.y && jb0 + 31 < L) continue;   // kept as a whole
            changed = true;
            if (dmax < run.x || dmin > run.y || jb0 >= L) {                    // dropped as a whole
#pragma unroll
              for (int i = 0; i < 16; ++i) s[kb2][qb][i] = kNegInf;
              continue;
            }
          }
          changed = true;
          const int iq = q0 + qb * 32 + l32;
          const int jb = jb0 + half * 4;   // key of element 0
          f32x16 kept;
#pragma unroll
          for (int i = 0; i < 16; ++i) kept[i] = kNegInf;
          for (int r = r0; r < r0 + rn; ++r) {
            const i32x2 run = runs[r];
            // kept iff run.x <= j - iq <= run.y and j < L
            int hi = run.y;
            hi = hi < L - 1 - iq ? hi : L - 1 - iq;
            const int t0 = jb - iq - run.x;
            const unsigned span = (unsigned)(hi - run.x);    // wraps when nothing is kept: tested below
            if (hi >= run.x) {
#pragma unroll
              for (int i = 0; i < 16; ++i) {
                const unsigned d = (unsigned)(t0 + (i / 4) * 8 + (i % 4));
                kept[i] = d <= span ? s[kb2][qb][i] : kept[i];
              }
            }
          }
          s[kb2][qb] = kept;
        }
      }
    } else {
      // dense: keys past L in the last tile; gather: padding of the column list
      // (the lane-dependent part goes into the limit so that every element is
      // compared with a literal and nothing per element is kept across tiles)
      const int limit = (MODE == MODE_DENSE ? L - (t + t_base) * BC : n_cols - t * BC) - half * 4;
      changed = true;
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            s[kb2][qb][i] = kb2 * 32 + (i / 4) * 8 + (i % 4) < limit ? s[kb2][qb][i] : kNegInf;
    }
    return changed;
  };

  // ---- maximum of a tile's relative scores (per lane: the keys of its half) ----
  auto tile_max = [&](const f32x16 (&s)[KB2][QB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float a = kNegInf, b = kNegInf;   // two chains of v_max3
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          a = fmaxf(fmaxf(a, s[kb2][qb][i]), s[kb2][qb][i + 1]);
          b = fmaxf(fmaxf(b, s[kb2][qb][8 + i]), s[kb2][qb][8 + i + 1]);
        }
      mx_raw[qb] = fmaxf(a, b);
    }
  };

  // ---- lazy reference update.  The reference is only moved when a tile exceeds
  // it by more than kLazyLog2 in the exponent (2^8): until then P keeps the
  // stale reference, which changes no result (any reference cancels in O / l).
  // Moving it shifts the scores already computed and the accumulator seed nm,
  // and rescales l and O; the branch is wave-uniform and rarely taken. ----
  auto settle_max = [&](f32x16 (&s)[KB2][QB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float mx = half_max(mx_raw[qb]);
      const bool grow = mx > thr[qb];   // false when the lane's tile is fully masked
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float delta = grow ? mx : 0.f;
        const float alpha = (grow && thr[qb] != kNegInf) ? __builtin_amdgcn_exp2f(-mx) : 1.0f;
        thr[qb] = grow ? kLazyLog2 : thr[qb];
#pragma unroll
        for (int kb2 = 0; kb2 < KB2; ++kb2)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[kb2][qb][i] -= delta;
#pragma unroll
        for (int i = 0; i < 16; ++i) nm[qb][i] -= delta;
        l4[qb][0] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][qb][i] *= alpha;
      }
    }
  };

  // ---- P = exp2(relative score), rounded to bf16 in the B-operand layout ----
  auto exponentiate = [&](const f32x16 (&s)[KB2][QB], bf16x8 (&pf)[KB2][2][QB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int kb2 = 0; kb2 < KB2; ++kb2) {
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          bf16x8 pk;
#pragma unroll
          for (int i = 0; i < 8; i += 2) {
            const float p0 = __builtin_amdgcn_exp2f(s[kb2][qb][sub * 8 + i]);
            const float p1 = __builtin_amdgcn_exp2f(s[kb2][qb][sub * 8 + i + 1]);
            const f32x2 pp = {p0, p1};
            const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
            pk[i] = pb[0];
            pk[i + 1] = pb[1];
          }
          pf[kb2][sub][qb] = pk;
        }
      }
    }
  };

  // ---- O^T += V^T P^T and l += rowsum(P) for the tile held in V buffer BUF ----
  auto accumulate = [&](auto buf_tag, const bf16x8 (&pf)[KB2][2][QB]) {
    constexpr int BUF = decltype(buf_tag)::value;
    const unsigned char* vbase = sV + BUF * TILE_BYTES;
#pragma unroll
    for (int kb2 = 0; kb2 < KB2; ++kb2) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          // a lane supplies the address of (key row, 4 d) and receives 4 keys of one d
          const unsigned char* src = vbase + (kb2 * 32 + sub * 16) * ROW_BYTES + v_off[db];
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src + 8 * ROW_BYTES));
          const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8 a = __builtin_bit_cast(bf16x8, both);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[kb2][sub][qb], o[db][qb], 0, 0, 0);
        }
        // row sums of the rounded P (numerator and denominator see the same values)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          l4[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sum_a, pf[kb2][sub][qb], l4[qb], 0, 0, 0);
      }
    }
  };

  // ---- prologue: K(0), V(0), K(1) into LDS, scores of tile 0 ----
  f32x16 s_a[KB2][QB], s_b[KB2][QB];
  if (n_tiles > 0) {
    load_tile(Int<1>{}, Int<0>{}, 0, 0);
    load_tile(Int<0>{}, Int<0>{}, 0, 0);
    if (n_tiles > 1) load_tile(Int<1>{}, Int<0>{}, 1, 1);
  }
  __syncthreads();
  if (n_tiles > 0) {
    scores(Int<0>{}, s_a);
    tile_max(s_a);
  }
  // The first stage requests K(2) into the buffer of K(0) at once: every wave must
  // have read K(0) before any wave gets there (the stages end with a barrier, the
  // prologue needs its own).
  __syncthreads();

  // One pipeline stage.  On entry s_cur holds the raw scores of tile t; LDS holds
  // K(t+1) in K buffer (t+1)&1 and V(t) in V buffer t&1, while K(t+2) and V(t+1)
  // travel global -> registers -> LDS.  NEXT: 1 = a tile t + 1 is known
  // to exist, 0 = tile t is the last one.  With NEXT the two products and the
  // exponentials sit in one basic block: the matrix pipe computes the scores of
  // tile t + 1 and then O += P V of tile t while the vector pipe turns the
  // scores of tile t into P.
  // INNER: t + 2 is not the last tile of the list.  Lists are ascending, so only
  // their last tile can reach past L (or hold padding of a column list): an INNER
  // stage loads without the ragged-tile test and, outside band lists, never masks.
  auto stage = [&](auto par_tag, auto next_tag, auto inner_tag, const int t, f32x16 (&s_cur)[KB2][QB],
                   f32x16 (&s_next)[KB2][QB]) {
    constexpr int PAR = decltype(par_tag)::value;     // t & 1
    constexpr bool has1 = decltype(next_tag)::value != 0;
    constexpr bool INNER = decltype(inner_tag)::value != 0;
    const bool has2 = INNER || t + 2 < n_tiles;
    if (has2) load_tile(Int<1>{}, inner_tag, PAR, t + 2);       // K(t+2) takes the place of K(t), read in the last stage
    if (has1) load_tile(Int<0>{}, inner_tag, PAR ^ 1, t + 1);   // V(t+1) takes the place of V(t-1)
    // partly kept tile?  band lists flag it per entry; the dense and gather loops
    // can only meet one at the very end (keys past L, padding of the column list)
    bool masked;
    if (kBand) masked = !(entries[t].y & 1);
    else if (INNER) masked = false;
    else if (MODE == MODE_DENSE) masked = (t + t_base + 1) * BC > L;
    else masked = (t + 1) * BC > n_cols;
    if (masked && apply_mask(s_cur, t)) tile_max(s_cur);   // the maximum taken before masking may belong to a dropped key
    settle_max(s_cur);
    bf16x8 pf[KB2][2][QB];
    if (has1) scores(Int<PAR ^ 1>{}, s_next);
    exponentiate(s_cur, pf);
    if (has1) tile_max(s_next);
    accumulate(Int<PAR>{}, pf);
    if (has1) {
      // Issue order for the block above: one MFMA, then the LDS reads that feed
      // the MFMAs a few steps later, then a handful of VALU ops that hide behind
      // the MFMA's passes (0x008 MFMA, 0x100 DS read, 0x002 VALU, 0x400 TRANS).
      constexpr int N_QK = KS * KB2 * QB, N_PVG = KB2 * 2, N_PV = N_PVG * DB * QB, N_SUM = N_PVG * QB;
      constexpr int N_KRD = KS * KB2, N_VRD = N_PVG * DB * 2;
      // per score element: one exp2, half a conversion, half a max3
      constexpr int VALU_PER = (KB2 * QB * 16 * 2 + N_QK + N_PV + N_SUM - 1) / (N_QK + N_PV + N_SUM);
      constexpr int K_AHEAD = 4, V_AHEAD = 8;
      __builtin_amdgcn_sched_group_barrier(0x100, K_AHEAD, 0);
#pragma unroll
      for (int i = 0; i < N_QK; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i * N_KRD / N_QK + K_AHEAD < N_KRD) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        else if (i >= N_QK - V_AHEAD / 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
      }
#pragma unroll
      for (int g = 0; g < N_PVG; ++g) {
#pragma unroll
        for (int j = 0; j < DB * QB; ++j) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if ((g * DB * QB + j) * 2 + V_AHEAD < N_VRD) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
        }
#pragma unroll
        for (int j = 0; j < QB; ++j) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x402, VALU_PER, 0);
        }
      }
    }
    // The maximum of the next tile is used only in the next stage: without this
    // anchor at the end of the block the compiler sinks the whole chain out of
    // it, away from the MFMAs that hide it.
    if (has1) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) asm volatile("" : "+v"(mx_raw[qb]));
    }
    // the loads issued at the top of the stage must have landed before anyone reads them
    __syncthreads();
  };

  // Two stages per trip keep buffer indices and the score registers static.
  // The bulk of a list runs through INNER stages (t + 3 is at most the last tile
  // but one for both stages of the trip); the generic stages finish it.
  int t = 0;
  for (; t + 5 <= n_tiles; t += 2) {
    stage(Int<0>{}, Int<1>{}, Int<1>{}, t, s_a, s_b);
    stage(Int<1>{}, Int<1>{}, Int<1>{}, t + 1, s_b, s_a);
  }
  for (; t + 2 < n_tiles; t += 2) {
    stage(Int<0>{}, Int<1>{}, Int<0>{}, t, s_a, s_b);
    stage(Int<1>{}, Int<1>{}, Int<0>{}, t + 1, s_b, s_a);
  }
  if (t + 1 < n_tiles) {
    stage(Int<0>{}, Int<1>{}, Int<0>{}, t, s_a, s_b);
    stage(Int<1>{}, Int<0>{}, Int<0>{}, t + 1, s_b, s_a);
  } else if (t < n_tiles) {
    stage(Int<0>{}, Int<0>{}, Int<0>{}, t, s_a, s_b);
  }

  // ---- split launch: leave the chunk's state for the merge kernel, register by
  // register (each a coalesced 256-byte row of the wave) ----
  if (MODE == MODE_DENSE && p.split > 1) {
    static_assert(MODE != MODE_DENSE || QB == 1, "the split path keeps one 32-row block per wave");
    typedef float __attribute__((address_space(1)))* global_float_ptr;   // global stores, not FLAT ones
    global_float_ptr dst = (global_float_ptr)(uintptr_t)(p.partial + ((size_t)item * NW + wave) * ((DB * 16 + 2) * 64) + lane);
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) dst[(db * 16 + i) * 64] = o[db][0][i];
    dst[(DB * 16) * 64] = -nm[0][0];      // reference exponent of this chunk
    dst[(DB * 16 + 1) * 64] = l4[0][0];   // row sum relative to it
    return;
  }

  // ---- epilogue: O = O^T / l, bf16, lane owns query l32: 4 consecutive d per store ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float inv = 1.0f / l4[qb][0];   // every lane holds the complete sum of its query
    const int row = q0 + qb * 32 + l32;
    if (row < L) {
      __bf16* dst = O + (int64_t)(MODE == MODE_PBAND ? cols[row] : row) * p.stride_l;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x2 a01 = {o[db][qb][g * 4 + 0] * inv, o[db][qb][g * 4 + 1] * inv};
          const f32x2 a23 = {o[db][qb][g * 4 + 2] * inv, o[db][qb][g * 4 + 3] * inv};
          const bf16x2 b01 = __builtin_convertvector(a01, bf16x2);
          const bf16x2 b23 = __builtin_convertvector(a23, bf16x2);
          const bf16x4 out4 = {b01[0], b01[1], b23[0], b23[1]};
          *reinterpret_cast<bf16x4*>(dst + db * 32 + g * 8 + half * 4) = out4;
        }
      }
    }
  }
}


// One launch per group: work-group = one item.
template <int D, int NW, int QB, int BC, int OCC, int MODE>
__global__ void __launch_bounds__(NW * 64, OCC) attn_fwd_kernel(const AttnLaunch p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * BC * D * 2];
  // which tile of which head (XCD-aware: consecutive items share an XCD)
  const int per_xcd = (p.n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (item >= p.n_items) return;
  attn_item<D, NW, QB, BC, OCC, MODE>(p, item, smem);
}


// Merge of a split dense launch: work-group = (query tile, head, batch entry,
// slice of RPS accumulator rows), same thread-to-element mapping as
// attn_fwd_kernel.  Chunks are folded one by one with the online-softmax rule:
// O = O * 2^(m - m') + O_c * 2^(m_c - m').  RPS = all rows for the few chunks of
// a dense group; launches with many chunks and few query tiles (the text rows
// of a layer with a text prefix) use slices of four rows, so that the chain over
// the chunks is short per thread and spread over many work-groups.
template <int D, int NW, int RPS>
__global__ void __launch_bounds__(NW * 64) combine_partials_kernel(const AttnLaunch p) {
  constexpr int DB = D / 32;
  constexpr int BR = NW * 32;
  static_assert(RPS % 4 == 0 && (DB * 16) % RPS == 0, "a slice is a whole number of 4-row groups");
  const int qblk = blockIdx.x % p.n_q_blocks;
  const int hb = blockIdx.x / p.n_q_blocks;
  const int hg = hb % p.n_heads;
  const int b = hb / p.n_heads;
  const int head = p.heads ? p.heads[hg] : hg;
  const int r0 = blockIdx.y * RPS;     // first accumulator row of this slice
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  float o[RPS];
#pragma unroll
  for (int r = 0; r < RPS; ++r) o[r] = 0.f;
  float m = kNegInf, l = 0.f;
#pragma unroll 2
  for (int c = 0; c < p.split; ++c) {
    const size_t item = ((size_t)hb * p.split + c) * p.n_q_blocks + qblk;
    const float* src = p.partial + (item * NW + wave) * ((DB * 16 + 2) * 64) + lane;
    const float mc = src[(DB * 16) * 64], lc = src[(DB * 16 + 1) * 64];
    const float m_new = fmaxf(m, mc);
    const float wa = __builtin_amdgcn_exp2f(m - m_new), wc = __builtin_amdgcn_exp2f(mc - m_new);
    l = l * wa + lc * wc;
#pragma unroll
    for (int r = 0; r < RPS; ++r) o[r] = o[r] * wa + src[(r0 + r) * 64] * wc;
    m = m_new;
  }
  const float inv = 1.0f / l;
  const int row = qblk * BR + wave * 32 + l32;
  if (row < p.L) {
    __bf16* dst = p.out + (int64_t)b * p.stride_b + (int64_t)head * p.stride_h + (int64_t)row * p.stride_l;
#pragma unroll
    for (int rr = 0; rr < RPS; rr += 4) {
      const int db = (r0 + rr) / 16, g = ((r0 + rr) % 16) / 4;
      const f32x2 a01 = {o[rr + 0] * inv, o[rr + 1] * inv};
      const f32x2 a23 = {o[rr + 2] * inv, o[rr + 3] * inv};
      const bf16x2 b01 = __builtin_convertvector(a01, bf16x2);
      const bf16x2 b23 = __builtin_convertvector(a23, bf16x2);
      const bf16x4 out4 = {b01[0], b01[1], b23[0], b23[1]};
      *reinterpret_cast<bf16x4*>(dst + db * 32 + g * 8 + half * 4) = out4;
    }
  }
}

// Pre-pass of a vertical-stripe group (M_4): work-group = 64 key slots of one (batch entry, head).
// Slot j of the head's gathered arrays takes row cols[j] of K and of V; slots past the padded list
// and padding entries are zero (a masked score times a zero row, never times stale bits).
template <int D>
__global__ void __launch_bounds__(256) gather_kv_kernel(const AttnLaunch p) {
  constexpr int CH = D / 8;
  const int hb = blockIdx.y;
  const int hg = hb % p.n_heads, b = hb / p.n_heads;
  const int head = p.heads[hg];
  const int* rec = p.ws + p.list_table + 4 * p.list_id[hg];
  const int* cols = p.ws + rec[0];
  const int padded = rec[1];
  const int64_t base = (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  __bf16* Kg = p.gathered + (size_t)hb * 2 * p.gather_pad * D;
  __bf16* Vg = Kg + (size_t)p.gather_pad * D;
  for (int c = threadIdx.x; c < 64 * CH; c += 256) {
    const int j = blockIdx.x * 64 + c / CH, piece = (c % CH) * 8;
    if (j >= p.gather_pad) continue;
    const int src = j < padded ? cols[j] : -1;
    uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
    if (src >= 0) {
      kk = *reinterpret_cast<const uint4*>(p.k + base + (int64_t)src * p.stride_l + piece);
      vv = *reinterpret_cast<const uint4*>(p.v + base + (int64_t)src * p.stride_l + piece);
    }
    *reinterpret_cast<uint4*>(Kg + (size_t)j * D + piece) = kk;
    *reinterpret_cast<uint4*>(Vg + (size_t)j * D + piece) = vv;
  }
}

// M_1 (Section 4.2): the output of a skipped head is zero.
__global__ void __launch_bounds__(256) zero_heads_kernel(const AttnLaunch p) {
  const int hg = blockIdx.y % p.n_heads;
  const int b = blockIdx.y / p.n_heads;
  const int head = p.heads ? p.heads[hg] : hg;
  __bf16* O = p.out + (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  const int chunks = p.D / 8;
  const int64_t total = (int64_t)p.L * chunks;
  for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total;
       g += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = g / chunks;
    const int c = (int)(g % chunks);
    *reinterpret_cast<uint4*>(O + row * p.stride_l + c * 8) = make_uint4(0, 0, 0, 0);
  }
}

// ---- the whole layer in one launch ----

__global__ void __launch_bounds__(128) reset_counters_kernel(int* counters) {
  if (threadIdx.x < kLayerCounterWords) counters[threadIdx.x] = 0;
}

// Waves per work-group of the layer kernel: eight, one work-group per compute unit, every item on the
// 256-row query tile (a K/V tile in LDS then serves twice the rows of the four-wave form, which ran the
// dense items 4-14 % and the wide-band items 4-7 % slower).
constexpr int kLayerWaves = 8;

// Zero fill of one query tile of a skipped head (M_1).
template <int D>
__device__ __forceinline__ void zero_item(const AttnLaunch& p, const int item) {
  constexpr int BR = kLayerWaves * 32, CH = D / 8;
  const int qblk = item % p.n_q_blocks;
  const int hb = item / p.n_q_blocks;
  const int hg = hb % p.n_heads, b = hb / p.n_heads;
  const int head = p.heads[hg];
  __bf16* O = p.out + (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  for (int c = threadIdx.x; c < BR * CH; c += blockDim.x) {
    const int row = qblk * BR + c / CH;
    if (row < p.L) *reinterpret_cast<uint4*>(O + (int64_t)row * p.stride_l + (c % CH) * 8) = make_uint4(0, 0, 0, 0);
  }
}

// The segment loops of the layer kernel are real functions, not inlined: inlined
// side by side into one kernel the four loop nests get in each other's way in the
// register allocator; as callees each is allocated like the kernel it also is
// elsewhere in this file.  Arguments of a callee travel in vector registers even
// when they are uniform, so everything is made scalar again on entry.
// One segment of the layer kernel: the work-group pulls items of the segment off the eight
// queues, its own XCD's first, until all are empty.  A real function, called once per segment
// (a call per item would save and restore the callee-saved half of the register file around
// every item: measured as more than a gigabyte of scratch traffic per layer).
// KIND = a MODE_* of attn_item, or kZeroKind for the zero fill of skipped heads.
constexpr int kZeroKind = 100;
template <int D, int BC, int KIND>
__device__ __attribute__((noinline)) void layer_segment(const AttnLaunch av, const int first_item_v, const int n_rest_v,
                                                        int* const counters_v, const int home_v, const unsigned smem_v,
                                                        const unsigned pick_v) {
  AttnLaunch a;
  a.q = uni(av.q);
  a.k = uni(av.k);
  a.v = uni(av.v);
  a.out = uni(av.out);
  a.B = uni(av.B);
  a.H = uni(av.H);
  a.L = uni(av.L);
  a.D = uni(av.D);
  a.stride_b = uni(av.stride_b);
  a.stride_h = uni(av.stride_h);
  a.stride_l = uni(av.stride_l);
  a.n_q_blocks = uni(av.n_q_blocks);
  a.n_heads = uni(av.n_heads);
  a.n_items = uni(av.n_items);
  a.heads = uni(av.heads);
  a.list_id = uni(av.list_id);
  a.ws = uni(av.ws);
  a.list_table = uni(av.list_table);
  a.scale_log2e = uni(av.scale_log2e);
  a.split = 1;
  a.partial = nullptr;
  a.gathered = uni(av.gathered);
  a.gather_pad = uni(av.gather_pad);
  a.skip_q_blocks = uni(av.skip_q_blocks);
  const int first_item = uni(first_item_v), n_rest = uni(n_rest_v), home = uni(home_v);
  int* const counters = uni(counters_v);   // this segment's eight queue positions
  typedef __attribute__((address_space(3))) unsigned char* lds_bytes;
  typedef __attribute__((address_space(3))) int* lds_int;
  unsigned char* const smem = (unsigned char*)(lds_bytes)(uintptr_t)uni((int)smem_v);
  lds_int const pick = (lds_int)(uintptr_t)uni((int)pick_v);
  const int per = (n_rest + 7) >> 3;
  // Every queue position only grows, so every loop below ends, and all waves of the
  // work-group take the same path (the position is read by all of them after a barrier).
  for (int probe = 0; probe < 8; ++probe) {
    const int x = (home + probe) & 7;
    int cnt = n_rest - x * per;
    cnt = cnt < 0 ? 0 : (cnt > per ? per : cnt);
    if (cnt == 0) continue;
    for (;;) {
      if (threadIdx.x == 0) *pick = atomicAdd(counters + x, 1);
      __syncthreads();
      const int pos = __builtin_amdgcn_readfirstlane(*pick);
      // the next pick overwrites `pick`, the next item the LDS tiles: everyone must be done with both
      if (pos >= cnt) {
        __syncthreads();
        break;
      }
      const int item = first_item + x * per + pos;
      if (KIND == kZeroKind) zero_item<D>(a, item);
      else attn_item<D, kLayerWaves, 1, BC, 2, (KIND == kZeroKind ? MODE_DENSE : KIND)>(a, item, smem);
      __syncthreads();
    }
  }
}

template <int D, int BC>
__global__ void __launch_bounds__(kLayerWaves * 64, 2) attn_layer_kernel(const LayerLaunch lp) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * BC * D * 2];
  __shared__ int pick;
  typedef __attribute__((address_space(3))) unsigned char* lds_bytes;
  typedef __attribute__((address_space(3))) int* lds_int;
  const unsigned smem_addr = (unsigned)(uintptr_t)(lds_bytes)smem;
  const unsigned pick_addr = (unsigned)(uintptr_t)(lds_int)&pick;
  const int home = blockIdx.x & 7;   // work-groups are dealt to the XCDs in turn
  // Segment after segment, heaviest first; inside a segment a work-group first drains
  // its own XCD's eighth, then the other XCDs' eighths.
  for (int s = 0; s < lp.n_segments; ++s) {
    const LayerSegment sg = lp.seg[s];
    AttnLaunch a = lp.a;
    a.n_q_blocks = sg.n_q_blocks;
    a.n_heads = sg.n_heads;
    a.n_items = sg.n_items + sg.first_item;
    a.heads = lp.a.ws + sg.heads;
    a.list_id = lp.a.ws + sg.list_id;
    a.list_table = sg.list_table;
    int* const counters = lp.counters + s * 8;
    switch (sg.kind) {
      case SEG_DENSE: layer_segment<D, BC, MODE_DENSE>(a, sg.first_item, sg.n_items, counters, home, smem_addr, pick_addr); break;
      case SEG_BAND: layer_segment<D, BC, MODE_BAND>(a, sg.first_item, sg.n_items, counters, home, smem_addr, pick_addr); break;
      case SEG_GATHER: layer_segment<D, BC, MODE_GATHER>(a, sg.first_item, sg.n_items, counters, home, smem_addr, pick_addr); break;
      case SEG_PBAND: layer_segment<D, BC, MODE_PBAND>(a, sg.first_item, sg.n_items, counters, home, smem_addr, pick_addr); break;
      default: layer_segment<D, BC, kZeroKind>(a, sg.first_item, sg.n_items, counters, home, smem_addr, pick_addr); break;
    }
  }
}

template <int D, int NW, int QB, int BC, int OCC>
hipError_t launch_mode(const AttnLaunch& p, int mode, hipStream_t stream) {
  const int per_xcd = (p.n_items + 7) / 8;
  const dim3 grid(per_xcd * 8), block(NW * 64);
  switch (mode) {
    case MODE_DENSE:
      hipLaunchKernelGGL((attn_fwd_kernel<D, NW, QB, BC, OCC, MODE_DENSE>), grid, block, 0, stream, p);
      break;
    case MODE_BAND:
      hipLaunchKernelGGL((attn_fwd_kernel<D, NW, QB, BC, OCC, MODE_BAND>), grid, block, 0, stream, p);
      break;
    case MODE_GATHER:
      hipLaunchKernelGGL((attn_fwd_kernel<D, NW, QB, BC, OCC, MODE_GATHER>), grid, block, 0, stream, p);
      break;
    case MODE_PBAND:
      hipLaunchKernelGGL((attn_fwd_kernel<D, NW, QB, BC, OCC, MODE_PBAND>), grid, block, 0, stream, p);
      break;
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// The band modes on the small query tile.
template <int D, int NW, int QB, int BC, int OCC>
hipError_t launch_band_small(const AttnLaunch& p, int mode, hipStream_t stream) {
  const int per_xcd = (p.n_items + 7) / 8;
  const dim3 grid(per_xcd * 8), block(NW * 64);
  if (mode == MODE_BAND) {
    hipLaunchKernelGGL((attn_fwd_kernel<D, NW, QB, BC, OCC, MODE_BAND>), grid, block, 0, stream, p);
  } else if (mode == MODE_PBAND) {
    hipLaunchKernelGGL((attn_fwd_kernel<D, NW, QB, BC, OCC, MODE_PBAND>), grid, block, 0, stream, p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
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

hipError_t launch_attention(const AttnLaunch& p, int mode, hipStream_t stream, bool small_q) {
  if (p.n_items <= 0) return hipSuccess;
  if (p.split < 1 || (p.split > 1 && (mode != MODE_DENSE || !p.partial))) return hipErrorInvalidValue;
  if (mode == MODE_GATHER && (!p.gathered || p.gather_pad < 1)) return hipErrorInvalidValue;
  if (small_q) {
    if (p.D == 128) return launch_band_small<128, Tile128s::NW, Tile128s::QB, Tile128s::BC, Tile128s::OCC>(p, mode, stream);
    if (p.D == 64) return launch_band_small<64, Tile64s::NW, Tile64s::QB, Tile64s::BC, Tile64s::OCC>(p, mode, stream);
    return hipErrorInvalidValue;
  }
  if (p.D == 128)
    return launch_mode<128, Tile128::NW, Tile128::QB, Tile128::BC, Tile128::OCC>(p, mode, stream);
  if (p.D == 64) return launch_mode<64, Tile64::NW, Tile64::QB, Tile64::BC, Tile64::OCC>(p, mode, stream);
  return hipErrorInvalidValue;
}

int layer_block_q(int) { return kLayerWaves * 32; }

hipError_t launch_layer(const LayerLaunch& p, int n_compute_units, hipStream_t stream) {
  if (p.n_segments < 1) return hipSuccess;
  if (p.n_segments > kMaxSegments || !p.counters || n_compute_units < 1) return hipErrorInvalidValue;
  static_assert(Tile128::NW == kLayerWaves && Tile64::NW == kLayerWaves && Tile128::QB == 1 && Tile64::QB == 1,
                "the layer kernel runs the kernels' own query tile: eight waves of 32 rows");
  long long total = 0;
  for (int s = 0; s < p.n_segments; ++s) {
    if (p.seg[s].n_items < 0 || p.seg[s].first_item < 0 || p.seg[s].kind < SEG_DENSE || p.seg[s].kind > SEG_ZERO)
      return hipErrorInvalidValue;
    total += p.seg[s].n_items;
  }
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(reset_counters_kernel, dim3(1), dim3(128), 0, stream, p.counters);
  static_assert(kLayerCounterWords <= 128, "one thread per queue position");
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  // one resident work-group of eight waves per compute unit, a multiple of eight so that every XCD gets its share
  long long groups = static_cast<long long>(8 / kLayerWaves) * n_compute_units;
  if (groups > total) groups = total;
  groups = (groups + 7) / 8 * 8;
  const dim3 grid((unsigned)groups), block(kLayerWaves * 64);
  if (p.a.D == 128) hipLaunchKernelGGL((attn_layer_kernel<128, Tile128::BC>), grid, block, 0, stream, p);
  else if (p.a.D == 64) hipLaunchKernelGGL((attn_layer_kernel<64, Tile64::BC>), grid, block, 0, stream, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

size_t partial_floats(int D, int n_items) {
  const int nw = D == 128 ? Tile128::NW : Tile64::NW;
  return (size_t)n_items * nw * ((D / 32 * 16 + 2) * 64);
}

hipError_t launch_combine(const AttnLaunch& p, hipStream_t stream) {
  if (p.split <= 1 || p.n_items <= 0) return hipSuccess;
  if (!p.partial) return hipErrorInvalidValue;
  const int tiles = p.n_items / p.split;
  if (p.D == 128) {
    // always in slices of four accumulator rows (measured: the merge of the Wan2.1-like
    // dense group, three chunks, takes 175 us unsliced and about 70 us sliced)
    hipLaunchKernelGGL((combine_partials_kernel<128, Tile128::NW, 4>), dim3(tiles, 16), dim3(Tile128::NW * 64), 0, stream, p);
  } else if (p.D == 64) {
    // sliced for many chunks only; for the few chunks of a dense group the unsliced form is as fast
    if (p.split > 8)
      hipLaunchKernelGGL((combine_partials_kernel<64, Tile64::NW, 4>), dim3(tiles, 8), dim3(Tile64::NW * 64), 0, stream, p);
    else
      hipLaunchKernelGGL((combine_partials_kernel<64, Tile64::NW, 32>), dim3(tiles, 1), dim3(Tile64::NW * 64), 0, stream, p);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_gather_kv(const AttnLaunch& p, hipStream_t stream) {
  if (p.n_heads <= 0) return hipSuccess;
  if (!p.gathered || p.gather_pad < 1 || !p.heads || !p.list_id || !p.ws) return hipErrorInvalidValue;
  const dim3 grid((p.gather_pad + 63) / 64, p.n_heads * p.B), block(256);
  if (p.D == 128) hipLaunchKernelGGL(gather_kv_kernel<128>, grid, block, 0, stream, p);
  else if (p.D == 64) hipLaunchKernelGGL(gather_kv_kernel<64>, grid, block, 0, stream, p);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_zero_heads(const AttnLaunch& p, hipStream_t stream) {
  if (p.n_heads <= 0) return hipSuccess;
  const int64_t total = (int64_t)p.L * (p.D / 8);
  int bx = (int)((total + 255) / 256);
  if (bx > 2048) bx = 2048;
  const dim3 grid(bx, p.n_heads * p.B), block(256);
  hipLaunchKernelGGL(zero_heads_kernel, grid, block, 0, stream, p);
  return hipGetLastError();
}

}  // namespace svd
