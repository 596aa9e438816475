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
// column: the row maximum and row sum are per-lane scalars (one cross-half
// exchange), and the exponentiated scores already sit in the operand layout of
// the second product O^T += V^T P^T.  V^T fragments come from the row-major V
// tile in LDS through the transposing LDS read (ds_read_b64_tr_b16).
// Accumulation, scores and softmax are fp32; P is rounded to bf16 for the
// second product.
//
// The loop is software-pipelined inside each wave: while the VALU turns the
// scores of tile t into P, the matrix pipe already computes the scores of tile
// t + 1; K therefore runs one tile ahead of V through the LDS buffers.
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
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
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
__device__ __forceinline__ float half_sum(float x) {
  float lo, hi;
  half_pair(x, &lo, &hi);
  return lo + hi;
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

template <int D, int NW, int QB, int BC, int OCC, int MODE>
__global__ void __launch_bounds__(NW * 64, OCC) attn_fwd_kernel(const AttnLaunch p) {
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

  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * TILE_BYTES];
  unsigned char* const sK = smem;                    // [2][BC][D] bf16, swizzled
  unsigned char* const sV = smem + 2 * TILE_BYTES;   // [2][BC][D] bf16, swizzled

  // ---- which tile of which head (XCD-aware: consecutive items share an XCD) ----
  const int per_xcd = (p.n_items + 7) >> 3;
  const int item = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (item >= p.n_items) return;
  const int qblk = item % p.n_q_blocks;
  const int hb = item / p.n_q_blocks;
  const int hg = hb % p.n_heads;
  const int b = hb / p.n_heads;
  const int head = p.heads ? p.heads[hg] : hg;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int half = lane >> 5;

  const int64_t base = (int64_t)b * p.stride_b + (int64_t)head * p.stride_h;
  const __bf16* __restrict__ Q = p.q + base;
  const __bf16* __restrict__ K = p.k + base;
  const __bf16* __restrict__ V = p.v + base;
  __bf16* __restrict__ O = p.out + base;
  const int L = p.L;

  // ---- the list this head walks ----
  int n_tiles = 0;
  const int2* __restrict__ entries = nullptr;  // BAND
  const int2* __restrict__ runs = nullptr;     // BAND
  const int* __restrict__ cols = nullptr;      // GATHER
  int n_cols = 0;
  if (MODE == MODE_DENSE) {
    n_tiles = (L + BC - 1) / BC;
  } else {
    const int* rec = p.ws + p.list_table + 4 * p.list_id[hg];
    if (MODE == MODE_BAND) {
      const int* row_ptr = p.ws + rec[0];
      const int e0 = row_ptr[qblk], e1 = row_ptr[qblk + 1];
      entries = reinterpret_cast<const int2*>(p.ws + rec[1]) + e0;
      runs = reinterpret_cast<const int2*>(p.ws + rec[2]);
      n_tiles = e1 - e0;
    } else {
      cols = p.ws + rec[0];
      n_tiles = rec[1] / BC;
      n_cols = rec[2];
    }
  }

  // ---- Q fragments: B operand of S^T = K Q^T (lane: query l32, 8 of 16 d) ----
  const int q0 = qblk * BR + wave * QW;
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int row = q0 + qb * 32 + l32;
    row = row < L ? row : L - 1;
    const __bf16* src = Q + (int64_t)row * p.stride_l + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(src + ks * 16);
  }

  f32x16 o[DB][QB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = kNegInf;
    l_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][qb][i] = 0.f;
  }

  // ---- tile loaders: global -> registers -> LDS, K and V separately ----
  u32x4 kreg[NCH], vreg[NCH];
  int st_off_k[NCH], st_off_v[NCH], ld_row[NCH], ld_col[NCH];
#pragma unroll
  for (int u = 0; u < NCH; ++u) {
    const int g = u * NT + tid;
    const int r = g / CH, c = g % CH;
    ld_row[u] = r;
    ld_col[u] = c * 8;
    st_off_k[u] = r * ROW_BYTES + ((c ^ swz_k<D>(r)) << 4);
    st_off_v[u] = r * ROW_BYTES + ((c ^ swz_v<D>(r)) << 4);
  }
  // global row of key slot r of tile t
  auto key_row = [&](const int t, const int r) -> int {
    if (MODE == MODE_GATHER) {
      const int c = cols[t * BC + r];
      return c < 0 ? 0 : c;
    }
    const int kb = MODE == MODE_BAND ? entries[t].x : t;
    const int j = kb * BC + r;
    return j < L ? j : L - 1;
  };
#define SVD_LOAD(REG, PTR, T)                                                             \
  _Pragma("unroll") for (int u = 0; u < NCH; ++u)                                         \
    REG[u] = *reinterpret_cast<const u32x4*>(PTR + (int64_t)key_row((T), ld_row[u]) * p.stride_l + ld_col[u]);
#define SVD_STORE(REG, SBASE, OFF, BUF)                                                   \
  _Pragma("unroll") for (int u = 0; u < NCH; ++u)                                         \
    *reinterpret_cast<u32x4*>(SBASE + (BUF) * TILE_BYTES + OFF[u]) = REG[u];

  const float c_scale = p.scale_log2e;
  // The running maximum is only raised when a tile exceeds it by more than
  // kLazyLog2 in the exponent (2^8 = 256x): until then P keeps the stale
  // reference, which changes no result (any reference cancels in O / l) but
  // saves the rescale of O and l on most tiles.
  constexpr float kLazyLog2 = 8.0f;
  const float tau = kLazyLog2 / c_scale;

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

  // The pipeline unit is a block of 32 keys (one 32x32 score block per 32 query
  // rows); a key tile of BC keys in LDS holds KB2 of them.  Score registers of
  // one block: s[qb], element i of a lane is key (i/4)*8 + half*4 + i%4.

  // ---- S^T = K Q^T of block kb2 of the tile in K buffer buf (prologue only) ----
  auto scores = [&](const int buf, const int kb2, f32x16 (&s)[QB]) {
    const unsigned char* kbase = sK + buf * TILE_BYTES + kb2 * 32 * ROW_BYTES;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s[qb][i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(kbase + k_off[ks]);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[qb], 0, 0, 0);
    }
  };

  // ---- element masks of block kb2 of tile t ----
  auto apply_mask = [&](f32x16 (&s)[QB], const int t, const int kb2) {
    if (MODE == MODE_BAND) {
      const int2 ent = entries[t];
      const int kv0 = ent.x * BC;
      const int r0 = (ent.y >> 1) & 0x7fff, rn = ent.y >> 16;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int iq = q0 + qb * 32 + l32;
        const int jb = kv0 + kb2 * 32 + half * 4;   // key of element 0
        f32x16 kept;
#pragma unroll
        for (int i = 0; i < 16; ++i) kept[i] = kNegInf;
        for (int r = r0; r < r0 + rn; ++r) {
          const int2 run = runs[r];
          // kept iff run.x <= j - iq <= run.y and j < L
          int hi = run.y;
          hi = hi < L - 1 - iq ? hi : L - 1 - iq;
          const int t0 = jb - iq - run.x;
          const int span = hi - run.x;    // may be negative: nothing kept
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int d = t0 + (i / 4) * 8 + (i % 4);
            kept[i] = (d >= 0 && d <= span) ? s[qb][i] : kept[i];
          }
        }
        s[qb] = kept;
      }
    } else {
      // dense: keys past L in the last tile; gather: padding of the column list
      const int limit = (MODE == MODE_DENSE ? L - t * BC : n_cols - t * BC) - kb2 * 32 - half * 4;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[qb][i] = (i / 4) * 8 + (i % 4) < limit ? s[qb][i] : kNegInf;
    }
  };

  // ---- maximum of a block per query column (lane), both half-waves combined ----
  auto block_max = [&](const f32x16 (&s)[QB], float (&mx)[QB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float m = kNegInf;
#pragma unroll
      for (int i = 0; i < 16; i += 2) m = fmaxf(m, fmaxf(s[qb][i], s[qb][i + 1]));
      mx[qb] = half_max(m);
    }
  };

  // ---- lazy update of the reference maximum; rescales O and l when it moves ----
  float mc[QB];   // reference maximum times the scale, per 32-row block
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) mc[qb] = 0.f;
  auto raise_max = [&](const float (&mx)[QB]) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const bool grow = mx[qb] > m_run[qb] + tau;   // false when the lane's block is fully masked
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float alpha = grow ? __builtin_amdgcn_exp2f((m_run[qb] - mx[qb]) * c_scale) : 1.0f;
        m_run[qb] = grow ? mx[qb] : m_run[qb];
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][qb][i] *= alpha;
        mc[qb] = (m_run[qb] == kNegInf ? 0.f : m_run[qb]) * c_scale;
      }
    }
  };

  // ---- one block without a successor: P = exp2(S c - m c), O^T += V^T P^T ----
  auto finish_block = [&](const int vbuf, const int kb2, const f32x16 (&s)[QB]) {
    const unsigned char* vbase = sV + vbuf * TILE_BYTES + kb2 * 32 * ROW_BYTES;
    bf16x8 pf[2][QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float rs = 0.f;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub)
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          const f32x2 pp = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][sub * 8 + i], c_scale, -mc[qb])),
                            __builtin_amdgcn_exp2f(__builtin_fmaf(s[qb][sub * 8 + i + 1], c_scale, -mc[qb]))};
          const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
          rs += pp[0] + pp[1];
          pf[sub][qb][i] = pb[0];
          pf[sub][qb][i + 1] = pb[1];
        }
      l_run[qb] += rs;
    }
#pragma unroll
    for (int sub = 0; sub < 2; ++sub)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const unsigned char* src = vbase + sub * 16 * ROW_BYTES + v_off[db];
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src + 8 * ROW_BYTES));
        const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 a = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[sub][qb], o[db][qb], 0, 0, 0);
      }
  };

  // ---- the steady-state step of the pipeline, in explicit issue order ----
  // Matrix pipe: S_next = K Q^T of the next block (KS slots of one K fragment
  // and QB MFMAs each), then O += P V of the current block (2 DB slots of one
  // V^T fragment and QB MFMAs each).  Vector pipe, in the shadow of the MFMAs:
  // P = exp2(S_cur c - m c) pair by pair in the order the second product
  // consumes it (the bf16 packing one slot after the exponentials, so that it
  // never waits for the exp unit), the row sums, and the maximum of S_next.
  // LDS fragments are requested PF slots ahead of their use.
  //   kn_buf/kn_blk: K buffer and block of the next block; v_buf/v_blk: V of the current one.
  auto fused = [&](auto kn_buf_tag, auto kn_blk_tag, auto v_buf_tag, auto v_blk_tag,
                   const f32x16 (&s_cur)[QB], f32x16 (&s_next)[QB], float (&mx_out)[QB]) {
    const unsigned char* kbase =
        sK + decltype(kn_buf_tag)::value * TILE_BYTES + decltype(kn_blk_tag)::value * 32 * ROW_BYTES;
    const unsigned char* vbase =
        sV + decltype(v_buf_tag)::value * TILE_BYTES + decltype(v_blk_tag)::value * 32 * ROW_BYTES;
    constexpr int NQ = KS, NP = 2 * DB;
    constexpr int PFK = NQ < 4 ? NQ : 4, PFV = NP < 4 ? NP : 4;
    constexpr int PAIRS = 2 * 4 * QB;                       // pairs of P elements per lane
    constexpr int PQ = (PAIRS + NQ - 1) / NQ;               // pairs exponentiated per QK slot
    constexpr int NMAX = 8 * QB;                            // max steps for S_next
    constexpr int MP = (NMAX + NP - 1) / NP;                // per PV slot
    constexpr int SP = (PAIRS + NP - 1) / NP;               // row-sum steps per PV slot
    static_assert(NQ * PQ >= PAIRS, "all of P is exponentiated under the first product");
    bf16x8 kfr[NQ], vfr[NP];
    bf16x8 pf[2][QB];
    float e0[PAIRS], e1[PAIRS];
    float rs[QB], mxa[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      rs[qb] = 0.f;
      mxa[qb] = kNegInf;
    }
    auto read_k = [&](const int slot) {
#ifdef SVD_PROBE_NOLDS
      kfr[slot] = qf[0][slot];
#else
      kfr[slot] = *reinterpret_cast<const bf16x8*>(kbase + k_off[slot]);
#endif
    };
    auto read_v = [&](const int slot) {
      const int sub = slot / DB, db = slot % DB;
#ifdef SVD_PROBE_NOLDS
      vfr[slot] = qf[0][(sub + db) % KS];
#else
      const unsigned char* src = vbase + sub * 16 * ROW_BYTES + v_off[db];
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(src + 8 * ROW_BYTES));
      const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      vfr[slot] = __builtin_bit_cast(bf16x8, both);
#endif
    };
    // pair n in consumption order: sub = n / (4 QB), then qb, then i
    auto expo = [&](const int n) {
      const int sub = n / (4 * QB), qb = (n / 4) % QB, i = (n % 4) * 2;
#ifdef SVD_PROBE_NOVALU
      e0[n] = s_cur[qb][sub * 8 + i];
      e1[n] = s_cur[qb][sub * 8 + i + 1];
#else
      e0[n] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[qb][sub * 8 + i], c_scale, -mc[qb]));
      e1[n] = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[qb][sub * 8 + i + 1], c_scale, -mc[qb]));
#endif
    };
    auto pack = [&](const int n) {
      const int sub = n / (4 * QB), qb = (n / 4) % QB, i = (n % 4) * 2;
#ifdef SVD_PROBE_NOVALU
      const unsigned raw = __builtin_bit_cast(unsigned, e0[n]) ^ __builtin_bit_cast(unsigned, e1[n]);
      const bf16x2 pb = __builtin_bit_cast(bf16x2, raw);
#else
      const f32x2 pp = {e0[n], e1[n]};
      const bf16x2 pb = __builtin_convertvector(pp, bf16x2);
#endif
      pf[sub][qb][i] = pb[0];
      pf[sub][qb][i + 1] = pb[1];
    };
    // row sums with plain adds, under the second product (the dot instructions
    // run on the matrix pipe and would serialise with the MFMAs)
    auto sum_pair = [&](const int n) {
      const int qb = (n / 4) % QB;
#ifndef SVD_PROBE_NOVALU
      rs[qb] += e0[n] + e1[n];
#endif
    };
    auto do_max = [&](const int n) {   // elements 2n, 2n+1 of S_next[qb]
      const int qb = n / 8, i = (n % 8) * 2;
#ifndef SVD_PROBE_NOVALU
      mxa[qb] = fmaxf(mxa[qb], fmaxf(s_next[qb][i], s_next[qb][i + 1]));
#else
      if (n % 8 == 0) mxa[qb] = s_next[qb][i];
#endif
    };
    auto pairs_before = [&](const int k) -> int {   // pairs exponentiated before slot k
      if (k <= 0) return 0;
      return k * PQ < PAIRS ? k * PQ : PAIRS;
    };
    // The row-sum and maximum chains feed nothing inside the block, so the
    // compiler would sink them below the MFMAs they are meant to hide behind; an
    // empty volatile asm per slot keeps each step in its slot.
    auto anchor = [&]() {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) asm volatile("" : "+v"(rs[qb]), "+v"(mxa[qb]));
    };

#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) s_next[qb][i] = 0.f;
#pragma unroll
    for (int f = 0; f < PFK; ++f) read_k(f);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int slot = 0; slot < NQ; ++slot) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        s_next[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[slot], qf[qb][slot], s_next[qb], 0, 0, 0);
      if (slot + PFK < NQ) read_k(slot + PFK);
      else if (slot + PFK - NQ < PFV) read_v(slot + PFK - NQ);
#pragma unroll
      for (int n = pairs_before(slot - 1); n < pairs_before(slot); ++n) pack(n);
#pragma unroll
      for (int n = pairs_before(slot); n < pairs_before(slot + 1); ++n) expo(n);
      anchor();
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int n = pairs_before(NQ - 1); n < PAIRS; ++n) pack(n);
#pragma unroll
    for (int slot = 0; slot < NP; ++slot) {
      const int sub = slot / DB, db = slot % DB;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[slot], pf[sub][qb], o[db][qb], 0, 0, 0);
      if (slot + PFV < NP) read_v(slot + PFV);
#pragma unroll
      for (int n = slot * MP; n < (slot + 1) * MP && n < NMAX; ++n) do_max(n);
#pragma unroll
      for (int n = slot * SP; n < (slot + 1) * SP && n < PAIRS; ++n) sum_pair(n);
      anchor();
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      l_run[qb] += rs[qb];
      mx_out[qb] = half_max(mxa[qb]);
    }
  };

  // does tile t need element masks?  band lists say so per entry; the dense and
  // gather loops can only meet a partly valid tile at the very end
  const bool tail_ragged = MODE == MODE_DENSE ? (L % BC != 0) : (n_cols % BC != 0);
  auto needs_mask = [&](const int t) -> bool {
    if (MODE == MODE_BAND) return !(entries[t].y & 1);
    return tail_ragged && t == n_tiles - 1;
  };

  // ---- prologue: K(0), V(0), K(1) into LDS, scores of block 0 ----
  static_assert(KB2 % 2 == 0, "an even number of 32-key blocks per tile keeps the score registers static");
  f32x16 s_a[QB], s_b[QB];
  float mx[QB];
  if (n_tiles > 0) {
    SVD_LOAD(kreg, K, 0);
    SVD_LOAD(vreg, V, 0);
    SVD_STORE(kreg, sK, st_off_k, 0);
    SVD_STORE(vreg, sV, st_off_v, 0);
    if (n_tiles > 1) {
      SVD_LOAD(kreg, K, 1);
      SVD_STORE(kreg, sK, st_off_k, 1);
    }
  }
  __syncthreads();
  if (n_tiles > 0) {
    scores(0, 0, s_a);
    if (needs_mask(0)) apply_mask(s_a, 0, 0);
    block_max(s_a, mx);
    raise_max(mx);
  }

  // After the fused step of block (t, kb2): mask and reference maximum of the
  // block whose scores it produced.
  auto settle = [&](f32x16 (&s_next)[QB], const int t_next, const int kb2_next) {
#ifdef SVD_PROBE_NOSETTLE
    return;
#endif
    if (needs_mask(t_next)) {
      asm volatile("" ::: "memory");   // keeps this a branch (the selects must not run on full tiles)
      apply_mask(s_next, t_next, kb2_next);
      block_max(s_next, mx);
    }
    raise_max(mx);
  };

  // One key tile: KB2 pipeline steps.  On entry s_a holds the settled scores of
  // block 0 of tile t; LDS holds K(t), V(t) in buffers t & 1 and K(t+1) in K
  // buffer (t+1) & 1.  K(t+2) and V(t+1) travel global -> registers -> LDS
  // meanwhile.  LAST: tile t is the last one (its last block has no successor).
  auto tile_steps = [&](auto par_tag, auto last_tag, const int t) {
    constexpr int PAR = decltype(par_tag)::value;     // t & 1
    constexpr bool LAST = decltype(last_tag)::value != 0;
#ifdef SVD_PROBE_NOLOAD
    const bool has2 = false, has1 = false;
#else
    const bool has2 = t + 2 < n_tiles, has1 = !LAST;
#endif
    if (has2) SVD_LOAD(kreg, K, t + 2);
    if (has1) SVD_LOAD(vreg, V, t + 1);
#define SVD_STEP(KB, CUR, NXT)                                                              \
    if (KB + 1 < KB2) {                                                                     \
      fused(Int<PAR>{}, Int<(KB + 1) % KB2>{}, Int<PAR>{}, Int<KB>{}, CUR, NXT, mx);        \
      settle(NXT, t, KB + 1);                                                               \
    } else if (!LAST) {                                                                     \
      fused(Int<PAR ^ 1>{}, Int<0>{}, Int<PAR>{}, Int<KB>{}, CUR, NXT, mx);                 \
      settle(NXT, t + 1, 0);                                                                \
    } else {                                                                                \
      finish_block(PAR, KB, CUR);                                                           \
    }
    SVD_STEP(0, s_a, s_b)
    SVD_STEP(1, s_b, s_a)
    if (KB2 > 2) {
      SVD_STEP(2, s_a, s_b)
      SVD_STEP(3, s_b, s_a)
    }
#undef SVD_STEP
    // K(t) (this tile's own K buffer) was still being read by the steps above:
    // every wave must be past them before K(t+2) may overwrite it
#ifndef SVD_PROBE_NOBAR
    if (has2) __syncthreads();
#endif
    if (has2) SVD_STORE(kreg, sK, st_off_k, PAR);
    if (has1) SVD_STORE(vreg, sV, st_off_v, PAR ^ 1);
#ifndef SVD_PROBE_NOBAR
    __syncthreads();
#endif
  };

  // two tiles per trip keep the buffer indices static
  int t = 0;
  for (; t + 2 < n_tiles; t += 2) {
    tile_steps(Int<0>{}, Int<0>{}, t);
    tile_steps(Int<1>{}, Int<0>{}, t + 1);
  }
  if (t + 1 < n_tiles) {
    tile_steps(Int<0>{}, Int<0>{}, t);
    tile_steps(Int<1>{}, Int<1>{}, t + 1);
  } else if (t < n_tiles) {
    tile_steps(Int<0>{}, Int<1>{}, t);
  }

  // ---- epilogue: O = O^T / l, bf16, lane owns query l32: 4 consecutive d per store ----
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = half_sum(l_run[qb]);
    const float inv = 1.0f / l_tot;
    const int row = q0 + qb * 32 + l32;
    if (row < L) {
      __bf16* dst = O + (int64_t)row * p.stride_l;
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

#undef SVD_LOAD
#undef SVD_STORE

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
    default:
      return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

void kernel_blocks(int D, int* block_q, int* block_k) {
  if (D == 128) {
    *block_q = Tile128::NW * Tile128::QB * 32;
    *block_k = Tile128::BC;
  } else {
    *block_q = Tile64::NW * Tile64::QB * 32;
    *block_k = Tile64::BC;
  }
}

hipError_t launch_attention(const AttnLaunch& p, int mode, hipStream_t stream) {
  if (p.n_items <= 0) return hipSuccess;
  if (p.D == 128)
    return launch_mode<128, Tile128::NW, Tile128::QB, Tile128::BC, Tile128::OCC>(p, mode, stream);
  if (p.D == 64) return launch_mode<64, Tile64::NW, Tile64::QB, Tile64::BC, Tile64::OCC>(p, mode, stream);
  return hipErrorInvalidValue;
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
