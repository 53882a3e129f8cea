// fs_prefill_attention: chunked-prefill attention over the paged KVCache, gfx950 only.
//
// The paper's fine-grained chunked prefill (Section 3.1) puts chunks of several requests into
// one batch: N new tokens of a request behind L processed ones.  Every new token attends to the
// cache up to and including itself (prefill phase, Section 2.1.1).  The paper describes no
// kernel; this one is built on the decode kernel's slot layout, which already stores K and V
// pages in matrix-core operand order.
//
// One workgroup per item: a tile of query tokens of one (request, KV head) pair against one
// split-K chunk of the keys the tile sees.  A query row is a (token, q-head of the group)
// combination; 16 rows form a column tile of the transposed score matrix and every wavefront
// owns CT column tiles.  The workgroup walks the chunk in pairs of KV pages (32 tokens):
//   * every wavefront fetches its share of the next pairs from global memory into registers (two
//     pairs in flight) and copies it into a double-buffered LDS stage, so the whole workgroup
//     reads each page from L2/HBM once;
//   * from LDS every wavefront takes the K operands (16-byte reads, conflict-free), and for each
//     of its column tiles
//         S^T[tok][row] = K . Q^T        2 x 4 v_mfma_f32_16x16x32_bf16
//     then the V operands and, per column tile, the online softmax (fp32, log2 domain, causal
//     mask only on the pairs that straddle a row's position) and
//         O^T[d][row]  += V^T . P^T      8 x v_mfma_f32_16x16x32_f16 over the 32 tokens: the weights as fp16,
//                                         V converted bf16 -> fp16 on its way into LDS (when the caller
//                                         states FS_V_FP16_RANGE; else V as bf16 and the weights as bf16 hi + lo).
// The S^T accumulators of the two pages are, lane by lane, the 8 reduction elements the second
// product wants from P^T (4 tokens of the first page, the same 4 of the second); the copy into
// LDS pairs the V rows of the two pages the same way, so nothing crosses lanes except the
// running max.  This is a dense contraction (G*N rows against L+N keys): the matrix cores bound
// it, not HBM.  fp8 K/V takes the same walk; only the copy into LDS differs (see prefill_tile).
#include <hip/hip_runtime.h>

#include <cmath>

#include "fs_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

struct PrefillParams {
  const uint16_t* __restrict__ q;
  const char* __restrict__ k_pool;
  const char* __restrict__ v_pool;
  int64_t k_stride;
  int64_t v_stride;
  const float* __restrict__ k_scale;      // fp8: by slot, or (page_scales given) the (K, V) pairs in page-table order
  const float* __restrict__ v_scale;      //      by slot, or page_scales + 1
  int32_t scale_by_page;                  // 1: scale of page i of the table sits at k_scale[2i] / v_scale[2i]
  const int64_t* __restrict__ page_indptr;
  const int32_t* __restrict__ page_ids;
  const fs_prefill_item* __restrict__ items;
  const int32_t* __restrict__ sched;
  float* __restrict__ part_o;
  float* __restrict__ part_lse;
  // One-call form only (else NULL): an item that is all of its tile writes the tile's final rows,
  // out_indptr[pair] + token*G + g, and needs no merge.
  const int64_t* __restrict__ out_indptr;
  float* __restrict__ out;
  float* __restrict__ lse;
  int32_t group;        // G
  int32_t group_pad;    // G rounded up to a power of two (divides 16)
  int32_t n_q_heads;
  int32_t tile_tokens;  // query tokens per tile as the list was built (rows per item = tile_tokens * G)
  float scale_log2;
};

constexpr float kLn2 = 0.6931471805599453f;
constexpr int kStageBytes = 16384;     // one pair of pages: K0, K1 (4 KiB each), then the paired V halves (2 x 4 KiB)
constexpr int kVaOffset = 8192;        // V rows d = 32c + lane%16:      (page 0 tokens 4kb..+3 | page 1 tokens 4kb..+3)
constexpr int kVbOffset = 12288;       // V rows d = 32c + 16 + lane%16: likewise

// A wavefront's share of one page pair on its way from global memory to LDS: NP (K block, V block)
// couples of 1 KiB, each couple from one page h and one 32-d block c.
// fp8 K/V: the same couples are 512 bytes each (8 bytes per lane) and carry the page's V scale.
template <int NP, bool FP8>
struct InFlight {
  u32x4 k[NP];
  u32x4 v[NP];
};
template <int NP>
struct InFlight<NP, true> {
  uint2 k[NP];
  uint2 v[NP];
  float vs[NP];
};

// max of three / of two as IEEE-754 maximum (v_maximum3_f32): no NaN-quieting moves around it, unlike fmaxf,
// and, being an instruction the compiler knows, it gets the wait states that a read of a matrix-core result
// needs.  (An asm statement does not: the compiler cannot see that it reads registers a matrix instruction has
// just written, and the hardware does not interlock, so it would read what the registers held before.)
// The inputs are matrix-core outputs or -inf; a NaN can only come from a row that is never stored.
__device__ __forceinline__ float max3(float a, float b, float c) {
  return __builtin_elementwise_maximum(__builtin_elementwise_maximum(a, b), c);
}

__device__ __forceinline__ float max2(float a, float b) { return __builtin_elementwise_maximum(a, b); }
// x *= a in place.  As asm with a tied operand so that, inside a rarely taken branch, the accumulators
// stay in their registers (with a plain multiply the compiler copies all of them on every step instead).
// The compiler does not see that these statements read and write registers of matrix instructions, so the
// branch that holds them opens and closes with the wait states itself (FS_MATRIX_RESULT_WAIT).
#define FS_MATRIX_RESULT_WAIT() asm volatile("s_nop 7\n\ts_nop 4" ::: "memory")   // 13 wait states: above the 12 of an 8-pass result
#define FS_SCALE_IN_PLACE(vec, k, a)                                  \
  do {                                                                \
    float t_ = (vec)[k];                                              \
    asm volatile("v_mul_f32 %0, %0, %1" : "+v"(t_) : "v"(a));         \
    (vec)[k] = t_;                                                    \
  } while (0)

struct TileState {
  float m;          // reference max (log2 domain) of this lane's query row: within 2^8 below the true running max
  float neg_ref;    // -m, or -0 while the row has seen no key (m = -inf)
  f32x4 l;          // running sum of the row's weights, element 0 (kept on the matrix cores: a row of ones above V^T)
  f32x4 acc[8];     // O^T[d = 16b + 4*(lane/16) + r][row = lane%16]
};

constexpr float kLazy = 8.0f;   // the reference max follows the running max only when it falls 2^8 behind

// Online softmax of one column tile over one page pair and its share of O^T += V^T . P^T.
// sa/sb: raw scores of the tile against the two pages (this lane: tokens t0 + 4kb + r and
// t0 + 16 + 4kb + r).  mask: some of the 32 tokens lie beyond some row's position `pos`.
// WIDE = false: the weights and the V operands enter the second product as fp16 (V is converted on its
// way into LDS, exactly for magnitudes from 2^-14 to 65504; smaller ones land on fp16's subnormal grid,
// larger ones enter as +-65504).  WIDE = true: V stays bf16 and the weights go in as bf16 hi + lo, two
// products, for caches whose values leave fp16's range.
// TWO_SCALES (fp8 K): the scores of the second page take scale_b (softmax scale times that page's K scale, both
// positive) and those of the first scale_log2 (likewise); else one scale for both.
// With both WIDE and TWO_SCALES (fp8 V kept as its exact codes in bf16) the weights of the two pages are multiplied by
// the pages' V scales vs_a, vs_b before they are split, and the row sum is taken on the vector units from the
// unscaled weights, each lane its own 8 tokens (st.l[0] is then a partial sum: see the kernel's last step).
template <bool WIDE, bool TWO_SCALES>
__device__ __forceinline__ void softmax_pv(TileState& st, const f32x4 sa, const f32x4 sb, const u32x4 (&va)[4],
                                           const u32x4 (&vb)[4], float scale_log2, float scale_b, float vs_a, float vs_b,
                                           int t0, int pos, int kb, bool mask) {
  // no fused multiply-add on the wide path: there a row's top key must get exp2(0) = 1 exactly, which needs
  // the scaled score rounded the same way on both sides of the subtraction
#pragma clang fp contract(off)
  f32x8 s = {sa[0], sa[1], sa[2], sa[3], sb[0], sb[1], sb[2], sb[3]};
  if (mask) {   // wave-uniform; kept a real branch (the empty asm stops the compiler from turning it into 16 selects on every step)
    asm volatile("");
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (t0 + 4 * kb + r > pos) s[r] = -INFINITY;
      if (t0 + 16 + 4 * kb + r > pos) s[4 + r] = -INFINITY;
    }
  }
  // Lazy reference max: the exponentials are taken against st.m, which moves up to the row's max only
  // when that lies more than 2^8 above it (always on a row's first visible keys, where st.m is -inf, so
  // a row's first top key still gets exactly 1; rarely afterwards).  Weights stay below 2^8, which costs
  // fp32 sums and 16-bit weights no precision, and the rescale multiplies leave the common path.  The
  // common path does not even form the row's max: every lane checks its own 8 scores (the softmax scale
  // is positive, so the max of the raw scores is the max of the scaled ones), and only if some lane of the
  // wavefront is out of range are the four lanes of each row combined.
  // (TWO_SCALES: the lane's maximum is formed on scaled scores, one product per page, and `post` is 1)
  const float mx_lane = TWO_SCALES ? max2(max2(max3(s[0], s[1], s[2]), s[3]) * scale_log2, max2(max3(s[4], s[5], s[6]), s[7]) * scale_b)
                                   : max3(max3(s[0], s[1], s[2]), max3(s[3], s[4], s[5]), max2(s[6], s[7]));
  const float post = TWO_SCALES ? 1.0f : scale_log2;
  if (__any(mx_lane * post > st.m + kLazy)) {
    float mx = mx_lane;
    const unsigned u = __float_as_uint(mx);
    const auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned a = r16[0], b = r16[1];
    mx = max2(__uint_as_float(a), __uint_as_float(b));
    const unsigned v = __float_as_uint(mx);
    const auto r32 = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    const unsigned c = r32[0], d = r32[1];
    mx = max2(__uint_as_float(c), __uint_as_float(d)) * post;
    const bool move = mx > st.m + kLazy;
    const float alpha = move ? __builtin_amdgcn_exp2f(st.m - mx) : 1.0f;   // st.m = -inf: exp2(-inf) = 0
    FS_MATRIX_RESULT_WAIT();
    FS_SCALE_IN_PLACE(st.l, 0, alpha);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      FS_SCALE_IN_PLACE(st.acc[j], 0, alpha);
      FS_SCALE_IN_PLACE(st.acc[j], 1, alpha);
      FS_SCALE_IN_PLACE(st.acc[j], 2, alpha);
      FS_SCALE_IN_PLACE(st.acc[j], 3, alpha);
    }
    FS_MATRIX_RESULT_WAIT();
    st.m = move ? mx : st.m;
    // A row may have seen none of the item's keys so far (its position lies before the chunk): its
    // state stays at zero and its reference is 0.
    st.neg_ref = st.m == -INFINITY ? -0.f : -st.m;
  }
  const float m_ref = -st.neg_ref;
  f32x8 p;
  if constexpr (!WIDE) {
    // One fused multiply-add per score: the top key's weight may miss 1 by an ulp of fp32, which the
    // rounding to fp16 below takes back, so a row's first key still weighs exactly 1.
#pragma unroll
    for (int r = 0; r < 8; ++r) p[r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], (TWO_SCALES && r >= 4) ? scale_b : scale_log2, st.neg_ref));
    const f16x8 ph = __builtin_convertvector(p, f16x8);          // weights are below 2^8: no overflow
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const f16x8 a = __builtin_bit_cast(f16x8, va[c]), b = __builtin_bit_cast(f16x8, vb[c]);
      st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, ph, st.acc[2 * c], 0, 0, 0);
      st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(b, ph, st.acc[2 * c + 1], 0, 0, 0);
    }
    // the row sums: a row of ones in place of V^T leaves sum_t p_t in every element of the result column
    const u32x4 ones_bits = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
    st.l = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, ones_bits), ph, st.l, 0, 0, 0);
  } else {
#pragma unroll
    for (int r = 0; r < 8; ++r) p[r] = __builtin_amdgcn_exp2f(s[r] * ((TWO_SCALES && r >= 4) ? scale_b : scale_log2) - m_ref);   // product rounded first: the row's top key gets exactly 1
    // Weights as bf16 hi + lo (16 significant bits).  hi is p cut to its upper 16 bits (one byte
    // permute packs two of them), lo = p - hi is exact in fp32 and is rounded to bf16.
    if constexpr (TWO_SCALES) {
      st.l[0] += ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
#pragma unroll
      for (int r = 0; r < 8; ++r) p[r] *= r < 4 ? vs_a : vs_b;
    }
    u32x4 hi_packed;
    f32x8 lo;
#pragma unroll
    for (int r = 0; r < 8; r += 2) {
      const uint32_t b0 = __float_as_uint(p[r]), b1 = __float_as_uint(p[r + 1]);
      hi_packed[r / 2] = __builtin_amdgcn_perm(b1, b0, 0x07060302u);     // (b1 & 0xFFFF0000) | (b0 >> 16)
      lo[r] = p[r] - __uint_as_float(b0 & 0xFFFF0000u);
      lo[r + 1] = p[r + 1] - __uint_as_float(b1 & 0xFFFF0000u);
    }
    const bf16x8 ph = __builtin_bit_cast(bf16x8, hi_packed);
    const bf16x8 pl = __builtin_convertvector(lo, bf16x8);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, va[c]), b = __builtin_bit_cast(bf16x8, vb[c]);
      st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, ph, st.acc[2 * c], 0, 0, 0);
      st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, ph, st.acc[2 * c + 1], 0, 0, 0);
      st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pl, st.acc[2 * c], 0, 0, 0);
      st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b, pl, st.acc[2 * c + 1], 0, 0, 0);
    }
    // the row sums: a row of ones in place of V^T leaves sum_t p_t in every element of the result column
    if constexpr (!TWO_SCALES) {
      const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
      const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
      st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, ph, st.l, 0, 0, 0);
      st.l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pl, st.l, 0, 0, 0);
    }
  }
}

// One 4 KiB slot of a pool as a raw buffer resource (base in scalar registers).
template <int BYTES = 4096>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t slot_buffer(const char* base) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(a >> 32));
  return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>((static_cast<uint64_t>(hi) << 32) | lo), 0, BYTES,
                                           0x00020000 /* raw 32-bit data format */);
}

// Two bf16 values (one 32-bit word) as two fp16 values, same order.  Round-toward-zero conversion: exact
// inside fp16's normal range, and a magnitude above 65504 becomes 65504, not infinity.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t w) {
  const float lo = __uint_as_float(w << 16), hi = __uint_as_float(w & 0xFFFF0000u);
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi));
}

// Eight e4m3 bytes to eight bf16, exactly (the conversion takes a power-of-two scale; 1.0 is 2^0).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x4 fp8x8_to_bf16x8(uint2 w) {
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, false), b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.x, 1.0f, true);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, false), d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w.y, 1.0f, true);
  return u32x4{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, c), __builtin_bit_cast(uint32_t, d)};
}

// The 8-wavefront, one-column-tile shape is held to 128 registers so that two workgroups (four
// wavefronts per SIMD) share a CU: the softmax is a long dependent chain and needs the company.
// FP8: e4m3 K/V (slots in 16-byte pieces per (token, 16 d), a scale per slot for K and for V).  Only the way into
// LDS differs: a lane fetches 8 bytes of K and 8 of V where the bf16 kernel fetches 16 and 16 (the same 8 d of the same
// token that its bf16 piece would hold), K is converted to bf16 (exact) and lands where the bf16 piece would; V must
// arrive as (one d, four tokens) and is transposed by the matrix cores on the way: its bytes are the A operand of an
// fp8 product with a constant matrix of ones and zeros, whose result - (token, d) in (d, four tokens) order - is
// scaled, rounded to fp16 (bf16 when WIDE) and stored where the bf16 kernel stores its converted V.  The K scales
// of the two pages join the softmax scale.
template <int WAVES, int CT, bool WIDE, bool FP8>
__device__ __forceinline__ void prefill_tile(const PrefillParams& P) {
  constexpr int NP = 8 / WAVES;        // (K, V) block couples a wavefront moves per page pair
  static_assert(NP >= 1, "at most 8 wavefronts");
  __shared__ __attribute__((aligned(16))) unsigned char stage[2][kStageBytes];

  const int item_idx = P.sched ? P.sched[blockIdx.x] : static_cast<int>(blockIdx.x);
  const fs_prefill_item it = P.items[item_idx];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, kb = lane >> 4;
  const int G = P.group, Gp = P.group_pad;
  const int tpc = 16 / Gp;                       // query tokens per column tile
  const int n_tok = it.q_end - it.q_begin;       // query tokens of this item
  const int tok0 = wave * CT * tpc;              // first token (within the item) of this wavefront
  const bool wave_live = tok0 < n_tok;           // a short last tile leaves some wavefronts without rows
  const int L0 = it.n_done + it.q_begin;         // position of the item's first token
  const int last_key = it.n_done + it.q_end - 1; // last key any row of the tile may see
  const int n_it = (it.kv_end - it.kv_begin + 31) / 32;       // page pairs of this item
  const int page_begin = it.kv_begin / fs::kPageTokens;
  const int page_end = (it.kv_end + fs::kPageTokens - 1) / fs::kPageTokens;
  // The page table is read through the constant address space: the kernel also stores to global memory, so
  // the compiler would otherwise fetch the ids with vector loads and do the slot arithmetic per lane.
  typedef const int32_t __attribute__((address_space(4))) * const_ids_ptr;
  const const_ids_ptr ids = (const_ids_ptr)(reinterpret_cast<uintptr_t>(P.page_ids + P.page_indptr[it.pair]));

  // this lane's row of each column tile
  const int g = col % Gp, tl = col / Gp;
  bf16x8 qreg[CT][4];
  int pos[CT];
  bool live[CT];
#pragma unroll
  for (int t = 0; t < CT; ++t) {
    const int tok = tok0 + t * tpc + tl;                  // within the item
    live[t] = tok < n_tok && g < G;
    pos[t] = min(L0 + tok, last_key);                     // rows that do not exist look at existing keys only
    const int64_t qrow = static_cast<int64_t>(it.q_row) + static_cast<int64_t>(min(tok, n_tok - 1)) * P.n_q_heads + min(g, G - 1);
    const u32x4* qp = reinterpret_cast<const u32x4*>(P.q + qrow * fs::kHeadDim) + kb;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 v = qp[4 * c];
      if (!live[t]) v = u32x4{0u, 0u, 0u, 0u};
      qreg[t][c] = __builtin_bit_cast(bf16x8, v);
    }
  }
  TileState st[CT];
#pragma unroll
  for (int t = 0; t < CT; ++t) {
    st[t].m = -INFINITY;
    st[t].neg_ref = -0.f;
    st[t].l = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 8; ++j) st[t].acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  // fp8: where a page's scales sit (by slot, or in page-table order), read through the constant address space
  typedef const float __attribute__((address_space(4))) * const_scale_ptr;
  const int64_t table0 = FP8 ? P.page_indptr[it.pair] : 0;
  // (two real branches: as a select, the page-table order would pay for the slot number's read as well)
  auto scale_of = [&](const float* scales, int page) __attribute__((always_inline)) -> float {
    const const_scale_ptr sc = (const_scale_ptr)(reinterpret_cast<uintptr_t>(scales));
    if (P.scale_by_page) return sc[2 * (table0 + page)];
    asm volatile("");
    return sc[ids[page]];
  };

  // ---- global -> registers: this wavefront's couples of pair jp ---------------------------------
  // fp8: the scales of the pair that is computed next (pair jc) are read here too, next to the page ids that this step
  // waits for anyway: read where they are used, their wait would fall between the LDS reads of the walk.
  float ks_a = 1.0f, ks_b = 1.0f, vs_a = 1.0f, vs_b = 1.0f;
  auto fetch = [&](InFlight<NP, FP8>& r, int jp, int jc) __attribute__((always_inline)) {
    if constexpr (FP8) {
      if (jc >= 0) {
        const int pa = min(page_begin + 2 * jc, page_end - 1), pb = min(page_begin + 2 * jc + 1, page_end - 1);
        ks_a = scale_of(P.k_scale, pa);
        ks_b = scale_of(P.k_scale, pb);
        if constexpr (WIDE) {
          vs_a = scale_of(P.v_scale, pa);
          vs_b = scale_of(P.v_scale, pb);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int idx = wave * NP + i, h = idx >> 2, c = idx & 3;
      // Always a load, beyond the item's last page that page again (its keys are masked by position and
      // its values blanked on the way into LDS): with the same number of loads in flight on every path
      // the wait before a copy into LDS leaves the younger loads in flight.
      const int page = min(page_begin + 2 * jp + h, page_end - 1);
      // a slot as a raw buffer: its base stays in scalar registers, the lane's place in it is one 32-bit
      // offset (64-bit vector addresses cost this kernel registers it does not have)
      const int64_t slot = ids[page];
      if constexpr (FP8) {
        // the 8 bytes d = 32c + 8kb .. + 8 of token lane%16: half (kb & 1) of piece [c/2][2(c&1) + kb/2][tok];
        // the wavefront's 64 lanes cover 512 contiguous bytes
        const int off = (c >> 1) * 1024 + (c & 1) * 512 + (kb >> 1) * 256 + col * 16 + (kb & 1) * 8;
        r.k[i] = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(slot_buffer<2048>(P.k_pool + slot * P.k_stride), off, 0, 0));
        r.v[i] = __builtin_bit_cast(uint2, __builtin_amdgcn_raw_buffer_load_b64(slot_buffer<2048>(P.v_pool + slot * P.v_stride), off, 0, 0));
        r.vs[i] = WIDE ? 1.0f : scale_of(P.v_scale, page);
      } else {
        r.k[i] = __builtin_amdgcn_raw_buffer_load_b128(slot_buffer(P.k_pool + slot * P.k_stride), (c * 64 + lane) * 16, 0, 0);
        r.v[i] = __builtin_amdgcn_raw_buffer_load_b128(slot_buffer(P.v_pool + slot * P.v_stride), (c * 64 + lane) * 16, 0, 0);
      }
    }
  };
  // ---- registers -> LDS stage s ------------------------------------------------------------------
  auto deposit = [&](int s, const InFlight<NP, FP8>& r, int jp) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int idx = wave * NP + i, h = idx >> 2, c = idx & 3;
      unsigned char* base = stage[s];
      // value rows of tokens at or beyond the item's end may hold anything (the unused tail of a last
      // page is never initialised): blank them, 0 * NaN would be NaN in the product
      const int valid = it.kv_end - (page_begin + 2 * jp + h) * fs::kPageTokens;    // tokens of this page inside the item
      const bool blank = valid < fs::kPageTokens;          // same for the whole wavefront: only an item's last page
      auto mask01 = [&]() __attribute__((always_inline)) {   // which of this lane's four tokens (4kb .. 4kb+3, two to a word) exist
        return make_uint2((4 * kb + 0 < valid ? 0x0000FFFFu : 0u) | (4 * kb + 1 < valid ? 0xFFFF0000u : 0u),
                          (4 * kb + 2 < valid ? 0x0000FFFFu : 0u) | (4 * kb + 3 < valid ? 0xFFFF0000u : 0u));
      };
      if constexpr (FP8) {
        *reinterpret_cast<u32x4*>(base + ((h * 4 + c) * 64 + lane) * 16) = fp8x8_to_bf16x8(r.k[i]);
        // E[k][n] for the two halves of the 32-d block: column n = lane%16 takes k = 16h2 + n, which sits in the
        // lanes with kb = 2h2 + n/8 as byte n%8 (0x38 is 1.0 in e4m3)
        const long bytes = static_cast<long>((static_cast<unsigned long>(r.v[i].y) << 32) | r.v[i].x);
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const long pick = (kb == 2 * h2 + (col >> 3)) ? static_cast<long>(0x38ul << (8 * (col & 7))) : 0l;
          f32x4 t = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(bytes, pick, z, 0, 0, 0);
          uint2 v;     // lane (d = 32c + 16h2 + lane%16): tokens 4kb .. 4kb+3 of page h
          if constexpr (WIDE) {     // the codes as they are (every e4m3 value is a bf16 value); the scale goes to the weights
            v = make_uint2(__builtin_amdgcn_perm(__float_as_uint(t[1]), __float_as_uint(t[0]), 0x07060302u),
                           __builtin_amdgcn_perm(__float_as_uint(t[3]), __float_as_uint(t[2]), 0x07060302u));
          } else {     // times the page's scale, rounded toward zero: a magnitude above 65504 becomes 65504, not infinity
            t *= r.vs[i];
            v = make_uint2(__builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(t[0], t[1])),
                           __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(t[2], t[3])));
          }
          if (blank) {
            asm volatile("");      // a real branch: as selects the masks cost every step 16 instructions
            const uint2 m = mask01();
            v = make_uint2(v.x & m.x, v.y & m.y);
          }
          *reinterpret_cast<uint2*>(base + (h2 ? kVbOffset : kVaOffset) + (c * 64 + lane) * 16 + 8 * h) = v;
        }
      } else {
        *reinterpret_cast<u32x4*>(base + ((h * 4 + c) * 64 + lane) * 16) = r.k[i];
        u32x4 v = r.v[i];
        if constexpr (!WIDE) v = u32x4{bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w)};
        if (blank) {
          const uint2 m = mask01();
          v = u32x4{v.x & m.x, v.y & m.y, v.z & m.x, v.w & m.y};
        }
        *reinterpret_cast<uint2*>(base + kVaOffset + (c * 64 + lane) * 16 + 8 * h) = make_uint2(v.x, v.y);
        *reinterpret_cast<uint2*>(base + kVbOffset + (c * 64 + lane) * 16 + 8 * h) = make_uint2(v.z, v.w);
      }
    }
  };
  // ---- one page pair from LDS stage s against this wavefront's column tiles -----------------------
  auto compute = [&](int s, int jp) __attribute__((always_inline)) {
    if (!wave_live) return;
    const int t0 = it.kv_begin + 32 * jp;                 // first token of the pair
    bool need[CT], full[CT];
    bool any = false;
#pragma unroll
    for (int t = 0; t < CT; ++t) {
      const int first_pos = L0 + tok0 + t * tpc;                              // smallest position in the column tile
      const int last_pos = min(L0 + tok0 + t * tpc + tpc - 1, last_key);      // largest
      need[t] = tok0 + t * tpc < n_tok && t0 <= last_pos;
      full[t] = t0 + 31 <= first_pos;                                         // every row sees all 32 tokens
      any |= need[t];
    }
    if (!any) return;
    const unsigned char* base = stage[s];
    const float scale_a = P.scale_log2 * ks_a, scale_b = P.scale_log2 * ks_b;     // fp8: the two pages' K scales join the softmax scale
    f32x4 sa[CT], sb[CT];
    const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
    {
      u32x4 k0[4], k1[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        k0[c] = *reinterpret_cast<const u32x4*>(base + (c * 64 + lane) * 16);
        k1[c] = *reinterpret_cast<const u32x4*>(base + ((4 + c) * 64 + lane) * 16);
      }
#pragma unroll
      for (int t = 0; t < CT; ++t) {
        if (need[t]) {
          sa[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k0[0]), qreg[t][0], zero4, 0, 0, 0);
          sb[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k1[0]), qreg[t][0], zero4, 0, 0, 0);
#pragma unroll
          for (int c = 1; c < 4; ++c) {
            sa[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k0[c]), qreg[t][c], sa[t], 0, 0, 0);
            sb[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k1[c]), qreg[t][c], sb[t], 0, 0, 0);
          }
        }
      }
    }
    u32x4 va[4], vb[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      va[c] = *reinterpret_cast<const u32x4*>(base + kVaOffset + (c * 64 + lane) * 16);
      vb[c] = *reinterpret_cast<const u32x4*>(base + kVbOffset + (c * 64 + lane) * 16);
    }
#pragma unroll
    for (int t = 0; t < CT; ++t) {
      if (need[t]) softmax_pv<WIDE, FP8>(st[t], sa[t], sb[t], va, vb, scale_a, scale_b, vs_a, vs_b, t0, pos[t], kb, !full[t]);
    }
  };

  // ---- the walk: pair j is computed from stage j%2 while pair j+1 is copied into the other stage and
  // pairs j+2, j+3 are on their way from global memory.  One barrier per pair: after it, stage (j+1)%2 is
  // complete and nobody reads stage j%2 any more.  Every wavefront takes every branch below (n_it is the
  // workgroup's), so the barriers match.
  if (n_it < 1) return;        // not produced by the list builder (an item sees at least one key)
  InFlight<NP, FP8> r0, r1;
  fetch(r0, 0, -1);
  fetch(r1, 1, -1);
  deposit(0, r0, 0);
  fetch(r0, 2, -1);
  __syncthreads();
  for (int j = 0; j < n_it; j += 2) {
    // Copies and fetches run for pairs beyond the item's end too (into a stage nobody reads, from the last
    // page again): one shape of loop body, so every wait for a copy's data leaves exactly the two younger
    // loads in flight.
    deposit(1, r1, j + 1);
    fetch(r1, j + 3, j);
    compute(0, j);
    __syncthreads();
    deposit(0, r0, j + 2);
    fetch(r0, j + 4, j + 1);
    if (j + 1 < n_it) compute(1, j + 1);
    __syncthreads();
  }

  // ---- write the item's rows: partial rows, or the tile's final rows when the item is all of its tile ----
  // (an item that starts at key 0 and ends at the last key its tile may see is the tile's only chunk)
  const bool direct = P.out_indptr != nullptr && it.kv_begin == 0 && it.kv_end == it.n_done + it.q_end;
  float* const dst_o = direct ? P.out : P.part_o;
  float* const dst_lse = direct ? P.lse : P.part_lse;
  const int64_t row0 = direct ? P.out_indptr[it.pair] + static_cast<int64_t>(it.q_begin) * G : static_cast<int64_t>(it.part_row);
  // The lane's place is worked out again, from the lane counter: values derived from threadIdx before the walk
  // would be kept alive across it, in registers the walk does not have (they went to scratch memory).
  const int lane_w = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  const int col_w = lane_w & 15, kb_w = lane_w >> 4;
  const int g_w = col_w % Gp, tl_w = col_w / Gp;
#pragma unroll
  for (int t = 0; t < CT; ++t) {
    const int tok = tok0 + t * tpc + tl_w;
    float l_tot = st[t].l[0];
    if constexpr (WIDE && FP8) {      // partial sums of the four lanes that share the row (softmax_pv)
      const unsigned u = __float_as_uint(l_tot);
      const auto r16 = __builtin_amdgcn_permlane16_swap(u, u, false, false);
      const unsigned a16 = r16[0], b16 = r16[1];
      l_tot = __uint_as_float(a16) + __uint_as_float(b16);
      const unsigned v = __float_as_uint(l_tot);
      const auto r32 = __builtin_amdgcn_permlane32_swap(v, v, false, false);
      const unsigned a32 = r32[0], b32 = r32[1];
      l_tot = __uint_as_float(a32) + __uint_as_float(b32);
    }
    if (g_w >= G || tok >= P.tile_tokens) continue;          // no such row in the buffers
    const int64_t row = row0 + static_cast<int64_t>(tok) * G + g_w;
    float* o = dst_o + row * fs::kHeadDim + 4 * kb_w;
    if (tok < n_tok) {
      const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;  // a row that saw none of the item's keys: out = 0, lse = -inf
#pragma unroll
      for (int b = 0; b < 8; ++b) *reinterpret_cast<f32x4*>(o + 16 * b) = st[t].acc[b] * inv;
      if (kb_w == 0) dst_lse[row] = l_tot > 0.f ? (st[t].m + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
    } else {                                               // padding row of a short last tile
#pragma unroll
      for (int b = 0; b < 8; ++b) *reinterpret_cast<f32x4*>(o + 16 * b) = f32x4{0.f, 0.f, 0.f, 0.f};
      if (kb_w == 0) dst_lse[row] = 0.f;
    }
  }
}

#define FS_PREFILL_BOUNDS(W, C) __launch_bounds__(W * 64, (W == 8 && C == 1) ? 4 : (W == 4 && C == 2) ? 2 : (W == 4 && C == 1) ? 3 : 1)
template <int WAVES, int CT, bool WIDE>
__global__ void FS_PREFILL_BOUNDS(WAVES, CT) prefill_bf16_kernel(const PrefillParams P) {
  prefill_tile<WAVES, CT, WIDE, false>(P);
}
template <int WAVES, int CT, bool WIDE>
__global__ void FS_PREFILL_BOUNDS(WAVES, CT) prefill_fp8_kernel(const PrefillParams P) {
  prefill_tile<WAVES, CT, WIDE, true>(P);
}
#undef FS_PREFILL_BOUNDS

template <typename K>
fs_status launch(K kernel, int threads, const PrefillParams& P, int64_t n_items, hipStream_t stream) {
  hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(n_items)), dim3(threads), 0, stream, P);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fs::fail(FS_EHIP, "fs_prefill_attention: launch failed: %s", hipGetErrorString(e));
  return FS_OK;
}

int pad_group(int G) {
  int p = 1;
  while (p < G) p <<= 1;
  return p;
}

}  // namespace

extern "C" int32_t fs_prefill_tile_tokens(int32_t group) {
  if (group < 1 || group > fs::kMaxGroup) return -1;
  return fs::options().prefill_waves * fs::options().prefill_col_tiles * (16 / pad_group(group));
}

namespace {

// Argument checks and launch shared by the two entry points.  direct_* non-NULL: single-chunk tiles write final rows.
fs_status prefill_launch(const char* who, const fs_shape* shape, const fs_kv_view* kv,
                         const fs_prefill_item* items_dev, const int32_t* sched_dev,
                         int64_t n_items, int32_t tile_tokens, float* part_o, float* part_lse, bool partials_needed,
                         const int64_t* out_indptr_dev, float* out, float* lse, void* stream) {
  if (!shape || !kv) return fs::fail(FS_EINVAL, "%s: shape or kv is NULL", who);
  if (shape->n_kv_heads < 1 || shape->n_q_heads < shape->n_kv_heads || shape->n_q_heads % shape->n_kv_heads)
    return fs::fail(FS_EINVAL, "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who,
                    shape->n_q_heads, shape->n_kv_heads);
  if (shape->head_dim != fs::kHeadDim)
    return fs::fail(FS_EUNSUPPORTED, "%s: head_dim %d (only %d is built)", who, shape->head_dim, fs::kHeadDim);
  if (shape->page_tokens != fs::kPageTokens)
    return fs::fail(FS_EUNSUPPORTED, "%s: page_tokens %d (only %d is built)", who, shape->page_tokens,
                    fs::kPageTokens);
  const int G = shape->n_q_heads / shape->n_kv_heads;
  if (G > fs::kMaxGroup) return fs::fail(FS_EINVAL, "%s: group %d > %d", who, G, fs::kMaxGroup);
  if (kv->kv_dtype != FS_KV_BF16 && kv->kv_dtype != FS_KV_FP8_E4M3)
    return fs::fail(FS_EINVAL, "%s: unknown kv_dtype %d", who, kv->kv_dtype);
  const bool fp8 = kv->kv_dtype == FS_KV_FP8_E4M3;
  if (n_items < 0 || n_items > 0x7FFFFFFF) return fs::fail(FS_EINVAL, "%s: n_items out of range", who);
  const int ct = fs::options().prefill_col_tiles, waves = fs::options().prefill_waves;
  const int cap = waves * ct * (16 / pad_group(G));
  if (tile_tokens < 1 || tile_tokens > cap)
    return fs::fail(FS_EINVAL, "%s: tile_tokens %d outside [1, %d] for group %d", who, tile_tokens, cap, G);
  if (n_items == 0) return FS_OK;
  if (!kv->q || !kv->k_pool || !kv->v_pool || !kv->page_indptr || !kv->page_ids || !items_dev ||
      (partials_needed && (!part_o || !part_lse)))
    return fs::fail(FS_EINVAL, "%s: NULL device pointer", who);
  if (fp8 && !kv->page_scales && (!kv->k_scale || !kv->v_scale))
    return fs::fail(FS_EINVAL, "%s: fp8 KV needs page_scales, or k_scale and v_scale", who);
  const int64_t slot_bytes = static_cast<int64_t>(fs::kPageTokens) * fs::kHeadDim * (fp8 ? 1 : 2);
  if (kv->k_slot_stride < slot_bytes || kv->v_slot_stride < slot_bytes || (kv->k_slot_stride & 15) ||
      (kv->v_slot_stride & 15) || (reinterpret_cast<uintptr_t>(kv->k_pool) & 15) ||
      (reinterpret_cast<uintptr_t>(kv->v_pool) & 15) || (reinterpret_cast<uintptr_t>(kv->q) & 15) ||
      (reinterpret_cast<uintptr_t>(part_o) & 15))
    return fs::fail(FS_EINVAL, "%s: pools, strides, q and part_o must be 16-byte aligned and strides "
                               "at least one slot (%lld bytes)", who, static_cast<long long>(slot_bytes));
  // The kernel's lazy running maximum is taken on the raw scores and scaled afterwards, which orders them
  // correctly only for a positive scale.
  if (!std::isfinite(kv->sm_scale) || kv->sm_scale <= 0.f)
    return fs::fail(FS_EINVAL, "%s: sm_scale %g is not finite and positive", who, static_cast<double>(kv->sm_scale));
  if (kv->v_range != FS_V_ANY && kv->v_range != FS_V_FP16_RANGE)
    return fs::fail(FS_EINVAL, "%s: unknown v_range %d", who, kv->v_range);

  PrefillParams P;
  P.q = static_cast<const uint16_t*>(kv->q);
  P.k_pool = static_cast<const char*>(kv->k_pool);
  P.v_pool = static_cast<const char*>(kv->v_pool);
  P.k_stride = kv->k_slot_stride;
  P.v_stride = kv->v_slot_stride;
  P.k_scale = kv->page_scales ? kv->page_scales : kv->k_scale;
  P.v_scale = kv->page_scales ? kv->page_scales + 1 : kv->v_scale;
  P.scale_by_page = kv->page_scales ? 1 : 0;
  P.page_indptr = kv->page_indptr;
  P.page_ids = kv->page_ids;
  P.items = items_dev;
  P.sched = sched_dev;
  P.part_o = part_o;
  P.part_lse = part_lse;
  P.out_indptr = out_indptr_dev;
  P.out = out;
  P.lse = lse;
  P.group = G;
  P.group_pad = pad_group(G);
  P.n_q_heads = shape->n_q_heads;
  P.tile_tokens = tile_tokens;
  P.scale_log2 = kv->sm_scale * 1.4426950408889634f;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool wide = kv->v_range != FS_V_FP16_RANGE;   // no statement about V: keep it in bf16
#define FS_PREFILL_CASE(W, C)                                                                     \
  case W * 10 + C:                                                                                \
    if (fp8)                                                                                      \
      return wide ? launch(prefill_fp8_kernel<W, C, true>, W * 64, P, n_items, s)                 \
                  : launch(prefill_fp8_kernel<W, C, false>, W * 64, P, n_items, s);               \
    return wide ? launch(prefill_bf16_kernel<W, C, true>, W * 64, P, n_items, s)                  \
                : launch(prefill_bf16_kernel<W, C, false>, W * 64, P, n_items, s)
  switch (waves * 10 + ct) {
    FS_PREFILL_CASE(4, 1);
    FS_PREFILL_CASE(4, 2);
    FS_PREFILL_CASE(4, 4);
    FS_PREFILL_CASE(8, 1);
    FS_PREFILL_CASE(8, 2);
    default: return fs::fail(FS_EINVAL, "%s: no kernel for prefill_waves %d, prefill_col_tiles %d", who, waves, ct);
  }
#undef FS_PREFILL_CASE
}

}  // namespace

extern "C" fs_status fs_prefill_attention(const fs_shape* shape, const fs_kv_view* kv,
                                          const fs_prefill_item* items_dev, const int32_t* sched_dev,
                                          int64_t n_items, int32_t tile_tokens, float* part_o, float* part_lse,
                                          void* stream) {
  return prefill_launch("fs_prefill_attention", shape, kv, items_dev, sched_dev, n_items, tile_tokens, part_o, part_lse, true,
                        nullptr, nullptr, nullptr, stream);
}

extern "C" fs_status fs_prefill_attention_fused(const fs_shape* shape, const fs_kv_view* kv,
                                                const fs_prefill_item* items_dev, const int32_t* sched_dev,
                                                int64_t n_items, int32_t tile_tokens,
                                                const int64_t* chunk_indptr_dev, int64_t n_tiles,
                                                const int64_t* out_indptr_dev, float* part_o, float* part_lse,
                                                float* out, float* lse, void* stream) {
  const char* who = "fs_prefill_attention_fused";
  if (n_tiles < 0 || n_tiles > n_items) return fs::fail(FS_EINVAL, "%s: n_tiles %lld outside [0, n_items]", who,
                                                        static_cast<long long>(n_tiles));
  if (n_items > 0 && (n_tiles == 0 || !chunk_indptr_dev || !out_indptr_dev || !out || !lse || (reinterpret_cast<uintptr_t>(out) & 15)))
    return fs::fail(FS_EINVAL, "%s: no tiles, or chunk_indptr_dev, out_indptr_dev, out or lse is NULL, or out is not 16-byte aligned", who);
  const bool split = n_items > n_tiles;          // some tile has more than one chunk: partial rows and a merge
  const fs_status st = prefill_launch(who, shape, kv, items_dev, sched_dev, n_items, tile_tokens, part_o, part_lse, split,
                                      out_indptr_dev, out, lse, stream);
  if (st != FS_OK || n_items == 0 || !split) return st;
  const int G = shape->n_q_heads / shape->n_kv_heads;
  return fs::merge_lse_launch(who, part_o, part_lse, chunk_indptr_dev, n_tiles, tile_tokens * G, out, lse, /*skip_single=*/true,
                              stream);
}

