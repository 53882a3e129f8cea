// fs_decode_attention: per-item partial decode attention over a paged KVCache, gfx950 only.
//
// What is computed is the decode phase of Section 2.1.1 of the paper (one new query token per
// request against all cached keys) for the ragged (request, KV head, chunk) list that the
// paper's hybrid attention (Section 3.1) leaves on one rank.  The kernel design below is not
// from the paper, which describes no kernel.
//
// bf16 path (GQA groups up to 16 q-heads):
//   One workgroup per work item, in the longest-first order the list prescribes; the hardware
//   dispatcher hands the next item to whichever CU frees a slot, which is list scheduling.
//   The item's pages are dealt to the workgroup's wavefronts in turn.  A wavefront streams
//   K and V pages with 16-byte-per-lane loads that are each one contiguous 1 KiB run, straight
//   into MFMA operand registers (the in-slot element order is built for that), several pages
//   ahead of the arithmetic.  Per page:
//     S^T[tok][q] = K . Q^T      4 x v_mfma_f32_16x16x32_bf16   (A = K page, B = Q^T)
//     online softmax in fp32, log2 domain; a lane owns q-head lane%16 and tokens 4*(lane/16)+r
//     O^T[d][q]  += V^T . P^T    16 x v_mfma_f32_16x16x16_bf16  (A = V page, B = P^T as bf16 hi + lo)
//   The S^T accumulator layout is exactly the B-operand layout of the second product, so the
//   softmax weights never move between lanes; only the running max needs a 2-step cross-lane
//   exchange.  Wavefronts merge (max, sum, O) through LDS at the end of the item.
//
// fp8 path (e4m3 K/V with one fp32 scale per slot): the same two products on the matrix cores; K is converted
// to bf16 in registers and V is transposed by a product with a constant matrix (see decode_fp8_kernel).
//
// Forms of the sweep, all with the same arithmetic per item (their rows agree bit for bit): one workgroup
// per item; resident workgroups that claim items from a counter; resident workgroups on equal runs of pages
// (no counter).  Each is written once over the K/V format (Bf16Format, Fp8Format).  Items come as list
// entries that the kernel looks up, or as launch records that the host has resolved (one 64-byte read).  A
// pair that is one item writes its final rows; the chunks of a split pair are merged by fs_merge_lse, or,
// given a counter per pair, by the workgroup that writes the pair's last rows.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>

#include "fs_internal.h"
#include "merge_row.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));


struct DecodeParams {
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
  const fs_work_item* __restrict__ items;
  const int32_t* __restrict__ sched;
  // Instead of items + sched: one record per item in launch order with everything already looked up
  // (fs_build_launch_records); NULL: the kernels look an item up themselves (list entry, item, page-table
  // offset, chunk count - four dependent reads before the first page can be asked for).
  const fs_launch_record* __restrict__ records;
  float* __restrict__ part_o;
  float* __restrict__ part_lse;
  // Fused form only (else NULL): a pair that is a single item writes its rows straight to the final
  // arrays, rows [pair*G, pair*G+G), and needs no merge.
  const int64_t* __restrict__ chunk_indptr;
  float* __restrict__ out;
  float* __restrict__ lse;
  // One counter per pair, zero between launches (else NULL): a workgroup that has written partial rows of a
  // split pair counts itself in, and the one that completes the pair merges it on the spot (arrive_and_merge),
  // so that no merge kernel has to follow the sweep.
  int32_t* pair_counters;
  int32_t group;
  float scale_log2;   // sm_scale * log2(e): scores live in the log2 domain
};

constexpr float kLn2 = 0.6931471805599453f;
constexpr int kORow = 132;   // floats per q row of the LDS merge buffer (128 + pad against bank conflicts)

// Butterfly steps across the four 16-lane rows of a wavefront.  v_permlane16_swap / v_permlane32_swap
// exchange rows (halves) between two registers; fed the same value twice they leave, in every lane,
// the lane's own value in one result and its partner's (lane^16, lane^32) in the other.
__device__ __forceinline__ float max_xor16(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];   // (copy the elements out: a bit_cast of r[i] itself reads element 0)
  return fmaxf(__uint_as_float(a), __uint_as_float(b));
}
__device__ __forceinline__ float max_xor32(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];   // (copy the elements out: a bit_cast of r[i] itself reads element 0)
  return fmaxf(__uint_as_float(a), __uint_as_float(b));
}
__device__ __forceinline__ float sum_xor16(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  return __uint_as_float(a) + __uint_as_float(b);
}
__device__ __forceinline__ float sum_xor32(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  return __uint_as_float(a) + __uint_as_float(b);
}

// One page's operands in registers: K as 4 A-operands of the 16x16x32 product (k = 32 d each),
// V as 4 x (2 A-operands of the 16x16x16 product) (16 d rows each, k = 16 tokens).
struct PageRegs {
  u32x4 k[4];
  u32x4 v[4];
};

__device__ __forceinline__ void load_page(PageRegs& r, const char* __restrict__ k_pool,
                                          const char* __restrict__ v_pool, int64_t k_stride,
                                          int64_t v_stride, int32_t slot, int lane) {
  const u32x4* kp = reinterpret_cast<const u32x4*>(k_pool + slot * k_stride) + lane;
  const u32x4* vp = reinterpret_cast<const u32x4*>(v_pool + slot * v_stride) + lane;
#pragma unroll
  for (int s = 0; s < 4; ++s) r.k[s] = __builtin_nontemporal_load(kp + s * 64);
#pragma unroll
  for (int s = 0; s < 4; ++s) r.v[s] = __builtin_nontemporal_load(vp + s * 64);
}

struct SoftmaxState {
  float m;        // running max (log2 domain) of this lane's q-head, same in the 4 lanes that share it
  float l;        // this lane's share of the running sum
  f32x4 acc[8];   // O^T[d = 16j + 4*(lane/16) + r][q = lane%16]
};

template <bool FULL>
__device__ __forceinline__ void consume_page(SoftmaxState& st, PageRegs& pg, const bf16x8 (&qreg)[4],
                                             float scale_log2, int valid, int kb) {
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < 4; ++c)
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pg.k[c]), qreg[c], s, 0, 0, 0);

  float x[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) x[r] = s[r] * scale_log2;
  if (!FULL && valid < fs::kPageTokens) {   // last page of the context: tokens past the end do not exist
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * kb + r >= valid) x[r] = -INFINITY;
    const uint32_t m0 = (4 * kb + 0 < valid ? 0x0000FFFFu : 0u) | (4 * kb + 1 < valid ? 0xFFFF0000u : 0u);
    const uint32_t m1 = (4 * kb + 2 < valid ? 0x0000FFFFu : 0u) | (4 * kb + 3 < valid ? 0xFFFF0000u : 0u);
#pragma unroll
    for (int c = 0; c < 4; ++c) {   // whatever bits sit there (NaN included) must not reach the product
      pg.v[c].x &= m0; pg.v[c].y &= m1; pg.v[c].z &= m0; pg.v[c].w &= m1;
    }
  }
  float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
  mx = max_xor32(max_xor16(mx));
  const float m_new = fmaxf(st.m, mx);
  if (__any(m_new > st.m)) {
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // first page: exp2(-inf) = 0
    st.l *= alpha;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j] *= alpha;
    st.m = m_new;
  }
  f32x4 p;
#pragma unroll
  for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(x[r] - st.m);
  st.l += (p[0] + p[1]) + (p[2] + p[3]);
  // The weights enter the matrix cores as bf16.  One bf16 keeps 8 bits, which for a short context
  // (weights near 1/2) costs ~2e-3 of |V| - the whole error budget.  Splitting p = hi + lo into two
  // bf16 terms keeps 16 bits; the second product rides on matrix-core time that is idle anyway.
  const bf16x4 ph = __builtin_convertvector(p, bf16x4);
  const bf16x4 pl = __builtin_convertvector(p - __builtin_convertvector(ph, f32x4), bf16x4);
  const s16x4 pb = __builtin_bit_cast(s16x4, ph), pc = __builtin_bit_cast(s16x4, pl);
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint2 lo = make_uint2(pg.v[c].x, pg.v[c].y), hi = make_uint2(pg.v[c].z, pg.v[c].w);
    const s16x4 va = __builtin_bit_cast(s16x4, lo), vb = __builtin_bit_cast(s16x4, hi);
    st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, pb, st.acc[2 * c], 0, 0, 0);
    st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb, pb, st.acc[2 * c + 1], 0, 0, 0);
    st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va, pc, st.acc[2 * c], 0, 0, 0);
    st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vb, pc, st.acc[2 * c + 1], 0, 0, 0);
  }
}

// ---------------------------------------------------------------------------------------------
// fp8 e4m3 path (one fp32 scale per slot for K and one for V), on the matrix cores for every group size.
//
// The slot order [d/64][(d%64)/16][tok][d%16] makes a wave-wide 16-byte load one contiguous 1 KiB run in which
// lane (tok = lane%16, kb = lane/16) receives 16 consecutive d of its token: d = 64j + 16kb .. for load j = 0, 1
// (whole 128-byte lines per instruction; with token-major slots the same lanes read half lines and the launch
// ran at two thirds of the rate, bound by the number of requests a CU may have pending).
//
// The first product wants exactly that: a lane holds 8 consecutive d of one token per instruction,
// d = 64j + 16kb + 8half + e for instruction c = 2j + half (any order of d will do as long as the query operand
// follows it); K is converted e4m3 -> bf16 in registers, which is exact.
//     S^T[tok][q] = K . Q^T      4 x v_mfma_f32_16x16x32_bf16, times scale * k_scale of the page
// The second product reduces over tokens, so it wants a lane to hold several tokens of one d: the transpose of
// what was loaded.  The matrix cores do that on the way: V's bytes go in as they are, as the A operand of an fp8
// product whose B operand is a constant matrix of ones and zeros that picks 16 of the 32 d of the slice,
//     T[tok][n] = sum_k V[tok][k] * E[k][n] = V[tok][d(n)]      8 x v_mfma_f32_16x16x32_fp8_fp8
// exact in fp32 (one product by 1.0 plus zeros), and the result layout (lane n + 16kb holds tokens 4kb .. 4kb+3 of
// column n) is the A-operand layout of
//     O^T[d(n)][q] += V^T . P^T  16 x v_mfma_f32_16x16x16_bf16 (weights times v_scale, as bf16 hi + lo)
// after packing T to bf16 (exact again).  The rows of O^T come out in the order fp8_first_d states.
// A kernel that multiplied on the vector units instead (each K and V value once per q-head) kept pace with the
// page stream for one q-head per KV head and not beyond: with eight it ran at a quarter of this one's rate.
// ---------------------------------------------------------------------------------------------

// Where a lane's rows of O^T start: accumulator a = 4j + 2half + h2 of lane (q, kb) holds d = fp8_first_d(a, kb) .. + 4.
__device__ __forceinline__ int fp8_first_d(int a, int kb) {
  return 64 * (a >> 2) + 32 * (a & 1) + 16 * (kb >> 1) + 8 * ((a >> 1) & 1) + 4 * (kb & 1);
}

struct Fp8Page {
  u32x4 k[2];
  u32x4 v[2];
  float ks, vs;
};

__device__ __forceinline__ void load_page_fp8(Fp8Page& r, const DecodeParams& P, int32_t slot, int64_t page, int lane) {
  const u32x4* kp = reinterpret_cast<const u32x4*>(P.k_pool + slot * P.k_stride) + lane;
  const u32x4* vp = reinterpret_cast<const u32x4*>(P.v_pool + slot * P.v_stride) + lane;
  r.k[0] = __builtin_nontemporal_load(kp);
  r.k[1] = __builtin_nontemporal_load(kp + 64);
  r.v[0] = __builtin_nontemporal_load(vp);
  r.v[1] = __builtin_nontemporal_load(vp + 64);
  const int64_t si = P.scale_by_page ? 2 * page : static_cast<int64_t>(slot);
  r.ks = P.k_scale[si];
  r.vs = P.v_scale[si];
}

// Two fp32 values to one dword of two bf16 by dropping the low halves (exact for values that are bf16 already).
__device__ __forceinline__ uint32_t pack_bf16_trunc(float lo, float hi) {
  return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

// Eight e4m3 bytes (two dwords) to the eight bf16 of a first-product operand: exact, one instruction per pair
// (the conversion takes a power-of-two scale; 1.0 is 2^0).
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8 fp8x8_to_bf16x8(uint32_t w0, uint32_t w1) {
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false);
  const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false);
  const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true);
  const u32x4 r = {__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, b), __builtin_bit_cast(uint32_t, c),
                   __builtin_bit_cast(uint32_t, d)};
  return __builtin_bit_cast(bf16x8, r);
}

template <bool FULL>
__device__ __forceinline__ void consume_page_fp8(SoftmaxState& st, const Fp8Page& pg, const bf16x8 (&qreg)[4],
                                                  const long (&pick)[2], float scale_log2, int valid, int kb) {
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp8x8_to_bf16x8(pg.k[j].x, pg.k[j].y), qreg[2 * j], s, 0, 0, 0);
    s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fp8x8_to_bf16x8(pg.k[j].z, pg.k[j].w), qreg[2 * j + 1], s, 0, 0, 0);
  }
  // V's eight transposes go to the matrix cores now and run under the softmax below
  f32x4 t[8];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const uint32_t w[4] = {pg.v[j].x, pg.v[j].y, pg.v[j].z, pg.v[j].w};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const long bytes = static_cast<long>((static_cast<unsigned long>(w[2 * half + 1]) << 32) | w[2 * half]);
      const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
        t[4 * j + 2 * half + h2] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(bytes, pick[h2], z, 0, 0, 0);
    }
  }
  const float sc = scale_log2 * pg.ks;
  float x[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) x[r] = s[r] * sc;
  uint32_t m0 = 0xFFFFFFFFu, m1 = 0xFFFFFFFFu;
  if (!FULL && valid < fs::kPageTokens) {   // last page of the context: tokens past the end do not exist
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (4 * kb + r >= valid) x[r] = -INFINITY;
    m0 = (4 * kb + 0 < valid ? 0x0000FFFFu : 0u) | (4 * kb + 1 < valid ? 0xFFFF0000u : 0u);
    m1 = (4 * kb + 2 < valid ? 0x0000FFFFu : 0u) | (4 * kb + 3 < valid ? 0xFFFF0000u : 0u);
  }
  float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
  mx = max_xor32(max_xor16(mx));
  const float m_new = fmaxf(st.m, mx);
  if (__any(m_new > st.m)) {
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // first page: exp2(-inf) = 0
    st.l *= alpha;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j] *= alpha;
    st.m = m_new;
  }
  float p[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) p[r] = __builtin_amdgcn_exp2f(x[r] - st.m);
  st.l += (p[0] + p[1]) + (p[2] + p[3]);
  // The weights enter the second product as bf16 hi + lo (16 bits; see consume_page), times the page's V scale.
  // hi is the value cut to bf16, lo what is left, cut again: two instructions per pair and two per value.
  float pv[4], rest[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    pv[r] = p[r] * pg.vs;
    rest[r] = pv[r] - __uint_as_float(__float_as_uint(pv[r]) & 0xFFFF0000u);
  }
  const uint2 hi2 = make_uint2(pack_bf16_trunc(pv[0], pv[1]), pack_bf16_trunc(pv[2], pv[3]));
  const uint2 lo2 = make_uint2(pack_bf16_trunc(rest[0], rest[1]), pack_bf16_trunc(rest[2], rest[3]));
  const s16x4 pb = __builtin_bit_cast(s16x4, hi2), pc = __builtin_bit_cast(s16x4, lo2);
  s16x4 va[8];
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    uint2 tv = make_uint2(pack_bf16_trunc(t[a][0], t[a][1]), pack_bf16_trunc(t[a][2], t[a][3]));
    if (!FULL) { tv.x &= m0; tv.y &= m1; }   // whatever bits sit beyond the end (NaN included) must not reach the product
    va[a] = __builtin_bit_cast(s16x4, tv);
  }
  // eight independent accumulators: the hi products of all, then the lo products, so that none waits for the other
#pragma unroll
  for (int a = 0; a < 8; ++a) st.acc[a] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[a], pb, st.acc[a], 0, 0, 0);
#pragma unroll
  for (int a = 0; a < 8; ++a) st.acc[a] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(va[a], pc, st.acc[a], 0, 0, 0);
}

// The page table is read-only for the whole launch, but the kernels also write to global memory, so the
// compiler does not take its word for that and would fetch the page ids with vector loads, which queue up
// behind the page loads.  Reading them through the constant address space keeps them on the scalar path.
typedef const int32_t __attribute__((address_space(4))) * const_ids_ptr;

// What a wavefront needs to know of an item.  The item's pages are dealt to the workgroup's wavefronts in
// turn: wavefront w of W takes pages w, w + W, w + 2W, ... of the item, `n_mine` of them.
struct ItemDesc {
  const_ids_ptr ids;    // page ids of the item's first page onwards
  int32_t page_lo, page_hi;   // position of the item's first page in the whole page table (fp8 scales in page order)
  int n_tok;            // tokens of the item
  int n_mine;           // pages of the item this wavefront takes
  int row;              // first partial row of the item, or -(first final row) - 1 when the item is all of its pair (one-call forms)
  int q_row;            // first query row of the item's group
  int pair, n_chunks, pair_row;   // the item's pair, its chunk count and the first partial row of its first chunk (n_chunks = 1 when unknown)
  int32_t first_ids[3]; // slots of this wavefront's first pages (those the prologue fetches), asked for with the rest
  bf16x8 q[4];          // Q^T operand of this lane (load_desc_q; bf16 kernels)
  bool valid;
};

// The scalar part of the descriptor of the item at launch position k: everything but the query rows.  All of
// it stays in scalar registers.  With launch records that is one 64-byte read (and the first slots come out of
// the same record, asked for at the same time); without, the list entry, the item, the page-table offset and
// chunk count, and the page ids are read one after the other.
template <int WAVES, int NBUF>
__device__ __forceinline__ ItemDesc load_desc_head(const DecodeParams& P, int k, int n_items, int wave, int G) {
  static_assert(NBUF - 1 <= 3, "first_ids holds three slots");
  ItemDesc d;
  d.valid = k < n_items;
  d.ids = (const_ids_ptr)(uintptr_t)0;
  d.page_lo = d.page_hi = 0;
  d.n_tok = 0;
  d.n_mine = 0;
  d.row = 0;
  d.q_row = 0;
  d.pair = 0;
  d.n_chunks = 1;
  d.pair_row = 0;
#pragma unroll
  for (int u = 0; u < 3; ++u) d.first_ids[u] = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) d.q[c] = bf16x8{};
  if (d.valid) {
    int64_t first_page;
    int32_t rec_slot[3] = {0, 0, 0};
    if (P.records) {
      // k is the same in every lane (it may come from LDS, which the compiler cannot see): saying so keeps
      // the descriptor and, above all, the page ids on the scalar path
      const fs_launch_record* rec = P.records + __builtin_amdgcn_readfirstlane(k);
      first_page = rec->first_page;
      d.n_tok = __builtin_amdgcn_readfirstlane(rec->n_tok);
      d.q_row = __builtin_amdgcn_readfirstlane(rec->q_row);
      d.row = __builtin_amdgcn_readfirstlane(rec->row);
      d.pair = __builtin_amdgcn_readfirstlane(rec->pair);
      d.n_chunks = __builtin_amdgcn_readfirstlane(rec->n_chunks);
      d.pair_row = __builtin_amdgcn_readfirstlane(rec->pair_row);
#pragma unroll
      for (int u = 0; u < NBUF - 1; ++u)           // the record holds the item's first eight slots
        if (wave + u * WAVES < 8) rec_slot[u] = __builtin_amdgcn_readfirstlane(rec->first_slots[wave + u * WAVES]);
    } else {
      const int item_idx = __builtin_amdgcn_readfirstlane(P.sched ? P.sched[k] : k);
      fs_work_item it = P.items[item_idx];
      it.pair = __builtin_amdgcn_readfirstlane(it.pair);
      it.tok_begin = __builtin_amdgcn_readfirstlane(it.tok_begin);
      it.tok_end = __builtin_amdgcn_readfirstlane(it.tok_end);
      d.n_tok = it.tok_end - it.tok_begin;
      d.q_row = __builtin_amdgcn_readfirstlane(it.q_row);
      d.row = __builtin_amdgcn_readfirstlane(it.part_row);
      first_page = P.page_indptr[it.pair] + it.tok_begin / fs::kPageTokens;
      d.pair = it.pair;
      if (P.chunk_indptr) {
        const int64_t c0 = P.chunk_indptr[it.pair];
        d.n_chunks = __builtin_amdgcn_readfirstlane(static_cast<int32_t>(P.chunk_indptr[it.pair + 1] - c0));
        d.pair_row = __builtin_amdgcn_readfirstlane(static_cast<int32_t>(c0) * G);
        if (d.n_chunks == 1) d.row = -(it.pair * G) - 1;
      }
    }
    d.page_lo = __builtin_amdgcn_readfirstlane(static_cast<int32_t>(first_page));
    d.page_hi = __builtin_amdgcn_readfirstlane(static_cast<int32_t>(first_page >> 32));
    d.ids = (const_ids_ptr)(reinterpret_cast<uintptr_t>(P.page_ids + ((static_cast<int64_t>(d.page_hi) << 32) | static_cast<uint32_t>(d.page_lo))));
    const int n_pages = (d.n_tok + fs::kPageTokens - 1) / fs::kPageTokens;
    d.n_mine = n_pages > wave ? (n_pages - wave + WAVES - 1) / WAVES : 0;
#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u) {
      if (u < d.n_mine) d.first_ids[u] = (P.records && wave + u * WAVES < 8) ? rec_slot[u] : d.ids[wave + u * WAVES];
    }
  }
  return d;
}

// The query rows of the item, as the Q^T operand of this lane: lane (q = lane%16, kb = lane/16) holds
// Q[q][32c + 8kb .. +8) for c = 0..3; rows beyond the group are zero (read from a row that exists, then blanked).
__device__ __forceinline__ void load_desc_q(ItemDesc& d, const DecodeParams& P, int lane, int G) {
  if (d.valid) {
    const int qi = lane & 15, kb = lane >> 4;
    const int qrow = d.q_row + min(qi, G - 1);
    const u32x4* qp = reinterpret_cast<const u32x4*>(P.q + static_cast<int64_t>(qrow) * fs::kHeadDim) + kb;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 v = qp[4 * c];
      if (qi >= G) v = u32x4{0u, 0u, 0u, 0u};
      d.q[c] = __builtin_bit_cast(bf16x8, v);
    }
  }
}

// The same for the fp8 kernels, in the order of d that their K operand has: instruction c = 2j + half takes
// d = 64j + 16kb + 8half .. + 8.
__device__ __forceinline__ void load_desc_q_fp8(ItemDesc& d, const DecodeParams& P, int lane, int G) {
  if (d.valid) {
    const int qi = lane & 15, kb = lane >> 4;
    const int qrow = d.q_row + min(qi, G - 1);
    const u32x4* qp = reinterpret_cast<const u32x4*>(P.q + static_cast<int64_t>(qrow) * fs::kHeadDim) + 2 * kb;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 v = qp[8 * (c >> 1) + (c & 1)];
      if (qi >= G) v = u32x4{0u, 0u, 0u, 0u};
      d.q[c] = __builtin_bit_cast(bf16x8, v);
    }
  }
}

__device__ __forceinline__ int64_t first_page_of(const ItemDesc& d) {
  return (static_cast<int64_t>(d.page_hi) << 32) | static_cast<uint32_t>(d.page_lo);
}

// What the two K/V formats differ in, for the kernels below: the registers of a page in flight, how a page is
// loaded and consumed, the order of d in the query operand and in a lane's rows of O^T (acc[j] holds four
// consecutive d from first_d(j, lane/16) on).  `page` is the page's position in the whole page table.
struct Bf16Format {
  using Page = PageRegs;
  struct Consts {};
  static __device__ __forceinline__ Consts consts(int) { return Consts{}; }
  static __device__ __forceinline__ void load(Page& r, const DecodeParams& P, int32_t slot, int64_t, int lane) {
    load_page(r, P.k_pool, P.v_pool, P.k_stride, P.v_stride, slot, lane);
  }
  template <bool FULL>
  static __device__ __forceinline__ void consume(SoftmaxState& st, Page& pg, const bf16x8 (&q)[4], const Consts&,
                                                 float scale_log2, int valid, int kb) {
    consume_page<FULL>(st, pg, q, scale_log2, valid, kb);
  }
  static __device__ __forceinline__ void load_q(ItemDesc& d, const DecodeParams& P, int lane, int G) { load_desc_q(d, P, lane, G); }
  static __device__ __forceinline__ int first_d(int j, int kb) { return 16 * j + 4 * kb; }
};
struct Fp8Format {
  using Page = Fp8Page;
  struct Consts { long pick[2]; };
  // E[k][n] for the two halves of a 32-d slice: column n = lane%16 takes k = 16h2 + n, which sits in the lanes
  // with kb = 2h2 + n/8 as byte n%8 (0x38 is 1.0 in e4m3)
  static __device__ __forceinline__ Consts consts(int lane) {
    const int qi = lane & 15, kb = lane >> 4;
    Consts c;
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
      c.pick[h2] = (kb == 2 * h2 + (qi >> 3)) ? static_cast<long>(0x38ul << (8 * (qi & 7))) : 0l;
    return c;
  }
  static __device__ __forceinline__ void load(Page& r, const DecodeParams& P, int32_t slot, int64_t page, int lane) {
    load_page_fp8(r, P, slot, page, lane);
  }
  template <bool FULL>
  static __device__ __forceinline__ void consume(SoftmaxState& st, Page& pg, const bf16x8 (&q)[4], const Consts& c,
                                                 float scale_log2, int valid, int kb) {
    consume_page_fp8<FULL>(st, pg, q, c.pick, scale_log2, valid, kb);
  }
  static __device__ __forceinline__ void load_q(ItemDesc& d, const DecodeParams& P, int lane, int G) { load_desc_q_fp8(d, P, lane, G); }
  static __device__ __forceinline__ int first_d(int j, int kb) { return fp8_first_d(j, kb); }
};

// Where an item's G rows go, from the descriptor's row.
struct RowDest {
  float* o;
  float* lse;
  int row;
};
__device__ __forceinline__ RowDest row_dest(const DecodeParams& P, int row) {
  if (row < 0) return RowDest{P.out, P.lse, -row - 1};
  return RowDest{P.part_o, P.part_lse, row};
}

// A partial row on its way to the workgroup that will merge its pair inside the same launch: relaxed atomic stores
// at device scope, which are written through to memory instead of waiting in this XCD's L2 (the other workgroup
// may run on another XCD, whose L2 is not this one's).
__device__ __forceinline__ void store_f32_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_f32x4_coherent(float* p, const f32x4 v) {
  auto* q = reinterpret_cast<unsigned long long*>(p);
  const unsigned long long lo = (static_cast<unsigned long long>(__float_as_uint(v[1])) << 32) | __float_as_uint(v[0]);
  const unsigned long long hi = (static_cast<unsigned long long>(__float_as_uint(v[3])) << 32) | __float_as_uint(v[2]);
  __hip_atomic_store(q, lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store(q + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Split pairs merged inside the sweep.  The workgroup has just issued the stores of the partial rows of `n` items
// (s_pair/s_chunks/s_prow[j]: pair, chunk count and first partial row of the pair of item j; s_chunks[j] = 1: not
// split, nothing to do).  One thread per item counts the workgroup in on the pair's counter; the workgroup that
// brings a counter to the pair's chunk count is the last writer of that pair: it puts the counter back to zero for
// the next launch and merges the pair's chunks into its final rows, one wavefront per q-head, with the routine of
// the merge kernel (same bits).  Nobody waits for anybody.
// What makes the other workgroups' rows visible, without fences (a device-scope fence writes back and invalidates
// the whole L2 of the XCD, which on the 70B-shaped batch cost the sweep 150 us): partial rows are stored
// (store_f32*_coherent) and read (merge_rows<.., COHERENT>) as relaxed device-scope atomics, which go to memory
// past the caches, as the counter's atomic does; a thread counts in only after all the workgroup's stores have been
// acknowledged (vmcnt(0) in every thread, then the barrier), and the merging workgroup reads only after its atomic
// has returned the full count, i.e. after every other writer's atomic, each issued after its own stores were done.
// Takes the workgroup's barriers: every thread must call it.
template <int WAVES>
__device__ __forceinline__ void arrive_and_merge(const DecodeParams& P, int n, const int* s_pair, const int* s_chunks,
                                                 const int* s_prow, int* s_done, int G, int wave, int lane) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this thread's stores have reached memory
  __syncthreads();
  for (int j = threadIdx.x; j < n; j += WAVES * 64) {
    const int c = s_chunks[j];
    s_done[j] = c > 1 && __hip_atomic_fetch_add(P.pair_counters + s_pair[j], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == c - 1;
  }
  __syncthreads();
  for (int j = 0; j < n; ++j) {
    if (!__builtin_amdgcn_readfirstlane(s_done[j])) continue;
    const int pair = __builtin_amdgcn_readfirstlane(s_pair[j]);
    const int chunks = __builtin_amdgcn_readfirstlane(s_chunks[j]);
    const int prow = __builtin_amdgcn_readfirstlane(s_prow[j]);
    if (threadIdx.x == 0) __hip_atomic_store(P.pair_counters + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const float* po = P.part_o;
    const float* pl = P.part_lse;
    // a wavefront takes as many q-heads side by side as divide the group evenly over the workgroup (their loads travel
    // together: one trip to memory instead of one per q-head); the sums of a row are the same in every form
    const int64_t c0 = prow / G;
    float* const out0 = P.out + static_cast<int64_t>(pair) * G * fs::kHeadDim;
    float* const lse0 = P.lse + static_cast<int64_t>(pair) * G;
    if (G % (2 * WAVES) == 0) {
      for (int g = 2 * wave; g < G; g += 2 * WAVES)
        fs_merge::merge_rows<2, true>(po, pl, c0, chunks, G, g, out0 + g * fs::kHeadDim, lse0 + g, lane);
    } else {
      for (int g = wave; g < G; g += WAVES)
        fs_merge::merge_rows<1, true>(po, pl, c0, chunks, G, g, out0 + g * fs::kHeadDim, lse0 + g, lane);
    }
  }
}

// The same for the one item of a workgroup that has no more than that.
template <int WAVES>
__device__ __forceinline__ void arrive_and_merge_one(const DecodeParams& P, const ItemDesc& d, int* s_meta, int G, int wave,
                                                     int lane) {
  if (P.pair_counters == nullptr || d.n_chunks <= 1) return;     // the same for the whole workgroup
  if (threadIdx.x == 0) {
    s_meta[0] = d.pair;
    s_meta[1] = d.n_chunks;
    s_meta[2] = d.pair_row;
  }
  arrive_and_merge<WAVES>(P, 1, s_meta, s_meta + 1, s_meta + 2, s_meta + 3, G, wave, lane);
}

// Merge the wavefronts' (m, l, O^T) through LDS and write the item's G partial rows.
template <int WAVES, typename FMT>
__device__ __forceinline__ void merge_and_store(const SoftmaxState& st, float l_total, int wave, int lane,
                                                int G, float* __restrict__ part_o,
                                                float* __restrict__ part_lse, int part_row,
                                                float* sm_o, float* sm_m, float* sm_l, bool coherent) {
  const int qi = lane & 15, kb = lane >> 4;
  if (lane < 16) {
    sm_m[wave * 16 + lane] = st.m;
    sm_l[wave * 16 + lane] = l_total;
  }
  float* row = sm_o + (wave * 16 + qi) * kORow;
#pragma unroll
  for (int j = 0; j < 8; ++j) *reinterpret_cast<f32x4*>(row + FMT::first_d(j, kb)) = st.acc[j];
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * 32; idx += WAVES * 64) {
    const int q = idx >> 5, d4 = idx & 31;
    float M = sm_m[q];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) M = fmaxf(M, sm_m[w * 16 + q]);
    float L = 0.f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float wgt = __builtin_amdgcn_exp2f(sm_m[w * 16 + q] - M);   // a wave with no pages has m = -inf
      L += wgt * sm_l[w * 16 + q];
      o += wgt * *reinterpret_cast<const f32x4*>(sm_o + (w * 16 + q) * kORow + 4 * d4);
    }
    const float inv = 1.0f / L;
    // Streaming stores: the partial rows are read once, by the merge.  Measured on the 70B-shaped
    // batch, plain stores of these 9 MB cost the 2 GB read stream about 20 us, non-temporal ones 13.
    float* dst = part_o + static_cast<int64_t>(part_row + q) * fs::kHeadDim + 4 * d4;
    const float lse_q = (M + __builtin_amdgcn_logf(L)) * kLn2;
    if (coherent) {      // rows another workgroup of this launch will merge (arrive_and_merge)
      store_f32x4_coherent(dst, o * inv);
      if (d4 == 0) store_f32_coherent(part_lse + part_row + q, lse_q);
    } else {
      __builtin_nontemporal_store(o * inv, reinterpret_cast<f32x4*>(dst));
      if (d4 == 0) __builtin_nontemporal_store(lse_q, part_lse + part_row + q);
    }
  }
}

// One workgroup per item.  NBUF register buffers; NBUF-1 pages are in flight while one is consumed.  The
// steady-state loop is branch-free (every prefetch is in range, every page is full), so the loads of pages
// i+1.. stay outstanding while page i is consumed; the ragged end is a second loop.  Index i counts this
// wavefront's pages; its i-th page is page wave + i*WAVES of the item.
template <int WAVES, int NBUF, typename FMT>
__device__ __forceinline__ void sweep_one_item(const DecodeParams& P) {
  __shared__ __attribute__((aligned(16))) float sm_o[WAVES * 16 * kORow];
  __shared__ float sm_m[WAVES * 16];
  __shared__ float sm_l[WAVES * 16];
  __shared__ int s_meta[4];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kb = lane >> 4;
  const int G = P.group;
  ItemDesc d = load_desc_head<WAVES, NBUF>(P, static_cast<int>(blockIdx.x), 0x7FFFFFFF, wave, G);
  FMT::load_q(d, P, lane, G);
  const int64_t first_page = first_page_of(d);
  const typename FMT::Consts consts = FMT::consts(lane);

  SoftmaxState st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) st.acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

  typename FMT::Page buf[NBUF];
#pragma unroll
  for (int u = 0; u < NBUF - 1; ++u)
    if (u < d.n_mine) FMT::load(buf[u], P, d.first_ids[u], first_page + wave + u * WAVES, lane);

  int i = 0;
  for (; i + 2 * NBUF - 2 < d.n_mine; i += NBUF) {
#pragma unroll
    for (int u = 0; u < NBUF; ++u) {
      const int pg = wave + (i + u + NBUF - 1) * WAVES;
      FMT::load(buf[(u + NBUF - 1) % NBUF], P, d.ids[pg], first_page + pg, lane);
      FMT::template consume<true>(st, buf[u], d.q, consts, P.scale_log2, fs::kPageTokens, kb);
    }
  }
  // here pages i .. i+NBUF-2 (those below n_mine) are in flight in buf[0 .. NBUF-2]
#pragma unroll
  for (int u = 0; u < 2 * NBUF - 2; ++u) {
    const int pi = i + u;
    if (pi < d.n_mine) {
      const int pn = pi + NBUF - 1;
      if (pn < d.n_mine) FMT::load(buf[(u + NBUF - 1) % NBUF], P, d.ids[wave + pn * WAVES], first_page + wave + pn * WAVES, lane);
      FMT::template consume<false>(st, buf[u % NBUF], d.q, consts, P.scale_log2,
                                   min(fs::kPageTokens, d.n_tok - (wave + pi * WAVES) * fs::kPageTokens), kb);
    }
  }

  const RowDest dst = row_dest(P, d.row);
  const float l_total = sum_xor32(sum_xor16(st.l));
  merge_and_store<WAVES, FMT>(st, l_total, wave, lane, G, dst.o, dst.lse, dst.row, sm_o, sm_m, sm_l,
                              P.pair_counters != nullptr && d.n_chunks > 1);
  arrive_and_merge_one<WAVES>(P, d, s_meta, G, wave, lane);
}

// (at least two wavefronts per SIMD, for both formats: within 256 registers the compiler keeps the matrix results
// in ordinary registers; allowed 512 it parks them in accumulation registers and moves every one back before the
// vector units can touch it - with fp8 pages 57 extra instructions per page; with bf16 pages the launch is bound by
// memory and the long lists do not notice, the short ones start faster)
template <int WAVES, int NBUF>
__global__ void __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
decode_bf16_kernel(const DecodeParams P) {
  sweep_one_item<WAVES, NBUF, Bf16Format>(P);
}

template <int WAVES, int NBUF>
__global__ void __launch_bounds__(WAVES * 64) __attribute__((amdgpu_waves_per_eu(2)))
decode_fp8_kernel(const DecodeParams P) {
  sweep_one_item<WAVES, NBUF, Fp8Format>(P);
}

// ---------------------------------------------------------------------------------------------
// Persistent form of the sweep.  A fixed set of workgroups (two per CU) walks the list: the
// first gridDim.x items go one to each workgroup, every further item is claimed from a counter
// in the list's longest-first order at the moment a workgroup has streamed its current item
// (list scheduling, as the hardware dispatcher does for one workgroup per item).  Finished
// partial rows wait in LDS and leave in one burst when the staging area is full or the
// workgroup is done: writes scattered through the launch slow the read stream far more than
// their bytes explain, writes at the end of a workgroup's life mostly do not.  The next item's
// descriptor, query rows and first pages are fetched while the current item's rows are merged,
// and the barriers around that merge wait for LDS traffic only, so those loads stay in flight
// across them.  claim[0] counts the items handed out beyond the first gridDim.x, claim[1] the workgroups
// that have left; both are zero between launches.
// ---------------------------------------------------------------------------------------------

constexpr int kStageRows = 64;    // partial rows a workgroup keeps in LDS before it writes them (64 x 512 B)
constexpr int kSecondShare = 4;   // a CU's second workgroup claims only within the first 1/kSecondShare of the list

__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// UNITS = true is the form without a counter: workgroup u walks the items [unit_indptr[u], unit_indptr[u+1]) of a
// list that the host has cut into equal runs of pages (fs_build_worklist_units), so every workgroup streams
// the same number of bytes and nothing is handed out at run time; `claim` then carries nothing.
template <int WAVES, int NBUF, bool UNITS, typename FMT>
__device__ __forceinline__ void persistent_sweep(const DecodeParams& P, int n_items, int* __restrict__ claim, int n_first,
                                                 const int64_t* __restrict__ unit_indptr) {
  __shared__ __attribute__((aligned(16))) float sm_o[WAVES * 16 * kORow];
  __shared__ float sm_m[WAVES * 16];
  __shared__ float sm_l[WAVES * 16];
  __shared__ __attribute__((aligned(16))) float st_o[kStageRows * fs::kHeadDim];
  __shared__ float st_lse[kStageRows];
  __shared__ int st_row[kStageRows];
  __shared__ int s_next;
  // what arrive_and_merge needs to know of the items whose rows are staged (at most kStageRows items: G >= 1)
  __shared__ int st_pair[kStageRows], st_chunks[kStageRows], st_prow[kStageRows], st_done[kStageRows];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qi = lane & 15, kb = lane >> 4;
  const int G = P.group;
  const int n_groups = gridDim.x;

  int unit_end = 0, cur_k = static_cast<int>(blockIdx.x);
  if constexpr (UNITS) {
    cur_k = __builtin_amdgcn_readfirstlane(static_cast<int>(unit_indptr[blockIdx.x]));
    unit_end = __builtin_amdgcn_readfirstlane(static_cast<int>(unit_indptr[blockIdx.x + 1]));   // > cur_k: no unit is empty
  }
  ItemDesc cur = load_desc_head<WAVES, NBUF>(P, cur_k, n_items, wave, G);   // a valid item by the launch
  FMT::load_q(cur, P, lane, G);
  const typename FMT::Consts consts = FMT::consts(lane);

  typename FMT::Page buf[NBUF];
  auto prologue = [&](const ItemDesc& d) __attribute__((always_inline)) {
    const int64_t first_page = first_page_of(d);
#pragma unroll
    for (int u = 0; u < NBUF - 1; ++u)
      if (u < d.n_mine) FMT::load(buf[u], P, d.first_ids[u], first_page + wave + u * WAVES, lane);
  };
  prologue(cur);

  // Two workgroups share a CU, and the one launched second streams at about half the rate of the first (the
  // issue arbiter prefers the older wavefront) while the CU's total stays the same.  A late item in its hands
  // takes twice as long and ends the launch late, so the workgroups beyond the first n_first (one per CU) -
  // by launch order the second workgroup of a CU - stop claiming once a quarter of the list is handed out;
  // they are there to fill the CU while the list is long, and leave the rest to their siblings.  (Where launch
  // order does not map to CUs like that, as many workgroups retire early just the same, which costs nothing
  // measurable.)
  const bool second_on_cu = static_cast<int>(blockIdx.x) >= n_first;
  bool keep_claiming = true;
  int staged = 0, staged_items = 0;
  bool staged_split = false;       // some staged item belongs to a split pair
  for (;;) {
    // With equal runs the next item is known from the start: its descriptor and the slots of its first pages are
    // asked for now and travel while the current item streams, so that at the item's end the next pages can be
    // requested at once.  With a counter the next item is only known after the claim (below).
    ItemDesc nxt;
    if constexpr (UNITS) {
      ++cur_k;
      nxt = load_desc_head<WAVES, NBUF>(P, cur_k < unit_end ? cur_k : n_items, n_items, wave, G);
    }
    SoftmaxState st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int64_t first_page = first_page_of(cur);
    int i = 0;          // counts this wavefront's pages of the item: its i-th page is page wave + i*WAVES
    for (; i + 2 * NBUF - 2 < cur.n_mine; i += NBUF) {
#pragma unroll
      for (int u = 0; u < NBUF; ++u) {
        const int pg = wave + (i + u + NBUF - 1) * WAVES;
        FMT::load(buf[(u + NBUF - 1) % NBUF], P, cur.ids[pg], first_page + pg, lane);
        FMT::template consume<true>(st, buf[u], cur.q, consts, P.scale_log2, fs::kPageTokens, kb);
      }
    }
#pragma unroll
    for (int u = 0; u < 2 * NBUF - 2; ++u) {
      const int pi = i + u;
      if (pi < cur.n_mine) {
        const int pn = pi + NBUF - 1;
        if (pn < cur.n_mine) FMT::load(buf[(u + NBUF - 1) % NBUF], P, cur.ids[wave + pn * WAVES], first_page + wave + pn * WAVES, lane);
        FMT::template consume<false>(st, buf[u % NBUF], cur.q, consts, P.scale_log2,
                                     min(fs::kPageTokens, cur.n_tok - (wave + pi * WAVES) * fs::kPageTokens), kb);
      }
    }
    // merge the wavefronts through LDS into the staging rows
    const float l_total = sum_xor32(sum_xor16(st.l));
    if (lane < 16) {
      sm_m[wave * 16 + lane] = st.m;
      sm_l[wave * 16 + lane] = l_total;
    }
    {
      float* row = sm_o + (wave * 16 + qi) * kORow;
#pragma unroll
      for (int j = 0; j < 8; ++j) *reinterpret_cast<f32x4*>(row + FMT::first_d(j, kb)) = st.acc[j];
    }
    // The next item is claimed only now.  Claiming it earlier would hide the counter's round trip, but a
    // workgroup would then sit on an item another could have started: claiming at the start of the current
    // item cost 11 us of the launch on the 70B-shaped batch, two items ahead 20 us, four pages early 4 us.
    if constexpr (!UNITS) {
      if (threadIdx.x == 0) s_next = keep_claiming ? atomicAdd(claim, 1) + n_groups : n_items;
    }
    lds_barrier();
    // every page of the current item is consumed: fetch the next item's descriptor and first pages now,
    // so that they travel while the rows are merged
    if constexpr (!UNITS) {
      const int next_k = __builtin_amdgcn_readfirstlane(s_next);
      nxt = load_desc_head<WAVES, NBUF>(P, next_k, n_items, wave, G);
      if (second_on_cu) keep_claiming = static_cast<int64_t>(next_k) * kSecondShare < n_items;
    }
    FMT::load_q(nxt, P, lane, G);
    prologue(nxt);
    for (int idx = threadIdx.x; idx < G * 32; idx += WAVES * 64) {
      const int q = idx >> 5, d4 = idx & 31;
      float M = sm_m[q];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) M = fmaxf(M, sm_m[w * 16 + q]);
      float L = 0.f;
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < WAVES; ++w) {
        const float wgt = __builtin_amdgcn_exp2f(sm_m[w * 16 + q] - M);   // a wave with no pages has m = -inf
        L += wgt * sm_l[w * 16 + q];
        o += wgt * *reinterpret_cast<const f32x4*>(sm_o + (w * 16 + q) * kORow + 4 * d4);
      }
      const float inv = 1.0f / L;
      *reinterpret_cast<f32x4*>(st_o + (staged + q) * fs::kHeadDim + 4 * d4) = o * inv;
      if (d4 == 0) {
        st_lse[staged + q] = (M + __builtin_amdgcn_logf(L)) * kLn2;
        st_row[staged + q] = cur.row >= 0 ? cur.row + q : cur.row - q;
      }
    }
    if (P.pair_counters != nullptr) {
      if (threadIdx.x == 0) {
        st_pair[staged_items] = cur.pair;
        st_chunks[staged_items] = cur.n_chunks;
        st_prow[staged_items] = cur.pair_row;
      }
      staged_split |= cur.n_chunks > 1;
    }
    ++staged_items;
    staged += G;
    lds_barrier();                     // staging rows complete; the merge buffers may be reused
    const bool last = !nxt.valid;
    if (last || staged + G > kStageRows) {
      for (int idx = threadIdx.x; idx < staged * 32; idx += WAVES * 64) {
        const int r = idx >> 5, d4 = idx & 31;
        const int row = st_row[r];
        float* dst = row >= 0 ? P.part_o + static_cast<int64_t>(row) * fs::kHeadDim : P.out + static_cast<int64_t>(-row - 1) * fs::kHeadDim;
        const f32x4 v = *reinterpret_cast<const f32x4*>(st_o + r * fs::kHeadDim + 4 * d4);
        if (row >= 0 && P.pair_counters != nullptr) store_f32x4_coherent(dst + 4 * d4, v);     // rows for arrive_and_merge
        else __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst + 4 * d4));
      }
      for (int r = threadIdx.x; r < staged; r += WAVES * 64) {
        const int row = st_row[r];
        if (row >= 0 && P.pair_counters != nullptr) store_f32_coherent(P.part_lse + row, st_lse[r]);
        else __builtin_nontemporal_store(st_lse[r], row >= 0 ? P.part_lse + row : P.lse + (-row - 1));
      }
      if (staged_split) arrive_and_merge<WAVES>(P, staged_items, st_pair, st_chunks, st_prow, st_done, G, wave, lane);
      staged = 0;
      staged_items = 0;
      staged_split = false;
      // the next write into the staging rows comes after the next item's first barrier, which every
      // thread reaches only when it is done reading them here
    }
    if (last) break;
    cur = nxt;
  }
  // The last workgroup to leave puts both counters back to zero for the next launch (every other
  // workgroup has made its last claim by then).
  if constexpr (!UNITS) {
    if (threadIdx.x == 0 && atomicAdd(claim + 1, 1) == static_cast<int>(gridDim.x) - 1) {
      __atomic_store_n(claim, 0, __ATOMIC_RELAXED);
      __atomic_store_n(claim + 1, 0, __ATOMIC_RELAXED);
    }
  }
}

// (two wavefronts per SIMD - two workgroups per CU - is what the launch counts on: at most 256 registers)
template <int WAVES, int NBUF, bool UNITS>
__global__ void __launch_bounds__(WAVES * 64, 2) decode_bf16_persistent_kernel(const DecodeParams P, int n_items,
                                                                            int* __restrict__ claim, int n_first,
                                                                            const int64_t* __restrict__ unit_indptr) {
  persistent_sweep<WAVES, NBUF, UNITS, Bf16Format>(P, n_items, claim, n_first, unit_indptr);
}
template <int WAVES, int NBUF, bool UNITS>
__global__ void __launch_bounds__(WAVES * 64, 2) decode_fp8_persistent_kernel(const DecodeParams P, int n_items,
                                                                           int* __restrict__ claim, int n_first,
                                                                           const int64_t* __restrict__ unit_indptr) {
  persistent_sweep<WAVES, NBUF, UNITS, Fp8Format>(P, n_items, claim, n_first, unit_indptr);
}

template <typename K>
fs_status launch(const char* who, K kernel, int threads, const DecodeParams& P, int64_t n_items, hipStream_t stream) {
  hipLaunchKernelGGL(kernel, dim3(static_cast<unsigned>(n_items)), dim3(threads), 0, stream, P);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fs::fail(FS_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
  return FS_OK;
}

// ---------------------------------------------------------------------------------------------
// Device memory of the entry point that allocates nothing (fs_decode_attention_fused_static): the
// persistent sweep's two counters and the partial rows of split pairs live in this array instead of
// in buffers the caller brings.  Every GPU the library runs on holds its own copy, at its own
// address, until the process ends.  Layout: [0, 256) counters | partial rows | their lse values.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the address
// that call returns.
// ---------------------------------------------------------------------------------------------
constexpr int64_t kStaticRows = 32768;                                            // partial rows it holds
constexpr int64_t kStaticOffO = 256;
constexpr int64_t kStaticOffLse = kStaticOffO + kStaticRows * fs::kHeadDim * 4;
constexpr int64_t kStaticBytes = kStaticOffLse + kStaticRows * 4;                 // 16 MiB + 128 KiB + 256 B
static __device__ __align__(256) unsigned char scratch[kStaticBytes];

__global__ void zero_counters_kernel(int* __restrict__ claim) {
  if (threadIdx.x < 2) claim[threadIdx.x] = 0;
}

// ---- host side -------------------------------------------------------------------------------

// Argument checks shared by the entry points.  `who` names the call in messages.  On FS_OK with
// n_items > 0, *P is ready for a launch (the fused fields are left NULL).
fs_status prepare(const char* who, const fs_shape* shape, const fs_kv_view* kv, const void* items_dev,
                  const int32_t* sched_dev, int64_t n_items, float* part_o, float* part_lse, bool partials_needed,
                  DecodeParams* P) {
  if (!shape || !kv) return fs::fail(FS_EINVAL, "%s: shape or kv is NULL", who);
  if (shape->n_kv_heads < 1 || shape->n_q_heads < shape->n_kv_heads || shape->n_q_heads % shape->n_kv_heads)
    return fs::fail(FS_EINVAL, "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, shape->n_q_heads,
                    shape->n_kv_heads);
  if (shape->head_dim != fs::kHeadDim)
    return fs::fail(FS_EUNSUPPORTED, "%s: head_dim %d (only %d is built)", who, shape->head_dim, fs::kHeadDim);
  if (shape->page_tokens != fs::kPageTokens)
    return fs::fail(FS_EUNSUPPORTED, "%s: page_tokens %d (only %d is built)", who, shape->page_tokens, fs::kPageTokens);
  const int G = shape->n_q_heads / shape->n_kv_heads;
  if (G > fs::kMaxGroup) return fs::fail(FS_EINVAL, "%s: group %d > %d", who, G, fs::kMaxGroup);
  if (n_items < 0 || n_items > 0x7FFFFFFF) return fs::fail(FS_EINVAL, "%s: n_items out of range", who);
  if (kv->kv_dtype != FS_KV_BF16 && kv->kv_dtype != FS_KV_FP8_E4M3)
    return fs::fail(FS_EINVAL, "%s: unknown kv_dtype %d", who, kv->kv_dtype);
  if (n_items == 0) return FS_OK;
  if (!kv->q || !kv->k_pool || !kv->v_pool || !kv->page_indptr || !kv->page_ids || !items_dev ||
      (partials_needed && (!part_o || !part_lse)))
    return fs::fail(FS_EINVAL, "%s: NULL device pointer", who);
  if (kv->kv_dtype == FS_KV_FP8_E4M3 && !kv->page_scales && (!kv->k_scale || !kv->v_scale))
    return fs::fail(FS_EINVAL, "%s: fp8 KV needs page_scales, or k_scale and v_scale", who);
  const int64_t slot_bytes = static_cast<int64_t>(fs::kPageTokens) * fs::kHeadDim * (kv->kv_dtype == FS_KV_BF16 ? 2 : 1);
  if (kv->k_slot_stride < slot_bytes || kv->v_slot_stride < slot_bytes || (kv->k_slot_stride & 15) ||
      (kv->v_slot_stride & 15) || (reinterpret_cast<uintptr_t>(kv->k_pool) & 15) ||
      (reinterpret_cast<uintptr_t>(kv->v_pool) & 15) || (reinterpret_cast<uintptr_t>(kv->q) & 15) ||
      (reinterpret_cast<uintptr_t>(part_o) & 15))
    return fs::fail(FS_EINVAL, "%s: pools, strides, q and part_o must be 16-byte aligned and strides at least one slot "
                               "(%lld bytes)", who, static_cast<long long>(slot_bytes));
  if (!std::isfinite(kv->sm_scale)) return fs::fail(FS_EINVAL, "%s: sm_scale is not finite", who);
  P->q = static_cast<const uint16_t*>(kv->q);
  P->k_pool = static_cast<const char*>(kv->k_pool);
  P->v_pool = static_cast<const char*>(kv->v_pool);
  P->k_stride = kv->k_slot_stride;
  P->v_stride = kv->v_slot_stride;
  P->k_scale = kv->page_scales ? kv->page_scales : kv->k_scale;
  P->v_scale = kv->page_scales ? kv->page_scales + 1 : kv->v_scale;
  P->scale_by_page = kv->page_scales ? 1 : 0;
  P->page_indptr = kv->page_indptr;
  P->page_ids = kv->page_ids;
  P->items = static_cast<const fs_work_item*>(items_dev);   // the records call puts its list into P->records afterwards
  P->sched = sched_dev;
  P->records = nullptr;
  P->part_o = part_o;
  P->part_lse = part_lse;
  P->chunk_indptr = nullptr;
  P->pair_counters = nullptr;
  P->out = nullptr;
  P->lse = nullptr;
  P->group = G;
  P->scale_log2 = kv->sm_scale * 1.4426950408889634f;
  return FS_OK;
}

// CU count of the current device, asked once per device (the query is a runtime call on the launch path).
fs_status device_cu_count(const char* who, int* n_cu_out) {
  static int cu_of_device[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
    return fs::fail(FS_EHIP, "%s: cannot identify the current device", who);
  int n_cu = cu_of_device[dev];
  if (n_cu == 0) {
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
      return fs::fail(FS_EHIP, "%s: cannot read the device's CU count", who);
    cu_of_device[dev] = n_cu;      // racing first calls write the same value
  }
  *n_cu_out = n_cu;
  return FS_OK;
}

// One workgroup per item, in the launch shape the options select.
fs_status launch_plain(const char* who, const DecodeParams& P, int kv_dtype, int64_t n_items, hipStream_t s) {
  const int waves = fs::options().waves_per_group;
  const int nbuf = fs::options().prefetch_pages + 1;

#define FS_PICK(KERNEL)                                                                  \
  switch (waves * 10 + nbuf) {                                                           \
    case 12: return launch(who, KERNEL<1, 2>, 64, P, n_items, s);                        \
    case 13: return launch(who, KERNEL<1, 3>, 64, P, n_items, s);                        \
    case 14: return launch(who, KERNEL<1, 4>, 64, P, n_items, s);                        \
    case 22: return launch(who, KERNEL<2, 2>, 128, P, n_items, s);                       \
    case 23: return launch(who, KERNEL<2, 3>, 128, P, n_items, s);                       \
    case 24: return launch(who, KERNEL<2, 4>, 128, P, n_items, s);                       \
    case 42: return launch(who, KERNEL<4, 2>, 256, P, n_items, s);                       \
    case 43: return launch(who, KERNEL<4, 3>, 256, P, n_items, s);                       \
    case 44: return launch(who, KERNEL<4, 4>, 256, P, n_items, s);                       \
    default: return fs::fail(FS_EINVAL, "%s: no kernel for waves_per_group %d, prefetch_pages %d", who, waves, nbuf - 1); \
  }

  if (kv_dtype == FS_KV_BF16) {
    FS_PICK(decode_bf16_kernel)
  }
  FS_PICK(decode_fp8_kernel)
#undef FS_PICK
}

// Resident workgroups, for either K/V format.  unit_indptr_dev NULL: `groups` workgroups claim items from claim_dev
// (n_first of them the first on their CU); else workgroup u walks the items of run u.
fs_status launch_resident(const char* who, const DecodeParams& P, int kv_dtype, int64_t groups, int64_t n_items,
                          int32_t* claim_dev, int n_first, const int64_t* unit_indptr_dev, hipStream_t s) {
  const dim3 grid(static_cast<unsigned>(groups)), block(256);
  const int n = static_cast<int>(n_items);
  if (kv_dtype == FS_KV_BF16) {
    if (unit_indptr_dev)
      hipLaunchKernelGGL((decode_bf16_persistent_kernel<4, 3, true>), grid, block, 0, s, P, n, claim_dev, n_first, unit_indptr_dev);
    else
      hipLaunchKernelGGL((decode_bf16_persistent_kernel<4, 3, false>), grid, block, 0, s, P, n, claim_dev, n_first, unit_indptr_dev);
  } else {
    if (unit_indptr_dev)
      hipLaunchKernelGGL((decode_fp8_persistent_kernel<4, 3, true>), grid, block, 0, s, P, n, claim_dev, n_first, unit_indptr_dev);
    else
      hipLaunchKernelGGL((decode_fp8_persistent_kernel<4, 3, false>), grid, block, 0, s, P, n, claim_dev, n_first, unit_indptr_dev);
  }
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fs::fail(FS_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
  return FS_OK;
}

// The persistent form: two resident workgroups per CU claim items from claim_dev.
fs_status launch_persistent(const char* who, const DecodeParams& P, int kv_dtype, int64_t n_items, int32_t* claim_dev,
                            hipStream_t s) {
  int n_cu = 0;
  if (const fs_status st = device_cu_count(who, &n_cu); st != FS_OK) return st;
  return launch_resident(who, P, kv_dtype, std::min<int64_t>(n_items, 2ll * n_cu), n_items, claim_dev, n_cu, nullptr, s);
}

}  // namespace

extern "C" fs_status fs_decode_attention(const fs_shape* shape, const fs_kv_view* kv,
                                         const fs_work_item* items_dev, const int32_t* sched_dev,
                                         int64_t n_items, float* part_o, float* part_lse, void* stream) {
  DecodeParams P;
  if (const fs_status st = prepare("fs_decode_attention", shape, kv, items_dev, sched_dev, n_items, part_o, part_lse,
                                   true, &P); st != FS_OK || n_items == 0)
    return st;
  return launch_plain("fs_decode_attention", P, kv->kv_dtype, n_items, static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_decode_attention_persistent(const fs_shape* shape, const fs_kv_view* kv,
                                                    const fs_work_item* items_dev, const int32_t* sched_dev,
                                                    int64_t n_items, int32_t* claim_dev, float* part_o,
                                                    float* part_lse, void* stream) {
  DecodeParams P;
  if (const fs_status st = prepare("fs_decode_attention_persistent", shape, kv, items_dev, sched_dev, n_items, part_o,
                                   part_lse, true, &P); st != FS_OK || n_items == 0)
    return st;
  if (!claim_dev || (reinterpret_cast<uintptr_t>(claim_dev) & 7))
    return fs::fail(FS_EINVAL, "fs_decode_attention_persistent: claim_dev is NULL or not 8-byte aligned");
  return launch_persistent("fs_decode_attention_persistent", P, kv->kv_dtype, n_items, claim_dev, static_cast<hipStream_t>(stream));
}

extern "C" fs_status fs_decode_attention_fused(const fs_shape* shape, const fs_kv_view* kv,
                                               const fs_work_item* items_dev, const int32_t* sched_dev, int64_t n_items,
                                               const int64_t* chunk_indptr_dev, int64_t n_pairs, float* part_o,
                                               float* part_lse, int32_t* claim_dev, float* out, float* lse,
                                               void* stream) {
  const char* who = "fs_decode_attention_fused";
  if (n_pairs < 0 || n_pairs > n_items) return fs::fail(FS_EINVAL, "%s: n_pairs %lld outside [0, n_items]", who,
                                                        static_cast<long long>(n_pairs));
  const bool split = n_items > n_pairs;            // some pair has more than one item: partial rows and a merge
  DecodeParams P;
  if (const fs_status st = prepare(who, shape, kv, items_dev, sched_dev, n_items, part_o, part_lse, split, &P);
      st != FS_OK || n_items == 0)
    return st;
  if (n_pairs == 0) return fs::fail(FS_EINVAL, "%s: %lld items but no pairs", who, static_cast<long long>(n_items));
  if (!chunk_indptr_dev || !out || !lse || (reinterpret_cast<uintptr_t>(out) & 15))
    return fs::fail(FS_EINVAL, "%s: chunk_indptr_dev, out or lse is NULL, or out is not 16-byte aligned", who);
  if (claim_dev && (reinterpret_cast<uintptr_t>(claim_dev) & 7))
    return fs::fail(FS_EINVAL, "%s: claim_dev is not 8-byte aligned", who);
  P.chunk_indptr = chunk_indptr_dev;
  P.out = out;
  P.lse = lse;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // The persistent form pays once every resident workgroup walks several items; below that it is the same
  // work plus a counter.
  // (bf16 only: with fp8 K/V the resident forms measure no faster than one workgroup per item)
  const bool persistent = claim_dev && kv->kv_dtype == FS_KV_BF16 && n_items >= fs::kPersistentMinItems;
  const fs_status st = persistent ? launch_persistent(who, P, kv->kv_dtype, n_items, claim_dev, s)
                                  : launch_plain(who, P, kv->kv_dtype, n_items, s);
  if (st != FS_OK || !split) return st;
  return fs::merge_lse_launch(who, part_o, part_lse, chunk_indptr_dev, n_pairs, P.group, out, lse, /*skip_single=*/true, s);
}

extern "C" fs_status fs_decode_attention_units(const fs_shape* shape, const fs_kv_view* kv,
                                               const fs_work_item* items_dev, int64_t n_items,
                                               const int64_t* unit_indptr_dev, int64_t n_units,
                                               const int64_t* chunk_indptr_dev, int64_t n_pairs,
                                               float* part_o, float* part_lse, float* out, float* lse, void* stream) {
  const char* who = "fs_decode_attention_units";
  const bool partials_only = chunk_indptr_dev == nullptr;      // every item's rows to part_o / part_lse, no merge
  if (!partials_only && (n_pairs < 0 || n_pairs > n_items))
    return fs::fail(FS_EINVAL, "%s: n_pairs %lld outside [0, n_items]", who, static_cast<long long>(n_pairs));
  if (n_units < 0 || n_units > n_items) return fs::fail(FS_EINVAL, "%s: n_units %lld outside [0, n_items]", who,
                                                        static_cast<long long>(n_units));
  const bool split = partials_only || n_items > n_pairs;
  DecodeParams P;
  if (const fs_status st = prepare(who, shape, kv, items_dev, nullptr, n_items, part_o, part_lse, split, &P);
      st != FS_OK || n_items == 0)
    return st;
  if (n_units == 0 || (!partials_only && n_pairs == 0))
    return fs::fail(FS_EINVAL, "%s: %lld items but no pairs or no units", who, static_cast<long long>(n_items));
  if (!unit_indptr_dev) return fs::fail(FS_EINVAL, "%s: unit_indptr_dev is NULL", who);
  if (!partials_only && (!out || !lse || (reinterpret_cast<uintptr_t>(out) & 15)))
    return fs::fail(FS_EINVAL, "%s: out or lse is NULL, or out is not 16-byte aligned", who);
  if (!partials_only) {
    P.chunk_indptr = chunk_indptr_dev;
    P.out = out;
    P.lse = lse;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (const fs_status st = launch_resident(who, P, kv->kv_dtype, n_units, n_items, nullptr, 0, unit_indptr_dev, s); st != FS_OK)
    return st;
  if (partials_only || n_items == n_pairs) return FS_OK;
  return fs::merge_lse_launch(who, part_o, part_lse, chunk_indptr_dev, n_pairs, P.group, out, lse, /*skip_single=*/true, s);
}

extern "C" fs_status fs_decode_attention_records(const fs_shape* shape, const fs_kv_view* kv,
                                                 const fs_launch_record* records_dev, int64_t n_items,
                                                 const int64_t* unit_indptr_dev, int64_t n_units,
                                                 const int64_t* chunk_indptr_dev, int64_t n_pairs,
                                                 float* part_o, float* part_lse, float* out, float* lse,
                                                 int32_t* pair_counters_dev, int32_t* claim_dev, void* stream) {
  const char* who = "fs_decode_attention_records";
  const bool sweep_only = chunk_indptr_dev == nullptr;     // no merge: the rows go where the records say
  if (sweep_only && pair_counters_dev)
    return fs::fail(FS_EINVAL, "%s: pair_counters_dev without chunk_indptr_dev (a sweep that merges nothing needs no counters)", who);
  if (!sweep_only && (n_pairs < 0 || n_pairs > n_items))
    return fs::fail(FS_EINVAL, "%s: n_pairs %lld outside [0, n_items]", who, static_cast<long long>(n_pairs));
  const bool units = unit_indptr_dev != nullptr;
  if (units && (n_units < 0 || n_units > n_items))
    return fs::fail(FS_EINVAL, "%s: n_units %lld outside [0, n_items]", who, static_cast<long long>(n_units));
  if (claim_dev && units)
    return fs::fail(FS_EINVAL, "%s: claim_dev with unit_indptr_dev (equal runs are not claimed)", who);
  if (claim_dev && (reinterpret_cast<uintptr_t>(claim_dev) & 7))
    return fs::fail(FS_EINVAL, "%s: claim_dev is not 8-byte aligned", who);
  const bool split = sweep_only || n_items > n_pairs;
  DecodeParams P;
  if (const fs_status st = prepare(who, shape, kv, records_dev, nullptr, n_items, part_o, part_lse, split, &P);
      st != FS_OK || n_items == 0)
    return st;
  if ((!sweep_only && n_pairs == 0) || (units && n_units == 0))
    return fs::fail(FS_EINVAL, "%s: %lld items but no pairs or no units", who, static_cast<long long>(n_items));
  if (!out || !lse || (reinterpret_cast<uintptr_t>(out) & 15) || (reinterpret_cast<uintptr_t>(records_dev) & 7))
    return fs::fail(FS_EINVAL, "%s: out or lse is NULL, out is not 16-byte or records_dev not 8-byte aligned", who);
  P.items = nullptr;
  P.records = records_dev;
  P.out = out;
  P.lse = lse;
  const bool merge_in_sweep = pair_counters_dev != nullptr && n_items > n_pairs;
  if (merge_in_sweep) {
    if (reinterpret_cast<uintptr_t>(pair_counters_dev) & 3)
      return fs::fail(FS_EINVAL, "%s: pair_counters_dev is not 4-byte aligned", who);
    if (n_pairs * P.group > 0x7FFFFFFFll) return fs::fail(FS_EINVAL, "%s: n_pairs out of range", who);
    P.pair_counters = pair_counters_dev;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  fs_status st = FS_OK;
  if (units) {
    st = launch_resident(who, P, kv->kv_dtype, n_units, n_items, nullptr, 0, unit_indptr_dev, s);
  } else if (claim_dev) {
    st = launch_persistent(who, P, kv->kv_dtype, n_items, claim_dev, s);
  } else {
    st = launch_plain(who, P, kv->kv_dtype, n_items, s);
  }
  if (st != FS_OK || sweep_only || n_items == n_pairs || merge_in_sweep) return st;
  return fs::merge_lse_launch(who, part_o, part_lse, chunk_indptr_dev, n_pairs, P.group, out, lse, /*skip_single=*/true, s);
}

extern "C" fs_status fs_decode_attention_fused_static(const fs_shape* shape, const fs_kv_view* kv,
                                                      const fs_work_item* items_dev, const int32_t* sched_dev,
                                                      int64_t n_items, const int64_t* chunk_indptr_dev,
                                                      int64_t n_pairs, float* out, float* lse, void* stream) {
  const char* who = "fs_decode_attention_fused_static";
  if (n_pairs < 0 || n_pairs > n_items) return fs::fail(FS_EINVAL, "%s: n_pairs %lld outside [0, n_items]", who,
                                                        static_cast<long long>(n_pairs));
  const bool split = n_items > n_pairs;
  DecodeParams P;
  if (const fs_status st = prepare(who, shape, kv, items_dev, sched_dev, n_items, nullptr, nullptr, false, &P);
      st != FS_OK || n_items == 0)
    return st;
  if (n_pairs == 0) return fs::fail(FS_EINVAL, "%s: %lld items but no pairs", who, static_cast<long long>(n_items));
  if (!chunk_indptr_dev || !out || !lse || (reinterpret_cast<uintptr_t>(out) & 15))
    return fs::fail(FS_EINVAL, "%s: chunk_indptr_dev, out or lse is NULL, or out is not 16-byte aligned", who);
  if (split && n_items * P.group > kStaticRows)
    return fs::fail(FS_ECAPACITY, "%s: a split list of %lld items x %d q-heads needs %lld partial rows, the static "
                                  "array holds %lld; use fs_decode_attention_fused with buffers of your own", who,
                    static_cast<long long>(n_items), P.group, static_cast<long long>(n_items * P.group),
                    static_cast<long long>(kStaticRows));
  // The array's address on the current device, asked once per device with that device current.
  static unsigned char* base_of_device[64] = {};
  static std::mutex lock;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
    return fs::fail(FS_EHIP, "%s: cannot identify the current device", who);
  unsigned char* base = nullptr;
  {
    std::lock_guard<std::mutex> hold(lock);
    base = base_of_device[dev];
    if (!base) {
      void* p = nullptr;
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return fs::fail(FS_EHIP, "%s: cannot resolve the static array on device %d: %s", who, dev, hipGetErrorString(e));
      base = base_of_device[dev] = static_cast<unsigned char*>(p);
    }
  }
  int32_t* claim = reinterpret_cast<int32_t*>(base);
  P.part_o = reinterpret_cast<float*>(base + kStaticOffO);
  P.part_lse = reinterpret_cast<float*>(base + kStaticOffLse);
  P.chunk_indptr = chunk_indptr_dev;
  P.out = out;
  P.lse = lse;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool persistent = kv->kv_dtype == FS_KV_BF16 && n_items >= fs::kPersistentMinItems;
  fs_status st;
  if (persistent) {
    // The array keeps what the last call left.  A completed sweep leaves its counters at zero, but this
    // call does not rest on that: it clears them itself (a fill kernel, which a captured graph replays
    // faithfully).
    hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, s, claim);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fs::fail(FS_EHIP, "%s: launch failed: %s", who, hipGetErrorString(e));
    st = launch_persistent(who, P, kv->kv_dtype, n_items, claim, s);
  } else {
    st = launch_plain(who, P, kv->kv_dtype, n_items, s);
  }
  if (st != FS_OK || !split) return st;
  return fs::merge_lse_launch(who, P.part_o, P.part_lse, chunk_indptr_dev, n_pairs, P.group, out, lse, /*skip_single=*/true, s);
}
