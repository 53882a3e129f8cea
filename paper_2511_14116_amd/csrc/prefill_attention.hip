// fs_prefill_attention: chunked-prefill attention over the paged KVCache, gfx950 only.
//
// The paper's fine-grained chunked prefill (Section 3.1) puts chunks of several requests into
// one batch: N new tokens of a request behind L processed ones.  Every new token attends to the
// cache up to and including itself (prefill phase, Section 2.1.1).  The paper describes no
// kernel; this one is built on the decode kernel's slot layout, which already puts K and V
// pages into matrix-core operand order.
//
// One workgroup per tile of query tokens of one (request, KV head) pair.  A query row is a
// (token, q-head of the group) combination; 16 rows form a column tile of the transposed score
// matrix, and every wavefront owns CT column tiles.  Per pair of KV pages (32 tokens) a
// wavefront loads K and V once (16-byte loads straight into operand registers) and reuses them
// for all its column tiles:
//     S^T[tok][row] = K . Q^T        2 x 4 v_mfma_f32_16x16x32_bf16 per column tile
//     online softmax in fp32, log2 domain, causal mask only on the pages that straddle a row's position
//     O^T[d][row]  += V^T . P^T      8 x v_mfma_f32_16x16x32_bf16 over the 32 tokens, P as bf16 hi + lo
// The S^T accumulators of the two pages are, lane by lane, the 8 reduction elements the second
// product wants from P^T, and the V registers of the two pages pair up the same way, so nothing
// crosses lanes except the running max.  This is a dense contraction (G*N rows against L+N
// keys): the matrix cores bound it, not HBM.
#include <hip/hip_runtime.h>

#include <cmath>

#include "fs_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct PrefillParams {
  const uint16_t* __restrict__ q;
  const char* __restrict__ k_pool;
  const char* __restrict__ v_pool;
  int64_t k_stride;
  int64_t v_stride;
  const int64_t* __restrict__ page_indptr;
  const int32_t* __restrict__ page_ids;
  const fs_prefill_item* __restrict__ items;
  const int32_t* __restrict__ sched;
  float* __restrict__ out;
  float* __restrict__ lse;
  int32_t group;        // G
  int32_t group_pad;    // G rounded up to a power of two (divides 16)
  int32_t n_q_heads;
  float scale_log2;
};

constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float xor16(float v, bool take_max) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  return take_max ? fmaxf(__uint_as_float(a), __uint_as_float(b)) : __uint_as_float(a) + __uint_as_float(b);
}
__device__ __forceinline__ float xor32(float v, bool take_max) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  return take_max ? fmaxf(__uint_as_float(a), __uint_as_float(b)) : __uint_as_float(a) + __uint_as_float(b);
}

// Two KV pages (32 tokens) in operand registers.  The second product reduces over the 32 tokens of
// the pair, and a lane's 8 reduction elements are 4 tokens of the first page followed by the same 4
// of the second, so each V operand is filled by one 8-byte load from either page.
struct PagePair {
  u32x4 k[2][4];   // [page][32-d block]: A operand of K.Q^T
  u32x4 va[4];     // [32-d block], d = 32c + lane%16:      (page 0 tokens 4kb..4kb+3, page 1 tokens 4kb..4kb+3)
  u32x4 vb[4];     // [32-d block], d = 32c + 16 + lane%16: likewise
};

__device__ __forceinline__ void load_pair(PagePair& r, const PrefillParams& P, const int32_t* __restrict__ ids,
                                          int page0, int n_pages, int lane) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    if (page0 + h < n_pages) {
      const int64_t slot = ids[page0 + h];
      const u32x4* kp = reinterpret_cast<const u32x4*>(P.k_pool + slot * P.k_stride) + lane;
      const uint2* vp = reinterpret_cast<const uint2*>(P.v_pool + slot * P.v_stride) + 2 * lane;
#pragma unroll
      for (int s = 0; s < 4; ++s) r.k[h][s] = kp[s * 64];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint2 a = vp[s * 128], b = vp[s * 128 + 1];
        if (h == 0) { r.va[s].x = a.x; r.va[s].y = a.y; r.vb[s].x = b.x; r.vb[s].y = b.y; }
        else        { r.va[s].z = a.x; r.va[s].w = a.y; r.vb[s].z = b.x; r.vb[s].w = b.y; }
      }
    } else {   // no such page: its keys are masked, its values must be finite
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        r.k[h][s] = u32x4{0u, 0u, 0u, 0u};
        if (h == 0) { r.va[s].x = 0u; r.va[s].y = 0u; r.vb[s].x = 0u; r.vb[s].y = 0u; }
        else        { r.va[s].z = 0u; r.va[s].w = 0u; r.vb[s].z = 0u; r.vb[s].w = 0u; }
      }
    }
  }
}

// Blank the value rows of tokens at or beyond valid0 (page 0) / valid1 (page 1), each 0..16: whatever
// bits sit in the unused tail of a last page (NaN included) must not reach the product, where
// 0 * NaN is NaN.
__device__ __forceinline__ void blank_values(PagePair& r, int valid0, int valid1, int kb) {
  const uint32_t a0 = (4 * kb + 0 < valid0 ? 0x0000FFFFu : 0u) | (4 * kb + 1 < valid0 ? 0xFFFF0000u : 0u);
  const uint32_t a1 = (4 * kb + 2 < valid0 ? 0x0000FFFFu : 0u) | (4 * kb + 3 < valid0 ? 0xFFFF0000u : 0u);
  const uint32_t b0 = (4 * kb + 0 < valid1 ? 0x0000FFFFu : 0u) | (4 * kb + 1 < valid1 ? 0xFFFF0000u : 0u);
  const uint32_t b1 = (4 * kb + 2 < valid1 ? 0x0000FFFFu : 0u) | (4 * kb + 3 < valid1 ? 0xFFFF0000u : 0u);
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    r.va[c].x &= a0; r.va[c].y &= a1; r.va[c].z &= b0; r.va[c].w &= b1;
    r.vb[c].x &= a0; r.vb[c].y &= a1; r.vb[c].z &= b0; r.vb[c].w &= b1;
  }
}

struct TileState {
  float m;          // running max (log2 domain) of this lane's query row
  float l;          // this lane's share of the running sum
  f32x4 acc[8];     // O^T[d = 16b + 4*(lane/16) + r][row = lane%16]
};

// One column tile against one page pair.  `pos` is the last key this lane's row may see; `t0` the
// first token of the pair.
template <bool MASK>
__device__ __forceinline__ void consume_pair(TileState& st, const PagePair& pg, const bf16x8 (&qreg)[4],
                                             float scale_log2, int t0, int pos, int kb) {
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pg.k[0][c]), qreg[c], sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pg.k[1][c]), qreg[c], sb, 0, 0, 0);
  }
  float x[8];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    x[r] = sa[r] * scale_log2;
    x[4 + r] = sb[r] * scale_log2;
  }
  if (MASK) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (t0 + 4 * kb + r > pos) x[r] = -INFINITY;
      if (t0 + 16 + 4 * kb + r > pos) x[4 + r] = -INFINITY;
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  mx = xor32(xor16(mx, true), true);
  const float m_new = fmaxf(st.m, mx);     // finite from the first pair on: token 0 is visible to every row
  if (__any(m_new > st.m)) {
    const float alpha = __builtin_amdgcn_exp2f(st.m - m_new);   // first pair: exp2(-inf) = 0
    st.l *= alpha;
#pragma unroll
    for (int j = 0; j < 8; ++j) st.acc[j] *= alpha;
    st.m = m_new;
  }
  float p[8];
  float ps = 0.f;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    p[r] = __builtin_amdgcn_exp2f(x[r] - st.m);
    ps += p[r];
  }
  st.l += ps;
  // weights as bf16 hi + lo (16 significant bits), as in the decode kernel
  bf16x8 ph, pl;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    ph[r] = static_cast<__bf16>(p[r]);
    pl[r] = static_cast<__bf16>(p[r] - static_cast<float>(ph[r]));
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const bf16x8 va = __builtin_bit_cast(bf16x8, pg.va[c]), vb = __builtin_bit_cast(bf16x8, pg.vb[c]);
    st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, ph, st.acc[2 * c], 0, 0, 0);
    st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb, ph, st.acc[2 * c + 1], 0, 0, 0);
    st.acc[2 * c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pl, st.acc[2 * c], 0, 0, 0);
    st.acc[2 * c + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb, pl, st.acc[2 * c + 1], 0, 0, 0);
  }
}

template <int WAVES, int CT>
__global__ void __launch_bounds__(WAVES * 64) prefill_bf16_kernel(const PrefillParams P) {
  const int item_idx = P.sched ? P.sched[blockIdx.x] : static_cast<int>(blockIdx.x);
  const fs_prefill_item it = P.items[item_idx];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int col = lane & 15, kb = lane >> 4;
  const int G = P.group, Gp = P.group_pad;
  const int tpc = 16 / Gp;                       // query tokens per column tile
  const int n_tok = it.q_end - it.q_begin;       // query tokens of this item
  const int tok0 = wave * CT * tpc;              // first token (within the item) of this wavefront
  if (tok0 >= n_tok) return;                     // nothing for this wavefront (short last tile); no barriers below
  const int ctx = it.n_done + it.q_end;          // keys that exist as far as this item is concerned
  const int L0 = it.n_done + it.q_begin;         // position of the item's first token

  // this lane's row of each column tile
  const int g = col % Gp, tl = col / Gp;
  bf16x8 qreg[CT][4];
  int pos[CT];
  bool live[CT];
#pragma unroll
  for (int t = 0; t < CT; ++t) {
    const int tok = tok0 + t * tpc + tl;                  // within the item
    live[t] = tok < n_tok && g < G;
    pos[t] = min(L0 + tok, ctx - 1);                      // rows that do not exist look at valid keys only
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
    st[t].l = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) st[t].acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  const int tok_last = min(n_tok, tok0 + CT * tpc) - 1;   // last token of this wavefront
  const int pos_last = L0 + tok_last;
  const int n_pages = pos_last / fs::kPageTokens + 1;     // pages this wavefront needs
  const int n_pairs = (n_pages + 1) / 2;
  const int32_t* __restrict__ ids = P.page_ids + P.page_indptr[it.pair];

  PagePair buf[2];
  load_pair(buf[0], P, ids, 0, n_pages, lane);
  for (int j = 0; j < n_pairs; j += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int jj = j + u;
      if (jj < n_pairs) {
        if (jj + 1 < n_pairs) load_pair(buf[u ^ 1], P, ids, 2 * (jj + 1), n_pages, lane);
        PagePair& pg = buf[u];
        const int t0 = 32 * jj;
        if (t0 + 32 > ctx) {          // the cache ends inside this pair: blank what lies beyond it
          blank_values(pg, min(16, max(0, ctx - t0)), min(16, max(0, ctx - t0 - 16)), kb);
        }
#pragma unroll
        for (int t = 0; t < CT; ++t) {
          const int first_pos = L0 + tok0 + t * tpc;                       // smallest position in the column tile
          const int last_pos = min(L0 + tok0 + t * tpc + tpc - 1, ctx - 1);  // largest
          if (tok0 + t * tpc < n_tok && t0 <= last_pos) {
            if (t0 + 31 <= first_pos) consume_pair<false>(st[t], pg, qreg[t], P.scale_log2, t0, pos[t], kb);
            else consume_pair<true>(st[t], pg, qreg[t], P.scale_log2, t0, pos[t], kb);
          }
        }
      }
    }
  }

#pragma unroll
  for (int t = 0; t < CT; ++t) {
    const float l_tot = xor32(xor16(st[t].l, false), false);
    if (live[t]) {
      const int tok = tok0 + t * tpc + tl;
      const int64_t row = static_cast<int64_t>(it.out_row) + static_cast<int64_t>(tok) * G + g;
      const float inv = 1.0f / l_tot;
      float* o = P.out + row * fs::kHeadDim + 4 * kb;
#pragma unroll
      for (int b = 0; b < 8; ++b) *reinterpret_cast<f32x4*>(o + 16 * b) = st[t].acc[b] * inv;
      if (kb == 0) P.lse[row] = (st[t].m + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
  }
}

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

extern "C" fs_status fs_prefill_attention(const fs_shape* shape, const fs_kv_view* kv,
                                          const fs_prefill_item* items_dev, const int32_t* sched_dev,
                                          int64_t n_items, int32_t tile_tokens, float* out, float* lse,
                                          void* stream) {
  if (!shape || !kv) return fs::fail(FS_EINVAL, "fs_prefill_attention: shape or kv is NULL");
  if (shape->n_kv_heads < 1 || shape->n_q_heads < shape->n_kv_heads || shape->n_q_heads % shape->n_kv_heads)
    return fs::fail(FS_EINVAL, "fs_prefill_attention: n_q_heads %d is not a multiple of n_kv_heads %d",
                    shape->n_q_heads, shape->n_kv_heads);
  if (shape->head_dim != fs::kHeadDim)
    return fs::fail(FS_EUNSUPPORTED, "fs_prefill_attention: head_dim %d (only %d is built)", shape->head_dim, fs::kHeadDim);
  if (shape->page_tokens != fs::kPageTokens)
    return fs::fail(FS_EUNSUPPORTED, "fs_prefill_attention: page_tokens %d (only %d is built)", shape->page_tokens,
                    fs::kPageTokens);
  const int G = shape->n_q_heads / shape->n_kv_heads;
  if (G > fs::kMaxGroup) return fs::fail(FS_EINVAL, "fs_prefill_attention: group %d > %d", G, fs::kMaxGroup);
  if (kv->kv_dtype != FS_KV_BF16)
    return fs::fail(FS_EUNSUPPORTED, "fs_prefill_attention: only bf16 K/V is built (kv_dtype %d)", kv->kv_dtype);
  if (n_items < 0 || n_items > 0x7FFFFFFF) return fs::fail(FS_EINVAL, "fs_prefill_attention: n_items out of range");
  const int ct = fs::options().prefill_col_tiles, waves = fs::options().prefill_waves;
  const int cap = waves * ct * (16 / pad_group(G));
  if (tile_tokens < 1 || tile_tokens > cap)
    return fs::fail(FS_EINVAL, "fs_prefill_attention: tile_tokens %d outside [1, %d] for group %d", tile_tokens, cap, G);
  if (n_items == 0) return FS_OK;
  if (!kv->q || !kv->k_pool || !kv->v_pool || !kv->page_indptr || !kv->page_ids || !items_dev || !out || !lse)
    return fs::fail(FS_EINVAL, "fs_prefill_attention: NULL device pointer");
  const int64_t slot_bytes = static_cast<int64_t>(fs::kPageTokens) * fs::kHeadDim * 2;
  if (kv->k_slot_stride < slot_bytes || kv->v_slot_stride < slot_bytes || (kv->k_slot_stride & 15) ||
      (kv->v_slot_stride & 15) || (reinterpret_cast<uintptr_t>(kv->k_pool) & 15) ||
      (reinterpret_cast<uintptr_t>(kv->v_pool) & 15) || (reinterpret_cast<uintptr_t>(kv->q) & 15) ||
      (reinterpret_cast<uintptr_t>(out) & 15))
    return fs::fail(FS_EINVAL, "fs_prefill_attention: pools, strides, q and out must be 16-byte aligned and strides "
                               "at least one slot (%lld bytes)", static_cast<long long>(slot_bytes));
  if (!std::isfinite(kv->sm_scale)) return fs::fail(FS_EINVAL, "fs_prefill_attention: sm_scale is not finite");

  PrefillParams P;
  P.q = static_cast<const uint16_t*>(kv->q);
  P.k_pool = static_cast<const char*>(kv->k_pool);
  P.v_pool = static_cast<const char*>(kv->v_pool);
  P.k_stride = kv->k_slot_stride;
  P.v_stride = kv->v_slot_stride;
  P.page_indptr = kv->page_indptr;
  P.page_ids = kv->page_ids;
  P.items = items_dev;
  P.sched = sched_dev;
  P.out = out;
  P.lse = lse;
  P.group = G;
  P.group_pad = pad_group(G);
  P.n_q_heads = shape->n_q_heads;
  P.scale_log2 = kv->sm_scale * 1.4426950408889634f;
  hipStream_t s = static_cast<hipStream_t>(stream);
  switch (waves * 10 + ct) {
    case 41: return launch(prefill_bf16_kernel<4, 1>, 256, P, n_items, s);
    case 42: return launch(prefill_bf16_kernel<4, 2>, 256, P, n_items, s);
    case 44: return launch(prefill_bf16_kernel<4, 4>, 256, P, n_items, s);
    case 81: return launch(prefill_bf16_kernel<8, 1>, 512, P, n_items, s);
    case 82: return launch(prefill_bf16_kernel<8, 2>, 512, P, n_items, s);
    default: return fs::fail(FS_EINVAL, "fs_prefill_attention: no kernel for prefill_waves %d, prefill_col_tiles %d", waves, ct);
  }
}
