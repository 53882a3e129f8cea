// The split-K merge of one wavefront's output rows, shared by merge_lse_kernel and by the decode kernels that
// merge a pair themselves (the workgroup that writes a pair's last partial rows).  One definition, so both
// leave the same bits.
//
// Exact algebra on the partial (out, lse) pairs of a pair's chunks:
//     lse = ln sum_c exp(lse_c),   out = sum_c exp(lse_c - lse) * o_c.
#pragma once
#include <hip/hip_runtime.h>

#include "fs_internal.h"

namespace fs_merge {

static __device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
static __device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// Loads of partial rows.  COHERENT: as relaxed atomic loads at device scope, which are served from memory and not from
// this XCD's caches - for a caller that reads rows other workgroups of the same launch have written (the rows
// must have been stored the same way, see the decode kernels).
template <bool COHERENT>
static __device__ __forceinline__ float load_f32(const float* p) {
  if constexpr (COHERENT) return __hip_atomic_load(const_cast<float*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}
template <bool COHERENT>
static __device__ __forceinline__ float2 load_f32x2(const float2* p) {
  if constexpr (COHERENT) {
    const unsigned long long v = __hip_atomic_load(reinterpret_cast<unsigned long long*>(const_cast<float2*>(p)),
                                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float(static_cast<unsigned>(v)), __uint_as_float(static_cast<unsigned>(v >> 32)));
  } else {
    return *p;
  }
}

// RW consecutive output rows of one pair, by one wavefront.  The pair's chunks are c0 .. c0+n-1; chunk c's partial
// row of q-head g is row (c0 + c)*group + g of part_o / part_lse.  The rows merged are q-heads g0 .. g0+RW-1;
// out_rows / lse_rows point at the first of them in the final arrays.  A lane owns two of the 128 columns.
template <int RW, bool COHERENT = false>
static __device__ __forceinline__ void merge_rows(const float* part_o, const float* part_lse, int64_t c0, int n, int group,
                                                  int g0, float* out_rows, float* lse_rows, int lane) {
  // no fusing of multiplies into adds beyond the fmaf calls written out: every kernel that includes this must
  // round alike
#pragma clang fp contract(off)
  constexpr int U = RW == 1 ? 4 : 2;               // chunk rows in flight per output row
  // Chunks are taken 64 at a time (one lse per lane).  The first rows of a batch are requested before
  // its weights are known, so the two reads travel together; across batches (more than 64 chunks) the
  // running maximum moves and what has been summed is rescaled, as in an online softmax.
  float M[RW], sum[RW];
  float2 acc[RW];
#pragma unroll
  for (int r = 0; r < RW; ++r) { M[r] = -INFINITY; sum[r] = 0.f; acc[r] = make_float2(0.f, 0.f); }
  const int64_t stride = static_cast<int64_t>(group) * (fs::kHeadDim / 2);   // float2 units between chunk rows
  for (int base = 0; base < n; base += 64) {
    const int c = base + lane;
    const int cnt = min(64, n - base);
    float lv[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) lv[r] = c < n ? load_f32<COHERENT>(part_lse + (c0 + c) * group + g0 + r) : -INFINITY;
    // row r of chunk base+j: rows[j * stride + r * 64]
    const float2* rows = reinterpret_cast<const float2*>(part_o + ((c0 + base) * group + g0) * fs::kHeadDim) + lane;
    float2 o[U][RW];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < RW; ++r) o[u][r] = load_f32x2<COHERENT>(rows + min(u, cnt - 1) * stride + r * 64);   // the batch's first rows (repeats if it has fewer)
    float w[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
      const float Mb = fmaxf(M[r], wave_max(lv[r]));
      const float rescale = __expf(M[r] - Mb);          // first batch: exp(-inf) = 0 times zero sums
      M[r] = Mb;
      sum[r] *= rescale;
      acc[r].x *= rescale;
      acc[r].y *= rescale;
      w[r] = c < n ? __expf(lv[r] - Mb) : 0.f;
      sum[r] += w[r];                             // per lane; reduced once at the end
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        const float wj = u < cnt ? __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w[r]), u)) : 0.f;
        acc[r].x = fmaf(wj, o[u][r].x, acc[r].x);
        acc[r].y = fmaf(wj, o[u][r].y, acc[r].y);
      }
    }
    int j = U;
    // A pair cut into many chunks (a 131072-token context in 1024-token chunks: 128) is one wavefront's
    // serial walk; sixteen rows in flight instead of four turn its 32 round trips into 8.  Same order of sums.
    constexpr int D = 16 / RW;
    for (; j + D <= cnt; j += D) {
      float2 od[D][RW];
#pragma unroll
      for (int u = 0; u < D; ++u)
#pragma unroll
        for (int r = 0; r < RW; ++r) od[u][r] = load_f32x2<COHERENT>(rows + (j + u) * stride + r * 64);
#pragma unroll
      for (int u = 0; u < D; ++u) {
#pragma unroll
        for (int r = 0; r < RW; ++r) {
          const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w[r]), j + u));
          acc[r].x = fmaf(wj, od[u][r].x, acc[r].x);
          acc[r].y = fmaf(wj, od[u][r].y, acc[r].y);
        }
      }
    }
    for (; j + U <= cnt; j += U) {
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int r = 0; r < RW; ++r) o[u][r] = load_f32x2<COHERENT>(rows + (j + u) * stride + r * 64);
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int r = 0; r < RW; ++r) {
          const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w[r]), j + u));
          acc[r].x = fmaf(wj, o[u][r].x, acc[r].x);
          acc[r].y = fmaf(wj, o[u][r].y, acc[r].y);
        }
      }
    }
    for (; j < cnt; ++j) {
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        const float2 oj = load_f32x2<COHERENT>(rows + j * stride + r * 64);
        const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w[r]), j));
        acc[r].x = fmaf(wj, oj.x, acc[r].x);
        acc[r].y = fmaf(wj, oj.y, acc[r].y);
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const float total = wave_sum(sum[r]);
    const float inv = 1.0f / total;
    reinterpret_cast<float2*>(out_rows + r * fs::kHeadDim)[lane] = make_float2(acc[r].x * inv, acc[r].y * inv);
    if (lane == 0) lse_rows[r] = M[r] + __logf(total);
  }
}

}  // namespace fs_merge
