// fs_merge_lse: combine the split-K chunk partials of each (request, KV head) pair.
//
// Split-K is not in the paper; it is how one GPU keeps long contexts (Section 3.1 notes that
// skewed long-context batches produce stragglers) from serialising on one workgroup.  The merge
// is exact algebra on the partial (out, lse) pairs:
//     lse = ln sum_c exp(lse_c),   out = sum_c exp(lse_c - lse) * o_c.
//
// One wavefront per output row (pair, q-head), or per four consecutive rows of a pair when the group
// is a multiple of four.  A row's chunk lse values are read 64 at a time, one per lane, and reduced
// across the wavefront, so a pair cut into many chunks (a 131072-token context in 1024-token chunks
// has 128) costs a wide load per 64 chunks instead of a serial chain.  For the rows themselves a lane
// owns two of the 128 columns (one coalesced 512-byte read per chunk row); the first four chunk rows
// (two per output row in the four-row form) are requested together with the lse values, before the
// weights are known, and the rest follow sixteen at a time.  For decode the traffic is under 1% of
// the attention sweep's; for chunked prefill (a tile's rows per chunk) it is a sixth of the kernel time.
#include <hip/hip_runtime.h>

#include "fs_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// RW output rows per wavefront (consecutive rows of one pair, so group must be a multiple of RW): with many
// rows of few chunks each (a prefill tile's 128 rows, most tiles a single chunk) a wavefront with one row is
// a chain of three dependent loads and nothing else; four rows side by side keep four times the bytes in flight.
// The arithmetic of a row is the same for every RW, operation for operation.
template <int RW>
__global__ void __launch_bounds__(kWavesPerBlock * 64)
merge_lse_kernel(const float* __restrict__ part_o, const float* __restrict__ part_lse,
                 const int64_t* __restrict__ chunk_indptr, int64_t n_rows, int group,
                 float* __restrict__ out, float* __restrict__ lse, int skip_single) {
  constexpr int U = RW == 1 ? 4 : 2;               // chunk rows in flight per output row
  const int lane = threadIdx.x & 63;
  const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * kWavesPerBlock +
                        __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * RW;
  if (row0 >= n_rows) return;
  const int64_t p = row0 / group;
  const int g0 = static_cast<int>(row0 - p * group);
  const int64_t c0 = chunk_indptr[p];
  const int n = static_cast<int>(chunk_indptr[p + 1] - c0);
  if (skip_single && n == 1) return;   // fused decode: the sweep has already written this pair's final rows

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
    for (int r = 0; r < RW; ++r) lv[r] = c < n ? part_lse[(c0 + c) * group + g0 + r] : -INFINITY;
    // row r of chunk base+j: rows[j * stride + r * 64]
    const float2* rows = reinterpret_cast<const float2*>(part_o + ((c0 + base) * group + g0) * fs::kHeadDim) + lane;
    float2 o[U][RW];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < RW; ++r) o[u][r] = rows[min(u, cnt - 1) * stride + r * 64];   // the batch's first rows (repeats if it has fewer)
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
        for (int r = 0; r < RW; ++r) od[u][r] = rows[(j + u) * stride + r * 64];
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
        for (int r = 0; r < RW; ++r) o[u][r] = rows[(j + u) * stride + r * 64];
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
        const float2 oj = rows[j * stride + r * 64];
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
    reinterpret_cast<float2*>(out + (row0 + r) * fs::kHeadDim)[lane] = make_float2(acc[r].x * inv, acc[r].y * inv);
    if (lane == 0) lse[row0 + r] = M[r] + __logf(total);
  }
}

}  // namespace

namespace fs {

fs_status merge_lse_launch(const char* who, const float* part_o, const float* part_lse, const int64_t* chunk_indptr_dev,
                           int64_t n_pairs, int32_t group, float* out, float* lse, bool skip_single, void* stream_ptr) {
  hipStream_t stream = static_cast<hipStream_t>(stream_ptr);
  const int64_t n_rows = n_pairs * group;
  // Output rows per wavefront (within one pair): four once one row each would be more wavefronts than the
  // chip holds at a time (256 CUs x 32); below that, more wavefronts is what hides the latency.
  const int rw = group % 4 == 0 && n_rows > 8192 ? 4 : 1;
  const int64_t per_block = static_cast<int64_t>(kWavesPerBlock) * rw;
  const unsigned blocks = static_cast<unsigned>((n_rows + per_block - 1) / per_block);
  if (rw == 4)
    hipLaunchKernelGGL(merge_lse_kernel<4>, dim3(blocks), dim3(kWavesPerBlock * 64), 0, stream, part_o, part_lse,
                       chunk_indptr_dev, n_rows, group, out, lse, skip_single ? 1 : 0);
  else
    hipLaunchKernelGGL(merge_lse_kernel<1>, dim3(blocks), dim3(kWavesPerBlock * 64), 0, stream, part_o, part_lse,
                       chunk_indptr_dev, n_rows, group, out, lse, skip_single ? 1 : 0);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fs::fail(FS_EHIP, "%s: launch of the merge failed: %s", who, hipGetErrorString(e));
  return FS_OK;
}

}  // namespace fs

extern "C" fs_status fs_merge_lse(const float* part_o, const float* part_lse, const int64_t* chunk_indptr_dev,
                                  int64_t n_pairs, int32_t group, int32_t head_dim,
                                  float* out, float* lse, void* stream) {
  if (group < 1) return fs::fail(FS_EINVAL, "fs_merge_lse: group %d < 1", group);
  if (head_dim != fs::kHeadDim)
    return fs::fail(FS_EUNSUPPORTED, "fs_merge_lse: head_dim %d (only %d is built)", head_dim, fs::kHeadDim);
  if (n_pairs < 0 || n_pairs * group > 0x7FFFFFFFll)
    return fs::fail(FS_EINVAL, "fs_merge_lse: n_pairs out of range");
  if (n_pairs == 0) return FS_OK;
  if (!part_o || !part_lse || !chunk_indptr_dev || !out || !lse)
    return fs::fail(FS_EINVAL, "fs_merge_lse: NULL device pointer");
  return fs::merge_lse_launch("fs_merge_lse", part_o, part_lse, chunk_indptr_dev, n_pairs, group, out, lse, false, stream);
}
