// fs_merge_lse: combine the split-K chunk partials of each (request, KV head) pair.
//
// Split-K is not in the paper; it is how one GPU keeps long contexts (Section 3.1 notes that
// skewed long-context batches produce stragglers) from serialising on one workgroup.  The merge
// is exact algebra on the partial (out, lse) pairs:
//     lse = ln sum_c exp(lse_c),   out = sum_c exp(lse_c - lse) * o_c.
//
// One wavefront per output row (pair, q-head).  The row's chunk lse values are read 64 at a time,
// one per lane, and reduced across the wavefront, so a pair cut into many chunks (a 131072-token
// context in 1024-token chunks has 128) costs a wide load per 64 chunks instead of a serial chain.
// For the rows themselves a lane owns two of the 128 columns (one coalesced 512-byte read per
// chunk), four chunk rows are in flight at a time, and the first four are requested together with
// the lse values, before the weights are known.  For decode the traffic is under 1% of the
// attention sweep's; for chunked prefill (a tile's rows per chunk) it is a sixth of the kernel time.
#include <hip/hip_runtime.h>

#include "fs_internal.h"

namespace {

constexpr int kRowsPerBlock = 4;

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

__global__ void __launch_bounds__(kRowsPerBlock * 64)
merge_lse_kernel(const float* __restrict__ part_o, const float* __restrict__ part_lse,
                 const int64_t* __restrict__ chunk_indptr, int64_t n_rows, int group,
                 float* __restrict__ out, float* __restrict__ lse) {
  const int lane = threadIdx.x & 63;
  const int64_t row = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock +
                      __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (row >= n_rows) return;
  const int64_t p = row / group;
  const int g = static_cast<int>(row - p * group);
  const int64_t c0 = chunk_indptr[p];
  const int n = static_cast<int>(chunk_indptr[p + 1] - c0);

  // Chunks are taken 64 at a time (one lse per lane).  The first rows of a batch are requested before
  // its weights are known, so the two reads travel together; across batches (more than 64 chunks) the
  // running maximum moves and what has been summed is rescaled, as in an online softmax.
  float M = -INFINITY;
  float sum = 0.f;
  float2 acc = make_float2(0.f, 0.f);
  const int64_t stride = static_cast<int64_t>(group) * (fs::kHeadDim / 2);   // float2 units between chunk rows
  for (int base = 0; base < n; base += 64) {
    const int c = base + lane;
    const int cnt = min(64, n - base);
    const float lv = c < n ? part_lse[(c0 + c) * group + g] : -INFINITY;
    const float2* rows = reinterpret_cast<const float2*>(part_o + ((c0 + base) * group + g) * fs::kHeadDim) + lane;
    float2 o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) o[u] = rows[min(u, cnt - 1) * stride];        // the batch's first rows (repeats if it has fewer)
    const float Mb = fmaxf(M, wave_max(lv));
    const float rescale = __expf(M - Mb);              // first batch: exp(-inf) = 0 times zero sums
    M = Mb;
    sum *= rescale;
    acc.x *= rescale;
    acc.y *= rescale;
    const float w = c < n ? __expf(lv - M) : 0.f;
    sum += w;                                   // per lane; reduced once at the end
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wj = u < cnt ? __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), u)) : 0.f;
      acc.x = fmaf(wj, o[u].x, acc.x);
      acc.y = fmaf(wj, o[u].y, acc.y);
    }
    int j = 4;
    for (; j + 4 <= cnt; j += 4) {
#pragma unroll
      for (int u = 0; u < 4; ++u) o[u] = rows[(j + u) * stride];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), j + u));
        acc.x = fmaf(wj, o[u].x, acc.x);
        acc.y = fmaf(wj, o[u].y, acc.y);
      }
    }
    for (; j < cnt; ++j) {
      const float2 oj = rows[j * stride];
      const float wj = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), j));
      acc.x = fmaf(wj, oj.x, acc.x);
      acc.y = fmaf(wj, oj.y, acc.y);
    }
  }
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
  reinterpret_cast<float2*>(out + row * fs::kHeadDim)[lane] = make_float2(acc.x * inv, acc.y * inv);
  if (lane == 0) lse[row] = M + __logf(sum);
}

}  // namespace

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
  const int64_t n_rows = n_pairs * group;
  const unsigned blocks = static_cast<unsigned>((n_rows + kRowsPerBlock - 1) / kRowsPerBlock);
  hipLaunchKernelGGL(merge_lse_kernel, dim3(blocks), dim3(kRowsPerBlock * 64), 0,
                     static_cast<hipStream_t>(stream), part_o, part_lse, chunk_indptr_dev, n_rows, group, out, lse);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fs::fail(FS_EHIP, "fs_merge_lse: launch failed: %s", hipGetErrorString(e));
  return FS_OK;
}
