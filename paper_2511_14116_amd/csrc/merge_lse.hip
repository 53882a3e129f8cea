// fs_merge_lse: combine the split-K chunk partials of each (request, KV head) pair.
//
// Split-K is not in the paper; it is how one GPU keeps long contexts (Section 3.1 notes that
// skewed long-context batches produce stragglers) from serialising on one workgroup.  The merge
// is exact algebra on the partial (out, lse) pairs:
//     lse = ln sum_c exp(lse_c),   out = sum_c exp(lse_c - lse) * o_c.
//
// One wavefront per output row (pair, q-head); a lane owns two of the 128 columns, so a row of
// a partial is one coalesced 512-byte read.  HBM traffic is under 1% of the attention sweep's.
#include <hip/hip_runtime.h>

#include "fs_internal.h"

namespace {

constexpr int kRowsPerBlock = 4;

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
  const int64_t c0 = chunk_indptr[p], c1 = chunk_indptr[p + 1];

  float M = -INFINITY;
  for (int64_t c = c0; c < c1; ++c) M = fmaxf(M, part_lse[c * group + g]);
  float sum = 0.f;
  float2 acc = make_float2(0.f, 0.f);
  for (int64_t c = c0; c < c1; ++c) {
    const int64_t r = c * group + g;
    const float w = __expf(part_lse[r] - M);
    const float2 o = reinterpret_cast<const float2*>(part_o + r * fs::kHeadDim)[lane];
    sum += w;
    acc.x = fmaf(w, o.x, acc.x);
    acc.y = fmaf(w, o.y, acc.y);
  }
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
