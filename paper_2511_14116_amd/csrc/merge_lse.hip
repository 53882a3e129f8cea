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
#include "merge_row.h"

namespace {

constexpr int kWavesPerBlock = 4;

// RW output rows per wavefront (consecutive rows of one pair, so group must be a multiple of RW): with many
// rows of few chunks each (a prefill tile's 128 rows, most tiles a single chunk) a wavefront with one row is
// a chain of three dependent loads and nothing else; four rows side by side keep four times the bytes in flight.
// The arithmetic of a row is the same for every RW, operation for operation.
template <int RW>
__global__ void __launch_bounds__(kWavesPerBlock * 64)
merge_lse_kernel(const float* __restrict__ part_o, const float* __restrict__ part_lse,
                 const int64_t* __restrict__ chunk_indptr, int64_t n_rows, int group,
                 float* __restrict__ out, float* __restrict__ lse, int skip_single) {
  const int lane = threadIdx.x & 63;
  const int64_t row0 = (static_cast<int64_t>(blockIdx.x) * kWavesPerBlock +
                        __builtin_amdgcn_readfirstlane(threadIdx.x >> 6)) * RW;
  if (row0 >= n_rows) return;
  const int64_t p = row0 / group;
  const int g0 = static_cast<int>(row0 - p * group);
  const int64_t c0 = chunk_indptr[p];
  const int n = static_cast<int>(chunk_indptr[p + 1] - c0);
  if (skip_single && n == 1) return;   // fused decode: the sweep has already written this pair's final rows
  fs_merge::merge_rows<RW>(part_o, part_lse, c0, n, group, g0, out + row0 * fs::kHeadDim, lse + row0, lane);
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
