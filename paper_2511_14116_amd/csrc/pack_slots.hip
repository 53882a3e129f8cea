// fs_pack_kv_slots: KVCache slots from token-major order into the in-slot element order the
// attention kernels read (fs_kv_elem_offset is the definition), on the device.
//
// The paper says nothing about the order of the elements inside a KVCache block; the kernels here
// want K and V in the order of the matrix cores' operands.  An engine's KV-append step would write
// that order directly; this call is the stand-in for it when a cache already exists token-major
// (and what the harness uses to lay out its synthetic pools).  One workgroup per slot: the slot
// goes through LDS with 16-byte reads, every thread assembles one 16-byte piece of the new order
// and the slot leaves as one contiguous 4 KiB run.
#include <hip/hip_runtime.h>

#include "fs_internal.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kSlotElems = fs::kPageTokens * fs::kHeadDim;   // 2048

// Inverse of fs_kv_elem_offset for bf16: which (token, d) sits at element offset i of a packed slot.
__device__ __forceinline__ int source_index(int i, bool is_v) {
  const int c = i >> 9, r = i & 511;
  if (!is_v) {           // K: [d/32][(d%32)/8][tok][d%8]
    const int g = r >> 7, tok = (r & 127) >> 3, e = r & 7;
    return tok * fs::kHeadDim + 32 * c + 8 * g + e;
  }
  // V: [d/32][tok/4][d%16][(d/16)%2][tok%4]
  const int t4 = r >> 7, dl = (r & 127) >> 3, hi = (r & 7) >> 2, tl = r & 3;
  return (4 * t4 + tl) * fs::kHeadDim + 32 * c + dl + 16 * hi;
}

__global__ void __launch_bounds__(256)
pack_bf16_slots_kernel(const char* __restrict__ src, int64_t src_stride, char* __restrict__ dst, int64_t dst_stride,
                       int is_v) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[kSlotElems];
  const int64_t slot = blockIdx.x;
  reinterpret_cast<u32x4*>(tile)[threadIdx.x] = reinterpret_cast<const u32x4*>(src + slot * src_stride)[threadIdx.x];
  __syncthreads();
  uint16_t piece[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) piece[e] = tile[source_index(8 * threadIdx.x + e, is_v != 0)];
  u32x4 v;
  v.x = piece[0] | (static_cast<uint32_t>(piece[1]) << 16);
  v.y = piece[2] | (static_cast<uint32_t>(piece[3]) << 16);
  v.z = piece[4] | (static_cast<uint32_t>(piece[5]) << 16);
  v.w = piece[6] | (static_cast<uint32_t>(piece[7]) << 16);
  reinterpret_cast<u32x4*>(dst + slot * dst_stride)[threadIdx.x] = v;
}

// fp8, K and V alike, [d/64][(d%64)/16][tok][d%16]: 16-byte piece i of the new order is piece (tok, d/16) of the
// token-major one (2 KiB per slot, 128 threads x 16 bytes).
__global__ void __launch_bounds__(128)
pack_fp8_slots_kernel(const char* __restrict__ src, int64_t src_stride, char* __restrict__ dst, int64_t dst_stride) {
  const int64_t slot = blockIdx.x;
  const int i = threadIdx.x;
  const int from = (i & 15) * 8 + (i >> 6) * 4 + ((i & 63) >> 4);
  reinterpret_cast<u32x4*>(dst + slot * dst_stride)[i] = reinterpret_cast<const u32x4*>(src + slot * src_stride)[from];
}

}  // namespace

extern "C" fs_status fs_pack_kv_slots(const void* src_dev, int64_t src_slot_stride, void* dst_dev, int64_t dst_slot_stride,
                                      int64_t n_slots, int32_t kv_dtype, int32_t is_v, void* stream) {
  if (kv_dtype != FS_KV_BF16 && kv_dtype != FS_KV_FP8_E4M3)
    return fs::fail(FS_EINVAL, "fs_pack_kv_slots: unknown kv_dtype %d", kv_dtype);
  if (n_slots < 0 || n_slots > 0x7FFFFFFF) return fs::fail(FS_EINVAL, "fs_pack_kv_slots: n_slots out of range");
  if (n_slots == 0) return FS_OK;
  const int64_t slot_bytes = static_cast<int64_t>(kSlotElems) * (kv_dtype == FS_KV_BF16 ? 2 : 1);
  if (!src_dev || !dst_dev) return fs::fail(FS_EINVAL, "fs_pack_kv_slots: NULL device pointer");
  if (src_slot_stride < slot_bytes || dst_slot_stride < slot_bytes || (src_slot_stride & 15) || (dst_slot_stride & 15) ||
      (reinterpret_cast<uintptr_t>(src_dev) & 15) || (reinterpret_cast<uintptr_t>(dst_dev) & 15))
    return fs::fail(FS_EINVAL, "fs_pack_kv_slots: pools and strides must be 16-byte aligned and strides at least one slot "
                               "(%lld bytes)", static_cast<long long>(slot_bytes));
  // The two pools must not overlap (the order changes within a slot; nothing is done in place).
  const char* s0 = static_cast<const char*>(src_dev);
  const char* d0 = static_cast<const char*>(dst_dev);
  const char* s1 = s0 + (n_slots - 1) * src_slot_stride + slot_bytes;
  const char* d1 = d0 + (n_slots - 1) * dst_slot_stride + slot_bytes;
  if (s0 < d1 && d0 < s1)
    return fs::fail(FS_EINVAL, "fs_pack_kv_slots: source and destination slots overlap");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (kv_dtype == FS_KV_BF16)
    hipLaunchKernelGGL(pack_bf16_slots_kernel, dim3(static_cast<unsigned>(n_slots)), dim3(256), 0, s, s0,
                       src_slot_stride, static_cast<char*>(dst_dev), dst_slot_stride, is_v ? 1 : 0);
  else
    hipLaunchKernelGGL(pack_fp8_slots_kernel, dim3(static_cast<unsigned>(n_slots)), dim3(128), 0, s, s0, src_slot_stride,
                       static_cast<char*>(dst_dev), dst_slot_stride);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fs::fail(FS_EHIP, "fs_pack_kv_slots: launch failed: %s", hipGetErrorString(e));
  return FS_OK;
}
