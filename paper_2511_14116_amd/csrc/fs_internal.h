// Internal helpers shared by the library's translation units (not part of the ABI).
#pragma once
#include <cstdarg>
#include <cstdint>

#include "failsafe.h"

namespace fs {

// Record a message for fs_last_error() and hand the status back.
fs_status fail(fs_status st, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

constexpr int kHeadDim = 128;
constexpr int kPageTokens = 16;
constexpr int kMaxGroup = 16;       // q-heads per KV head that fit one MFMA tile column set
constexpr int kPersistentMinItems = 1024;   // list length from which the fused decode call takes the persistent sweep

struct Options {
  int waves_per_group;   // wavefronts cooperating on one work item (1, 2 or 4)
  int prefetch_pages;    // KV pages a wavefront keeps in flight ahead of the one it is consuming (1..3)
  int prefill_col_tiles; // 16-row column tiles of query rows per prefill wavefront (1, 2 or 4)
  int prefill_waves;     // wavefronts per prefill workgroup (4 or 8)
};
Options& options();

// The split-K merge as the fused decode call launches it (arguments already checked).  skip_single: pairs
// of one chunk are left alone (their final rows are already written).
fs_status merge_lse_launch(const char* who, const float* part_o, const float* part_lse, const int64_t* chunk_indptr_dev,
                           int64_t n_pairs, int32_t group, float* out, float* lse, bool skip_single, void* stream);

}  // namespace fs
