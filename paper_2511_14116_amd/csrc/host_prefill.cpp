// Host-side builder of one rank's chunked-prefill tile list (integer only).
//
// The paper's fine-grained chunked prefill (Section 3.1) batches chunks of several requests:
// n_new[r] new tokens behind n_done[r] processed ones.  Under hybrid attention a rank holds an
// irregular set of (request, KV head) pairs; every such pair whose request has new tokens
// contributes its chunk, cut into tiles of query tokens and, along the keys a tile sees, into
// split-K chunks: one kernel workgroup per (tile, chunk).  Split-K is this build's (the paper
// describes no kernel); it keeps one long context from serialising on one workgroup.
#include <algorithm>
#include <numeric>
#include <vector>

#include "fs_internal.h"

extern "C" fs_status fs_build_prefill_worklist(const fs_shape* shape, const int32_t* n_done, const int32_t* n_new,
                                               const int32_t* owner, int32_t rank, int32_t tile_tokens,
                                               int32_t kv_chunk_tokens,
                                               fs_prefill_item* items, int64_t items_cap,
                                               fs_prefill_pair* pairs, int64_t pairs_cap,
                                               int32_t* sched, int64_t* chunk_indptr, int64_t tiles_cap,
                                               int64_t* out_indptr,
                                               int64_t* n_items, int64_t* n_pairs, int64_t* n_tiles) {
  if (!shape) return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: shape is NULL");
  const int32_t B = shape->n_req, H = shape->n_kv_heads, R = shape->n_ranks;
  if (B < 0 || H < 1 || R < 1)
    return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: bad shape (n_req %d, n_kv_heads %d, n_ranks %d)", B, H, R);
  if (shape->n_q_heads < H || shape->n_q_heads % H)
    return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: n_q_heads %d is not a multiple of n_kv_heads %d",
                    shape->n_q_heads, H);
  if (!n_items || !n_pairs || !n_tiles) return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: count outputs are NULL");
  if (rank < 0 || rank >= R) return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: rank %d outside [0, %d)", rank, R);
  if (tile_tokens < 1) return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: tile_tokens %d < 1", tile_tokens);
  if (kv_chunk_tokens < 0 || kv_chunk_tokens % 32)
    return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: kv_chunk_tokens %d is not 0 or a multiple of 32", kv_chunk_tokens);
  if (B > 0 && (!n_done || !n_new || !owner)) return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: NULL input array");
  const bool count_only = !items && !pairs && !sched && !chunk_indptr && !out_indptr;
  if (items_cap < 0 || pairs_cap < 0 || tiles_cap < 0 || (!items && items_cap) || (!pairs && pairs_cap) ||
      (!sched && items_cap))
    return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: capacities do not match the arrays");
  const int64_t G = shape->n_q_heads / H, Hq = shape->n_q_heads, T = tile_tokens * G, C = kv_chunk_tokens;

  // Pass 1: validate and count.
  int64_t ni = 0, np = 0, nt = 0, q_tokens = 0;
  for (int32_t r = 0; r < B; ++r) {
    if (n_done[r] < 0 || n_new[r] < 0)
      return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: request %d has n_done %d, n_new %d", r, n_done[r], n_new[r]);
    if (static_cast<int64_t>(n_done[r]) + n_new[r] > 0x7FFFFFFF)
      return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: request %d is longer than int32 tokens", r);
    q_tokens += n_new[r];
    int64_t mine = 0;
    for (int32_t h = 0; h < H; ++h) {
      const int32_t o = owner[static_cast<int64_t>(r) * H + h];
      if (o < 0 || o >= R)
        return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: owner of (%d, %d) is %d, outside [0, %d)", r, h, o, R);
      mine += o == rank;
    }
    if (mine == 0 || n_new[r] == 0) continue;
    int64_t tiles = 0, chunks = 0;
    for (int64_t b = 0; b < n_new[r]; b += tile_tokens) {
      const int64_t keys = n_done[r] + std::min<int64_t>(n_new[r], b + tile_tokens);
      ++tiles;
      chunks += C ? (keys + C - 1) / C : 1;
    }
    np += mine;
    nt += mine * tiles;
    ni += mine * chunks;
  }
  if (q_tokens * Hq > 0x7FFFFFFF || ni * T > 0x7FFFFFFF || ni > 0x7FFFFFFF)
    return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: the batch has more rows than int32 holds");
  *n_items = ni;
  *n_pairs = np;
  *n_tiles = nt;
  if (count_only) return FS_OK;
  if (!chunk_indptr || !out_indptr) return fs::fail(FS_EINVAL, "fs_build_prefill_worklist: chunk_indptr or out_indptr is NULL");
  if (ni > items_cap || np > pairs_cap || nt > tiles_cap)
    return fs::fail(FS_ECAPACITY, "fs_build_prefill_worklist: needs %lld items, %lld pairs, %lld tiles; arrays hold %lld, %lld, %lld",
                    static_cast<long long>(ni), static_cast<long long>(np), static_cast<long long>(nt),
                    static_cast<long long>(items_cap), static_cast<long long>(pairs_cap), static_cast<long long>(tiles_cap));

  // Pass 2: fill.
  int64_t i = 0, p = 0, t = 0, q0 = 0;
  chunk_indptr[0] = 0;
  out_indptr[0] = 0;
  for (int32_t r = 0; r < B; ++r) {
    const int32_t N = n_new[r], L = n_done[r];
    if (N > 0) {
      for (int32_t h = 0; h < H; ++h) {
        if (owner[static_cast<int64_t>(r) * H + h] != rank) continue;
        pairs[p] = fs_prefill_pair{r, h, L, N};
        for (int32_t b = 0; b < N; b += tile_tokens) {
          const int32_t e = N - b < tile_tokens ? N : b + tile_tokens;
          const int64_t keys = static_cast<int64_t>(L) + e;
          const int64_t step = C ? C : keys;
          for (int64_t k0 = 0; k0 < keys; k0 += step) {
            items[i] = fs_prefill_item{static_cast<int32_t>(p), b, e, L, static_cast<int32_t>(k0),
                                       static_cast<int32_t>(std::min(keys, k0 + step)),
                                       static_cast<int32_t>((q0 + b) * Hq + h * G), static_cast<int32_t>(i * T)};
            ++i;
          }
          chunk_indptr[++t] = i;
        }
        out_indptr[++p] = t * T;
      }
    }
    q0 += N;
  }
  // Longest first: an item streams the keys of its chunk.
  std::iota(sched, sched + ni, 0);
  std::stable_sort(sched, sched + ni, [&](int32_t a, int32_t b) {
    return items[a].kv_end - items[a].kv_begin > items[b].kv_end - items[b].kv_begin;
  });
  return FS_OK;
}

extern "C" fs_status fs_choose_prefill_chunk(const fs_shape* shape, const int32_t* n_done, const int32_t* n_new,
                                             const int32_t* owner, int32_t rank, int32_t tile_tokens,
                                             int32_t max_chunk, int32_t min_chunk, int64_t n_slots,
                                             int32_t* kv_chunk_tokens, int64_t* n_items) {
  if (!kv_chunk_tokens || !n_items) return fs::fail(FS_EINVAL, "fs_choose_prefill_chunk: output pointers are NULL");
  if (min_chunk < 32 || min_chunk % 32 || max_chunk < min_chunk || max_chunk % 32)
    return fs::fail(FS_EINVAL, "fs_choose_prefill_chunk: chunks [%d, %d] must be multiples of 32, min <= max", min_chunk,
                    max_chunk);
  if (n_slots < 1) return fs::fail(FS_EINVAL, "fs_choose_prefill_chunk: n_slots %lld < 1", static_cast<long long>(n_slots));
  // The list builder checks the arguments (and counts the uncut list, which is not needed here).
  int64_t ni = 0, np = 0, nt = 0;
  if (const fs_status st = fs_build_prefill_worklist(shape, n_done, n_new, owner, rank, tile_tokens, 0, nullptr, 0, nullptr,
                                                     0, nullptr, nullptr, 0, nullptr, &ni, &np, &nt); st != FS_OK)
    return st;
  // Keys the rank's tiles see, all told: the tiles of a request see n_done + tile, n_done + 2 tile, ..., n_done + n_new.
  const int32_t B = shape->n_req, H = shape->n_kv_heads;
  int64_t total = 0;
  for (int32_t r = 0; r < B; ++r) {
    if (n_new[r] == 0) continue;
    int64_t mine = 0;
    for (int32_t h = 0; h < H; ++h) mine += owner[static_cast<int64_t>(r) * H + h] == rank;
    if (mine == 0) continue;
    const int64_t full = n_new[r] / tile_tokens, rest = n_new[r] % tile_tokens;      // full tiles, tokens of a last short one
    int64_t keys = full * n_done[r] + static_cast<int64_t>(tile_tokens) * full * (full + 1) / 2;
    if (rest) keys += static_cast<int64_t>(n_done[r]) + n_new[r];
    total += mine * keys;
  }
  // four thirds of a slot's fair share, up to a multiple of 32 keys, within the bounds
  const int64_t target = (4 * total + 3 * n_slots - 1) / (3 * n_slots);
  int64_t chunk = (target + 31) / 32 * 32;
  chunk = std::min<int64_t>(std::max<int64_t>(chunk, min_chunk), max_chunk);
  // the list's length with it: an item per chunk of the keys a tile sees
  int64_t count = 0;
  for (int32_t r = 0; r < B; ++r) {
    if (n_new[r] == 0) continue;
    int64_t mine = 0;
    for (int32_t h = 0; h < H; ++h) mine += owner[static_cast<int64_t>(r) * H + h] == rank;
    if (mine == 0) continue;
    int64_t chunks = 0;
    for (int64_t b = 0; b < n_new[r]; b += tile_tokens) {
      const uint32_t keys = static_cast<uint32_t>(n_done[r] + std::min<int64_t>(n_new[r], b + tile_tokens));   // < 2^31: checked by the builder
      chunks += (keys + static_cast<uint32_t>(chunk) - 1) / static_cast<uint32_t>(chunk);
    }
    count += mine * chunks;
  }
  *kv_chunk_tokens = static_cast<int32_t>(chunk);
  *n_items = count;
  return FS_OK;
}
