// Host-side router and prefill batch former (integer only, never touches the GPU).
//
// Section 3.1 of the paper, "Fine-grained Load-aware Router": an incoming request goes to
// the rank with the least pending DP work (Load-Aware DP-Rank Routing), and Algorithm 1
// (DP-aware Adaptive Chunked Prefill) fills a token budget one token at a time from the
// least-loaded rank that still has schedulable tokens, then picks the best of the batches
// it passed through.  What the paper leaves open (the token cost, the choice among the
// candidates, the unused workload input) is fixed as the header states.
#include <algorithm>
#include <cstddef>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "fs_internal.h"

extern "C" fs_status fs_route_request(int32_t n_ranks, int64_t* pending, int64_t work, int32_t* rank) {
  if (n_ranks < 1) return fs::fail(FS_EINVAL, "fs_route_request: n_ranks %d < 1", n_ranks);
  if (!pending || !rank) return fs::fail(FS_EINVAL, "fs_route_request: NULL pointer");
  if (work < 0) return fs::fail(FS_EINVAL, "fs_route_request: work %lld < 0", static_cast<long long>(work));
  int32_t best = 0;
  for (int32_t k = 1; k < n_ranks; ++k)
    if (pending[k] < pending[best]) best = k;   // strict: equal loads keep the lowest rank
  pending[best] += work;
  *rank = best;
  return FS_OK;
}

extern "C" fs_status fs_route_requests(int32_t n_ranks, int64_t* pending, const int64_t* work, int32_t n, int32_t* rank) {
  if (n_ranks < 1) return fs::fail(FS_EINVAL, "fs_route_requests: n_ranks %d < 1", n_ranks);
  if (n < 0) return fs::fail(FS_EINVAL, "fs_route_requests: n %d < 0", n);
  if (!pending || (n > 0 && (!work || !rank))) return fs::fail(FS_EINVAL, "fs_route_requests: NULL pointer");
  for (int32_t i = 0; i < n; ++i)
    if (work[i] < 0)
      return fs::fail(FS_EINVAL, "fs_route_requests: work[%d] = %lld < 0", i, static_cast<long long>(work[i]));
  for (int32_t i = 0; i < n; ++i) {
    int32_t best = 0;
    for (int32_t k = 1; k < n_ranks; ++k)
      if (pending[k] < pending[best]) best = k;   // strict: equal loads keep the lowest rank
    pending[best] += work[i];
    rank[i] = best;
  }
  return FS_OK;
}

namespace {
fs_status schedule_prefill(int32_t n_ranks, int32_t budget, int32_t min_tokens, const fs_prefill_entry* entries,
                           int32_t n_entries, const int64_t* init_load, int32_t* take, int64_t* load,
                           int32_t* n_tokens) {
  const int32_t R = n_ranks;
  if (R < 1) return fs::fail(FS_EINVAL, "fs_schedule_prefill: n_ranks %d < 1", R);
  if (budget < 0 || min_tokens < 0 || n_entries < 0)
    return fs::fail(FS_EINVAL, "fs_schedule_prefill: budget %d, min_tokens %d, n_entries %d must be >= 0", budget,
                    min_tokens, n_entries);
  if (!load || !n_tokens || (n_entries > 0 && (!entries || !take)))
    return fs::fail(FS_EINVAL, "fs_schedule_prefill: NULL pointer");
  for (int32_t e = 0; e < n_entries; ++e) {
    const fs_prefill_entry& q = entries[e];
    if (q.rank < 0 || q.rank >= R || q.n_done < 0 || q.n_new < 0)
      return fs::fail(FS_EINVAL, "fs_schedule_prefill: entry %d (rank %d, n_done %d, n_new %d) is out of range", e,
                      q.rank, q.n_done, q.n_new);
  }

  if (init_load)
    for (int32_t r = 0; r < R; ++r)
      if (init_load[r] < 0)
        return fs::fail(FS_EINVAL, "fs_schedule_prefill: init_load[%d] = %lld < 0 (a load is work in token units)", r,
                        static_cast<long long>(init_load[r]));

  // S_r: per rank, the entries routed to it in arrival order, and a cursor (entry, tokens taken).
  std::vector<int32_t> first(R, -1), next(n_entries > 0 ? n_entries : 1, -1), last(R, -1);
  for (int32_t e = 0; e < n_entries; ++e) {
    if (entries[e].n_new == 0) continue;
    const int32_t r = entries[e].rank;
    if (first[r] < 0) first[r] = e; else next[last[r]] = e;
    last[r] = e;
  }
  for (int32_t e = 0; e < n_entries; ++e) take[e] = 0;
  std::vector<int32_t> cur = first;          // entry at the head of S_r, -1 when S_r is empty
  std::vector<int32_t> cur_taken(R, 0);      // tokens already taken from that entry
  std::vector<int64_t> L(R);
  for (int32_t r = 0; r < R; ++r) L[r] = init_load ? init_load[r] : 0;

  // The loop of Algorithm 1.
  // Candidate i (the batch after i+1 tokens) is remembered as the rank it took from; from the first batch
  // choose_best_batch may pick on (min(min_tokens, all) tokens), also the largest load and the load sum.
  int64_t waiting = 0;
  for (int32_t e = 0; e < n_entries; ++e) waiting += entries[e].n_new;
  const size_t most = static_cast<size_t>(waiting < budget ? waiting : budget);   // tokens the loop can take
  if (most == 0) {
    for (int32_t r = 0; r < R; ++r) load[r] = L[r];
    *n_tokens = 0;
    return FS_OK;
  }
  const size_t lo = static_cast<size_t>(min_tokens) < most ? static_cast<size_t>(min_tokens) : most;
  const size_t first_cand = lo > 0 ? lo - 1 : 0;
  std::vector<uint8_t> took_from8;
  std::vector<int32_t> took_from32;
  const bool small_r = R <= 256;
  if (small_r) took_from8.resize(most); else took_from32.resize(most);
  std::vector<int64_t> cand_max(most - first_cand), cand_sum(most - first_cand);
  int64_t sum = 0, mx = 0;
  for (int32_t r = 0; r < R; ++r) { sum += L[r]; if (r == 0 || L[r] > mx) mx = L[r]; }
  // A rank whose S_r is empty is priced at the largest load so that the search below needs no test per
  // rank; the loop ends after `most` tokens, which is exactly when every S_r is empty or the budget is spent.
  constexpr int64_t kEmpty = std::numeric_limits<int64_t>::max();
  auto record = [&](size_t n_taken, int32_t rs) {
    if (small_r) took_from8[n_taken] = static_cast<uint8_t>(rs); else took_from32[n_taken] = rs;
    if (n_taken >= first_cand) {
      cand_max[n_taken - first_cand] = mx;
      cand_sum[n_taken - first_cand] = sum;
    }
  };
  // Up to 8 ranks (a node) with loads (never negative) that leave three bits to spare: load and rank travel as one key,
  // load*8 + rank, so the least key is the least load and, among equals, the lowest rank; the eight keys
  // stay in registers and the search is a tree of seven minima.  Same picks as the general loop below.
  constexpr int kPack = 8;
  bool packed = R <= kPack;
  if (packed) {
    int64_t top = 0, dearest = 0;
    for (int32_t r = 0; r < R; ++r) if (L[r] > top) top = L[r];
    for (int32_t e = 0; e < n_entries; ++e)
      dearest = std::max<int64_t>(dearest, static_cast<int64_t>(entries[e].n_done) + entries[e].n_new);
    // no load can pass top + most * dearest
    if (dearest > 0 && static_cast<int64_t>(most) > ((int64_t{1} << 59) - top) / dearest) packed = false;
  }
  if (packed) {
    int64_t k[kPack], cost[kPack], left[kPack];
    for (int32_t r = 0; r < kPack; ++r) {
      const bool has = r < R && cur[r] >= 0;
      k[r] = has ? L[r] * kPack + r : kEmpty;
      cost[r] = has ? static_cast<int64_t>(entries[cur[r]].n_done) + 1 : 0;   // keys the rank's next token attends to
      left[r] = has ? entries[cur[r]].n_new : 0;                             // tokens left in the entry at the head of S_r
    }
    for (size_t n_taken = 0; n_taken < most; ++n_taken) {
      const int64_t a = std::min(std::min(k[0], k[1]), std::min(k[2], k[3]));
      const int64_t b = std::min(std::min(k[4], k[5]), std::min(k[6], k[7]));
      const int64_t least = std::min(a, b);
      const int32_t rs = static_cast<int32_t>(least & (kPack - 1));
      const int64_t c = cost[rs];
      const int64_t grown = least / kPack + c;
      sum += c;
      if (grown > mx) mx = grown;
      cost[rs] = c + 1;
      bool has = true;
      if (--left[rs] == 0) {                      // the entry is used up: S_r goes on with the rank's next one
        const int32_t e = next[cur[rs]];
        cur[rs] = e;
        has = e >= 0;
        if (has) { cost[rs] = static_cast<int64_t>(entries[e].n_done) + 1; left[rs] = entries[e].n_new; }
      }
      const int64_t key_now = has ? grown * kPack + rs : kEmpty;
      for (int32_t r = 0; r < kPack; ++r) k[r] = r == rs ? key_now : k[r];
      record(n_taken, rs);
    }
  } else {
    std::vector<int64_t> key(R);
    for (int32_t r = 0; r < R; ++r) key[r] = cur[r] >= 0 ? L[r] : kEmpty;
    for (size_t n_taken = 0; n_taken < most; ++n_taken) {
      int32_t rs = 0;
      int64_t least = key[0];
      for (int32_t r = 1; r < R; ++r) {          // strict: equal loads keep the lowest rank
        const bool lt = key[r] < least;
        least = lt ? key[r] : least;
        rs = lt ? r : rs;
      }
      const fs_prefill_entry& q = entries[cur[rs]];
      const int64_t cost = static_cast<int64_t>(q.n_done) + cur_taken[rs] + 1;   // keys this token attends to
      L[rs] += cost;
      sum += cost;
      if (L[rs] > mx) mx = L[rs];
      if (++cur_taken[rs] == q.n_new) { cur[rs] = next[cur[rs]]; cur_taken[rs] = 0; }
      key[rs] = cur[rs] >= 0 ? L[rs] : kEmpty;
      record(n_taken, rs);
    }
  }

  // choose_best_batch: smallest max/mean among the eligible candidates, the larger batch among equals.
  // max_i/sum_i <= max_b/sum_b  <=>  max_i*sum_b <= max_b*sum_i.
  size_t best_c = 0;
  for (size_t c = 1; c < cand_max.size(); ++c) {
    const unsigned __int128 a = static_cast<unsigned __int128>(cand_max[c]) * static_cast<unsigned __int128>(cand_sum[best_c]);
    const unsigned __int128 b = static_cast<unsigned __int128>(cand_max[best_c]) * static_cast<unsigned __int128>(cand_sum[c]);
    if (a <= b) best_c = c;
  }
  const int32_t best = static_cast<int32_t>(first_cand + best_c);

  // The chosen batch: how many of its tokens came from each rank, dealt out over that rank's entries in
  // order; a rank's load grows by the costs n_done+1 .. n_done+t of the t tokens taken from an entry.
  std::vector<int64_t> from_rank(R, 0);
  for (int32_t i = 0; i <= best; ++i) ++from_rank[small_r ? took_from8[i] : took_from32[i]];
  for (int32_t r = 0; r < R; ++r) {
    L[r] = init_load ? init_load[r] : 0;
    int64_t left = from_rank[r];
    for (int32_t e = first[r]; e >= 0 && left > 0; e = next[e]) {
      const int64_t t = left < entries[e].n_new ? left : entries[e].n_new;
      take[e] = static_cast<int32_t>(t);
      L[r] += t * entries[e].n_done + t * (t + 1) / 2;
      left -= t;
    }
  }
  for (int32_t r = 0; r < R; ++r) load[r] = L[r];
  *n_tokens = best + 1;
  return FS_OK;
}
}  // namespace

extern "C" fs_status fs_schedule_prefill(int32_t n_ranks, int32_t budget, int32_t min_tokens,
                                         const fs_prefill_entry* entries, int32_t n_entries,
                                         const int64_t* init_load, int32_t* take, int64_t* load,
                                         int32_t* n_tokens) {
  try {   // nothing may throw across the C boundary
    return schedule_prefill(n_ranks, budget, min_tokens, entries, n_entries, init_load, take, load, n_tokens);
  } catch (const std::bad_alloc&) {
    return fs::fail(FS_ECAPACITY, "fs_schedule_prefill: out of host memory for a budget of %d tokens", budget);
  }
}
