// Host-side router and prefill batch former (integer only, never touches the GPU).
//
// Section 3.1 of the paper, "Fine-grained Load-aware Router": an incoming request goes to
// the rank with the least pending DP work (Load-Aware DP-Rank Routing), and Algorithm 1
// (DP-aware Adaptive Chunked Prefill) fills a token budget one token at a time from the
// least-loaded rank that still has schedulable tokens, then picks the best of the batches
// it passed through.  What the paper leaves open (the token cost, the choice among the
// candidates, the unused workload input) is fixed as the header states.
#include <cstddef>
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

  // The loop of Algorithm 1.  Candidate i (the batch after i+1 tokens) is remembered as the rank it
  // took from plus the largest load and the load sum at that point.
  std::vector<int32_t> took_from;
  std::vector<int64_t> cand_max, cand_sum;
  int64_t waiting = 0;
  for (int32_t e = 0; e < n_entries; ++e) waiting += entries[e].n_new;
  const size_t most = static_cast<size_t>(waiting < budget ? waiting : budget);   // tokens the loop can take
  took_from.reserve(most);
  cand_max.reserve(most);
  cand_sum.reserve(most);
  int64_t sum = 0, mx = 0;
  for (int32_t r = 0; r < R; ++r) { sum += L[r]; if (r == 0 || L[r] > mx) mx = L[r]; }
  while (static_cast<int32_t>(took_from.size()) < budget) {
    int32_t rs = -1;
    for (int32_t r = 0; r < R; ++r)
      if (cur[r] >= 0 && (rs < 0 || L[r] < L[rs])) rs = r;
    if (rs < 0) break;                                    // every S_r is empty
    const fs_prefill_entry& q = entries[cur[rs]];
    const int64_t cost = static_cast<int64_t>(q.n_done) + cur_taken[rs] + 1;   // keys this token attends to
    L[rs] += cost;
    sum += cost;
    if (L[rs] > mx) mx = L[rs];
    if (++cur_taken[rs] == q.n_new) { cur[rs] = next[cur[rs]]; cur_taken[rs] = 0; }
    took_from.push_back(rs);
    cand_max.push_back(mx);
    cand_sum.push_back(sum);
  }

  const int32_t n_all = static_cast<int32_t>(took_from.size());
  if (n_all == 0) {
    for (int32_t r = 0; r < R; ++r) load[r] = L[r];
    *n_tokens = 0;
    return FS_OK;
  }
  // choose_best_batch: smallest max/mean among the candidates of at least min(min_tokens, n_all) tokens,
  // the larger batch among equals.  max_i/sum_i <= max_b/sum_b  <=>  max_i*sum_b <= max_b*sum_i.
  const int32_t lo = min_tokens < n_all ? min_tokens : n_all;
  int32_t best = -1;
  for (int32_t i = (lo > 0 ? lo - 1 : 0); i < n_all; ++i) {
    if (best < 0) { best = i; continue; }
    const unsigned __int128 a = static_cast<unsigned __int128>(cand_max[i]) * static_cast<unsigned __int128>(cand_sum[best]);
    const unsigned __int128 b = static_cast<unsigned __int128>(cand_max[best]) * static_cast<unsigned __int128>(cand_sum[i]);
    if (a <= b) best = i;
  }

  // Replay the first best+1 steps to get the per-entry counts and the loads of the chosen batch.
  cur = first;
  for (int32_t r = 0; r < R; ++r) { cur_taken[r] = 0; L[r] = init_load ? init_load[r] : 0; }
  for (int32_t i = 0; i <= best; ++i) {
    const int32_t r = took_from[i];
    const int32_t e = cur[r];
    L[r] += static_cast<int64_t>(entries[e].n_done) + cur_taken[r] + 1;
    ++take[e];
    if (++cur_taken[r] == entries[e].n_new) { cur[r] = next[e]; cur_taken[r] = 0; }
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
