// Host-side integer builders: head -> rank placement and one rank's work list.
//
// Placement follows the paper's Section 3.1: KV heads go round the ranks
// cyclically with a rotating start (Cyclic Placement); a request is either
// spread that way or kept whole on one rank (Hybrid Attention at request
// granularity); whole requests go to the rank with the least running load
// (Load-Aware DP-Rank Routing).  The work list is the ragged set of (request,
// head) pairs this leaves on a rank, cut into split-K chunks, longest first.
#include <algorithm>
#include <limits>
#include <numeric>
#include <vector>

#include "fs_internal.h"

namespace {

fs_status check_shape(const fs_shape* s, const char* who) {
  if (!s) return fs::fail(FS_EINVAL, "%s: shape is NULL", who);
  if (s->n_req < 0) return fs::fail(FS_EINVAL, "%s: n_req %d < 0", who, s->n_req);
  if (s->n_ranks < 1) return fs::fail(FS_EINVAL, "%s: n_ranks %d < 1", who, s->n_ranks);
  if (s->n_kv_heads < 1) return fs::fail(FS_EINVAL, "%s: n_kv_heads %d < 1", who, s->n_kv_heads);
  return FS_OK;
}

inline int32_t floor_mod(int64_t a, int32_t m) {
  int64_t r = a % m;
  return static_cast<int32_t>(r < 0 ? r + m : r);
}

}  // namespace

extern "C" fs_status fs_build_placement(const fs_shape* shape, const int32_t* ctx_len,
                                        const uint8_t* mode, const int32_t* rot, int32_t layer,
                                        int32_t* owner, int32_t* dp_rank, int64_t* rank_load) {
  if (fs_status st = check_shape(shape, "fs_build_placement")) return st;
  const int32_t B = shape->n_req, H = shape->n_kv_heads, R = shape->n_ranks;
  if (!rank_load) return fs::fail(FS_EINVAL, "fs_build_placement: rank_load is NULL");
  if (B > 0 && (!ctx_len || !mode || !owner || !dp_rank))
    return fs::fail(FS_EINVAL, "fs_build_placement: NULL array with n_req %d", B);
  for (int32_t r = 0; r < B; ++r) {
    const int64_t L = ctx_len[r];
    if (L < 1) return fs::fail(FS_EINVAL, "fs_build_placement: ctx_len[%d] = %d < 1", r, ctx_len[r]);
    int32_t* own = owner + static_cast<int64_t>(r) * H;
    if (mode[r] == FS_MODE_TP) {
      const int64_t start = static_cast<int64_t>(rot ? rot[r] : r) + layer;
      int32_t k = floor_mod(start, R);
      for (int32_t h = 0; h < H; ++h) {
        own[h] = k;
        rank_load[k] += L;
        if (++k == R) k = 0;
      }
      dp_rank[r] = -1;
    } else if (mode[r] == FS_MODE_DP) {
      int32_t best = 0;
      for (int32_t k = 1; k < R; ++k)
        if (rank_load[k] < rank_load[best]) best = k;   // strict: equal loads keep the lowest rank
      std::fill(own, own + H, best);
      dp_rank[r] = best;
      rank_load[best] += static_cast<int64_t>(H) * L;
    } else {
      return fs::fail(FS_EINVAL, "fs_build_placement: mode[%d] = %d is neither TP nor DP", r, mode[r]);
    }
  }
  return FS_OK;
}

extern "C" fs_status fs_build_placement_hybrid_heads(const fs_shape* shape, const int32_t* ctx_len,
                                                     int32_t layer, const int32_t* route,
                                                     int32_t* owner, int32_t* dp_rank,
                                                     int64_t* rank_load, int64_t* dp_load) {
  if (fs_status st = check_shape(shape, "fs_build_placement_hybrid_heads")) return st;
  const int32_t B = shape->n_req, H = shape->n_kv_heads, R = shape->n_ranks;
  if (!rank_load || !dp_load) return fs::fail(FS_EINVAL, "fs_build_placement_hybrid_heads: load arrays are NULL");
  if (B > 0 && (!ctx_len || !owner || !dp_rank))
    return fs::fail(FS_EINVAL, "fs_build_placement_hybrid_heads: NULL array with n_req %d", B);
  const int32_t n_tp = (H / R) * R;     // heads every worker shares evenly
  const int32_t n_dp = H - n_tp;        // leftover heads, replicated and run data-parallel
  const int32_t first = floor_mod(layer, R);
  for (int32_t r = 0; r < B; ++r) {
    const int64_t L = ctx_len[r];
    if (L < 1)
      return fs::fail(FS_EINVAL, "fs_build_placement_hybrid_heads: ctx_len[%d] = %d < 1", r, ctx_len[r]);
    int32_t* own = owner + static_cast<int64_t>(r) * H;
    int32_t k = first;
    for (int32_t h = 0; h < n_tp; ++h) {
      own[h] = k;
      rank_load[k] += L;
      if (++k == R) k = 0;
    }
    if (n_dp == 0) {
      dp_rank[r] = -1;
      continue;
    }
    int32_t best = 0;
    if (route) {
      best = route[r];
      if (best < 0 || best >= R)
        return fs::fail(FS_EINVAL, "fs_build_placement_hybrid_heads: route[%d] = %d outside [0, %d)", r, best, R);
    } else {
      for (int32_t j = 1; j < R; ++j)
        if (dp_load[j] < dp_load[best]) best = j;   // pending DP work only; equal loads keep the lowest rank
    }
    std::fill(own + n_tp, own + H, best);
    dp_rank[r] = best;
    rank_load[best] += n_dp * L;
    dp_load[best] += n_dp * L;
  }
  return FS_OK;
}

extern "C" fs_status fs_choose_chunk_tokens(const fs_shape* shape, const int32_t* ctx_len, const int32_t* owner,
                                            int32_t rank, int32_t max_chunk, int32_t min_chunk, int64_t n_slots,
                                            int32_t* chunk_tokens, int64_t* n_items) {
  if (fs_status st = check_shape(shape, "fs_choose_chunk_tokens")) return st;
  const int32_t B = shape->n_req, H = shape->n_kv_heads, R = shape->n_ranks, T = shape->page_tokens;
  if (!chunk_tokens || !n_items) return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: outputs are NULL");
  if (T < 1) return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: page_tokens %d < 1", T);
  if (rank < 0 || rank >= R) return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: rank %d outside [0, %d)", rank, R);
  if (min_chunk < T || min_chunk % T || max_chunk < min_chunk || max_chunk % T)
    return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: chunks [%d, %d] must be multiples of page_tokens %d, min <= max",
                    min_chunk, max_chunk, T);
  if (n_slots < 1) return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: n_slots %lld < 1", static_cast<long long>(n_slots));
  if (B > 0 && (!ctx_len || !owner)) return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: NULL input array");
  for (int32_t r = 0; r < B; ++r) {
    if (ctx_len[r] < 1) return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: ctx_len[%d] = %d < 1", r, ctx_len[r]);
    for (int32_t h = 0; h < H; ++h) {
      const int32_t k = owner[static_cast<int64_t>(r) * H + h];
      if (k < 0 || k >= R)
        return fs::fail(FS_EINVAL, "fs_choose_chunk_tokens: owner[%d][%d] = %d outside [0, %d)", r, h, k, R);
    }
  }
  // Four thirds of a slot's fair share of the tokens the rank holds, up to whole pages, within the bounds.
  int64_t total = 0;
  for (int32_t r = 0; r < B; ++r)
    for (int32_t h = 0; h < H; ++h)
      if (owner[static_cast<int64_t>(r) * H + h] == rank) total += ctx_len[r];
  const int64_t target = (4 * total + 3 * n_slots - 1) / (3 * n_slots);
  int64_t C = (target + T - 1) / T * T;
  C = std::min<int64_t>(std::max<int64_t>(C, min_chunk), max_chunk);
  int64_t ni = 0;
  for (int32_t r = 0; r < B; ++r) {
    const int64_t nc = (static_cast<int64_t>(ctx_len[r]) + C - 1) / C;
    for (int32_t h = 0; h < H; ++h)
      if (owner[static_cast<int64_t>(r) * H + h] == rank) ni += nc;
  }
  *chunk_tokens = static_cast<int32_t>(C);
  *n_items = ni;
  return FS_OK;
}

extern "C" fs_status fs_build_worklist(const fs_shape* shape, const int32_t* ctx_len,
                                       const int32_t* owner, int32_t rank, int32_t chunk_tokens,
                                       fs_work_item* items, int64_t items_cap,
                                       fs_pair* pairs, int64_t pairs_cap,
                                       int32_t* sched, int64_t* chunk_indptr,
                                       int64_t* n_items, int64_t* n_pairs) {
  if (fs_status st = check_shape(shape, "fs_build_worklist")) return st;
  const int32_t B = shape->n_req, H = shape->n_kv_heads, R = shape->n_ranks;
  if (!n_items || !n_pairs) return fs::fail(FS_EINVAL, "fs_build_worklist: count outputs are NULL");
  if (shape->page_tokens < 1)
    return fs::fail(FS_EINVAL, "fs_build_worklist: page_tokens %d < 1", shape->page_tokens);
  if (shape->n_q_heads < H || shape->n_q_heads % H)
    return fs::fail(FS_EINVAL, "fs_build_worklist: n_q_heads %d is not a multiple of n_kv_heads %d",
                    shape->n_q_heads, H);
  if (rank < 0 || rank >= R) return fs::fail(FS_EINVAL, "fs_build_worklist: rank %d outside [0, %d)", rank, R);
  if (chunk_tokens < 0 || chunk_tokens % shape->page_tokens)
    return fs::fail(FS_EINVAL, "fs_build_worklist: chunk_tokens %d is not a multiple of page_tokens %d",
                    chunk_tokens, shape->page_tokens);
  if (B > 0 && (!ctx_len || !owner)) return fs::fail(FS_EINVAL, "fs_build_worklist: NULL input array");
  const bool count_only = !items && !pairs && !sched && !chunk_indptr;
  if (items_cap < 0 || pairs_cap < 0 || (!items && items_cap) || (!pairs && pairs_cap) || (!sched && items_cap))
    return fs::fail(FS_EINVAL, "fs_build_worklist: capacities do not match the arrays");
  const int32_t G = shape->n_q_heads / H;
  const int64_t C = chunk_tokens;

  // Pass 1: validate and count, so that a short array is reported before anything is written.
  int64_t ni = 0, np = 0;
  for (int32_t r = 0; r < B; ++r) {
    const int64_t L = ctx_len[r];
    if (L < 1) return fs::fail(FS_EINVAL, "fs_build_worklist: ctx_len[%d] = %d < 1", r, ctx_len[r]);
    const int64_t nc = C ? (L + C - 1) / C : 1;
    for (int32_t h = 0; h < H; ++h) {
      const int32_t k = owner[static_cast<int64_t>(r) * H + h];
      if (k < 0 || k >= R)
        return fs::fail(FS_EINVAL, "fs_build_worklist: owner[%d][%d] = %d outside [0, %d)", r, h, k, R);
      if (k == rank) { ++np; ni += nc; }
    }
  }
  *n_items = ni;
  *n_pairs = np;
  if (ni * G > std::numeric_limits<int32_t>::max() ||
      static_cast<int64_t>(B) * shape->n_q_heads > std::numeric_limits<int32_t>::max())
    return fs::fail(FS_EINVAL, "fs_build_worklist: row numbers exceed int32 (%lld items x G=%d)",
                    static_cast<long long>(ni), G);
  if (count_only) return FS_OK;
  if (items_cap < ni || pairs_cap < np)
    return fs::fail(FS_ECAPACITY, "fs_build_worklist: need %lld items and %lld pairs, have room for %lld and %lld",
                    static_cast<long long>(ni), static_cast<long long>(np),
                    static_cast<long long>(items_cap), static_cast<long long>(pairs_cap));

  if (!chunk_indptr) return fs::fail(FS_EINVAL, "fs_build_worklist: chunk_indptr is NULL (it has n_pairs+1 entries)");

  // Pass 2: emit.  (An array whose count is zero may be NULL: the capacity checks above cover it.)
  int64_t i = 0, p = 0;
  for (int32_t r = 0; r < B; ++r) {
    const int32_t L = ctx_len[r];
    const int32_t nc = static_cast<int32_t>(C ? (L + C - 1) / C : 1);
    for (int32_t h = 0; h < H; ++h) {
      if (owner[static_cast<int64_t>(r) * H + h] != rank) continue;
      pairs[p] = fs_pair{r, h, L, nc};
      chunk_indptr[p] = i;
      {
        for (int32_t c = 0; c < nc; ++c) {
          fs_work_item& it = items[i + c];
          it.req = r;
          it.kv_head = h;
          it.tok_begin = C ? static_cast<int32_t>(c * C) : 0;
          it.tok_end = C ? static_cast<int32_t>(std::min<int64_t>(L, (c + 1) * C)) : L;
          it.pair = static_cast<int32_t>(p);
          it.chunk = c;
          it.q_row = r * shape->n_q_heads + h * G;
          it.part_row = static_cast<int32_t>((i + c) * G);
        }
      }
      i += nc;
      ++p;
    }
  }
  chunk_indptr[np] = ni;

  if (ni > 0) {
    // Longest first; equal lengths keep index order.  Lengths are bounded by the chunk size (or
    // the longest context), so a counting sort keeps this linear for big batches.
    int32_t max_len = 0;
    for (int64_t j = 0; j < ni; ++j) max_len = std::max(max_len, items[j].tok_end - items[j].tok_begin);
    if (static_cast<int64_t>(max_len) <= 4 * ni + 1024) {
      std::vector<int64_t> start(static_cast<size_t>(max_len) + 2, 0);
      for (int64_t j = 0; j < ni; ++j) ++start[max_len - (items[j].tok_end - items[j].tok_begin) + 1];
      for (size_t b = 1; b < start.size(); ++b) start[b] += start[b - 1];
      for (int64_t j = 0; j < ni; ++j)
        sched[start[max_len - (items[j].tok_end - items[j].tok_begin)]++] = static_cast<int32_t>(j);
    } else {
      std::iota(sched, sched + ni, 0);
      std::stable_sort(sched, sched + ni, [&](int32_t a, int32_t b) {
        return items[a].tok_end - items[a].tok_begin > items[b].tok_end - items[b].tok_begin;
      });
    }
  }
  return FS_OK;
}

extern "C" fs_status fs_build_worklist_units(const fs_shape* shape, const int32_t* ctx_len, const int32_t* owner,
                                             int32_t rank, int32_t n_units,
                                             fs_work_item* items, int64_t items_cap,
                                             fs_pair* pairs, int64_t pairs_cap,
                                             int64_t* unit_indptr, int64_t units_cap, int64_t* chunk_indptr,
                                             int64_t* n_items, int64_t* n_pairs, int64_t* n_units_out) {
  const char* who = "fs_build_worklist_units";
  if (fs_status st = check_shape(shape, who)) return st;
  const int32_t B = shape->n_req, H = shape->n_kv_heads, R = shape->n_ranks, T = shape->page_tokens;
  if (!n_items || !n_pairs || !n_units_out) return fs::fail(FS_EINVAL, "%s: count outputs are NULL", who);
  if (T < 1) return fs::fail(FS_EINVAL, "%s: page_tokens %d < 1", who, T);
  if (shape->n_q_heads < H || shape->n_q_heads % H)
    return fs::fail(FS_EINVAL, "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, shape->n_q_heads, H);
  if (rank < 0 || rank >= R) return fs::fail(FS_EINVAL, "%s: rank %d outside [0, %d)", who, rank, R);
  if (n_units < 1) return fs::fail(FS_EINVAL, "%s: n_units %d < 1", who, n_units);
  if (B > 0 && (!ctx_len || !owner)) return fs::fail(FS_EINVAL, "%s: NULL input array", who);
  const bool count_only = !items && !pairs && !unit_indptr && !chunk_indptr;
  if (items_cap < 0 || pairs_cap < 0 || units_cap < 0 || (!items && items_cap) || (!pairs && pairs_cap))
    return fs::fail(FS_EINVAL, "%s: capacities do not match the arrays", who);
  const int32_t G = shape->n_q_heads / H;

  // Pass 1: validate, count the pairs and the pages of the stream.
  int64_t np = 0, P = 0;
  for (int32_t r = 0; r < B; ++r) {
    if (ctx_len[r] < 1) return fs::fail(FS_EINVAL, "%s: ctx_len[%d] = %d < 1", who, r, ctx_len[r]);
    const int64_t pages = (static_cast<int64_t>(ctx_len[r]) + T - 1) / T;
    for (int32_t h = 0; h < H; ++h) {
      const int32_t k = owner[static_cast<int64_t>(r) * H + h];
      if (k < 0 || k >= R) return fs::fail(FS_EINVAL, "%s: owner[%d][%d] = %d outside [0, %d)", who, r, h, k, R);
      if (k == rank) { ++np; P += pages; }
    }
  }
  const int64_t U = std::min<int64_t>(n_units, P);
  // Unit u holds stream pages [cut(u), cut(u+1)), cut(u) = floor(u*P/U): equal runs to within one page.
  auto cut = [&](int64_t u) { return U ? u * P / U : 0; };

  // One walk serves the count and the emission: pairs in (request, head) order, each cut where a unit ends.
  auto walk = [&](auto&& on_item, auto&& on_pair, auto&& on_unit) {
    int64_t start = 0, u = 0, next_cut = cut(1), i = 0, p = 0;
    for (int32_t r = 0; r < B; ++r) {
      const int32_t L = ctx_len[r];
      const int64_t pages = (static_cast<int64_t>(L) + T - 1) / T;
      for (int32_t h = 0; h < H; ++h) {
        if (owner[static_cast<int64_t>(r) * H + h] != rank) continue;
        int64_t done = 0;
        int32_t c = 0;
        const int64_t first_item = i;
        while (done < pages) {
          while (start + done >= next_cut) {      // the stream has left unit u
            ++u;
            on_unit(u, i);
            next_cut = cut(u + 1);
          }
          const int64_t take = std::min(pages - done, next_cut - (start + done));
          on_item(i, r, h, p, c, static_cast<int32_t>(done * T),
                  static_cast<int32_t>(std::min<int64_t>(L, (done + take) * T)));
          done += take;
          ++c;
          ++i;
        }
        on_pair(p, r, h, L, c, first_item);
        start += pages;
        ++p;
      }
    }
    return i;
  };
  const int64_t ni = walk([](auto...) {}, [](auto...) {}, [](auto...) {});
  *n_items = ni;
  *n_pairs = np;
  *n_units_out = U;
  if (ni * G > std::numeric_limits<int32_t>::max() ||
      static_cast<int64_t>(B) * shape->n_q_heads > std::numeric_limits<int32_t>::max())
    return fs::fail(FS_EINVAL, "%s: row numbers exceed int32 (%lld items x G=%d)", who, static_cast<long long>(ni), G);
  if (count_only) return FS_OK;
  if (items_cap < ni || pairs_cap < np || units_cap < U)
    return fs::fail(FS_ECAPACITY, "%s: need %lld items, %lld pairs and %lld units, have room for %lld, %lld and %lld", who,
                    static_cast<long long>(ni), static_cast<long long>(np), static_cast<long long>(U),
                    static_cast<long long>(items_cap), static_cast<long long>(pairs_cap), static_cast<long long>(units_cap));
  if (!unit_indptr || !chunk_indptr)
    return fs::fail(FS_EINVAL, "%s: unit_indptr (n_units+1 entries) or chunk_indptr (n_pairs+1 entries) is NULL", who);

  unit_indptr[0] = 0;
  walk(
      [&](int64_t i, int32_t r, int32_t h, int64_t p, int32_t c, int32_t tok_begin, int32_t tok_end) {
        items[i] = fs_work_item{r, h, tok_begin, tok_end, static_cast<int32_t>(p), c,
                                r * shape->n_q_heads + h * G, static_cast<int32_t>(i * G)};
      },
      [&](int64_t p, int32_t r, int32_t h, int32_t L, int32_t c, int64_t first_item) {
        pairs[p] = fs_pair{r, h, L, c};
        chunk_indptr[p] = first_item;
      },
      [&](int64_t u, int64_t i) { unit_indptr[u] = i; });
  chunk_indptr[np] = ni;
  unit_indptr[U] = ni;
  return FS_OK;
}

extern "C" fs_status fs_build_launch_records(const fs_shape* shape, const fs_work_item* items, const int32_t* order,
                                             int64_t n_items, const int64_t* chunk_indptr, int64_t n_pairs,
                                             const int64_t* page_indptr, const int32_t* page_ids, int64_t n_page_ids,
                                             int32_t direct_rows, fs_launch_record* records) {
  const char* who = "fs_build_launch_records";
  if (fs_status st = check_shape(shape, who)) return st;
  const int32_t H = shape->n_kv_heads, T = shape->page_tokens;
  if (T < 1 || shape->n_q_heads < H || shape->n_q_heads % H)
    return fs::fail(FS_EINVAL, "%s: bad page_tokens %d or head counts %d/%d", who, T, shape->n_q_heads, H);
  if (n_items < 0 || n_pairs < 0 || n_page_ids < 0) return fs::fail(FS_EINVAL, "%s: negative count", who);
  if (n_items == 0) return FS_OK;
  if (!items || !chunk_indptr || !page_indptr || !page_ids || !records)
    return fs::fail(FS_EINVAL, "%s: NULL pointer", who);
  const int32_t G = shape->n_q_heads / H;
  for (int64_t k = 0; k < n_items; ++k) {
    const int64_t i = order ? order[k] : k;
    if (i < 0 || i >= n_items) return fs::fail(FS_EINVAL, "%s: order[%lld] = %lld outside [0, %lld)", who,
                                               static_cast<long long>(k), static_cast<long long>(i), static_cast<long long>(n_items));
    const fs_work_item& it = items[i];
    if (it.pair < 0 || it.pair >= n_pairs || it.tok_begin < 0 || it.tok_end <= it.tok_begin || it.tok_begin % T)
      return fs::fail(FS_EINVAL, "%s: item %lld is malformed (pair %d, tokens [%d, %d))", who, static_cast<long long>(i),
                      it.pair, it.tok_begin, it.tok_end);
    const int64_t first_page = page_indptr[it.pair] + it.tok_begin / T;
    const int64_t n_pages = (static_cast<int64_t>(it.tok_end) - it.tok_begin + T - 1) / T;
    if (first_page < 0 || first_page + n_pages > page_indptr[it.pair + 1] || page_indptr[it.pair + 1] > n_page_ids)
      return fs::fail(FS_EINVAL, "%s: item %lld's pages [%lld, %lld) leave its pair's part of the page table", who,
                      static_cast<long long>(i), static_cast<long long>(first_page), static_cast<long long>(first_page + n_pages));
    const int64_t c0 = chunk_indptr[it.pair], n_chunks = chunk_indptr[it.pair + 1] - c0;
    if (n_chunks < 1 || it.chunk < 0 || it.chunk >= n_chunks || (c0 + n_chunks) * G > 0x7FFFFFFFll ||
        it.part_row != (c0 + it.chunk) * G)
      return fs::fail(FS_EINVAL, "%s: item %lld (pair %d, chunk %d, part_row %d) does not sit at row (chunk_indptr[pair] + chunk) * G "
                      "of its pair's %lld chunks", who, static_cast<long long>(i), it.pair, it.chunk, it.part_row,
                      static_cast<long long>(n_chunks));
    fs_launch_record& r = records[k];
    r.first_page = first_page;
    r.n_tok = it.tok_end - it.tok_begin;
    r.q_row = it.q_row;
    r.row = (direct_rows && n_chunks == 1) ? -(it.pair * G) - 1 : it.part_row;
    r.n_chunks = static_cast<int32_t>(n_chunks);
    for (int j = 0; j < 8; ++j) r.first_slots[j] = j < n_pages ? page_ids[first_page + j] : 0;
    r.pair = it.pair;
    r.pair_row = static_cast<int32_t>(c0 * G);
  }
  return FS_OK;
}

extern "C" int32_t fs_kv_elem_offset(int32_t kv_dtype, int32_t is_v, int32_t tok, int32_t d) {
  if (tok < 0 || tok >= fs::kPageTokens || d < 0 || d >= fs::kHeadDim) return -1;
  if (kv_dtype == FS_KV_FP8_E4M3)   // K and V: [d/64][(d%64)/16][tok][d%16]: one 16-byte piece per (token, 16 d), 64 pieces to a 1 KiB run
    return (d / 64) * 1024 + ((d % 64) / 16) * 256 + tok * 16 + (d % 16);
  if (kv_dtype != FS_KV_BF16) return -1;
  if (!is_v)   // K: [d/32][(d%32)/8][tok][d%8]: one 16-byte piece per (token, 8 d) in MFMA A-operand order
    return (d / 32) * 512 + ((d % 32) / 8) * 128 + tok * 8 + (d % 8);
  // V: [d/32][tok/4][d%16][(d/16)%2][tok%4]: four tokens of one d sit together (the MFMA reduces over tokens)
  return (d / 32) * 512 + (tok / 4) * 128 + (d % 16) * 8 + ((d / 16) % 2) * 4 + (tok % 4);
}
