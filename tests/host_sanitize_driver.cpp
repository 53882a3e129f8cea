// Host-side builders under AddressSanitizer + UBSan: random batches through the host
// entry points with exactly-sized output arrays (so any write past the end is caught) and a few
// structural checks.  Built and run by tests/test_host_sanitizers.py; touches no GPU.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "failsafe.h"

#define REQUIRE(c)                                                        \
  do {                                                                    \
    if (!(c)) {                                                           \
      std::fprintf(stderr, "FAILED %s at line %d (case %d)\n", #c, __LINE__, g_case); \
      return 1;                                                           \
    }                                                                     \
  } while (0)

static int g_case = 0;

int main() {
  std::mt19937 rng(12345);
  for (g_case = 0; g_case < 400; ++g_case) {
    const int R = 1 + rng() % 8, H = 1 + rng() % 9, G = 1 + rng() % 4, B = rng() % 20;
    fs_shape sh{B, H * G, H, 128, 16, R};
    std::vector<int32_t> ctx(B);
    std::vector<uint8_t> mode(B);
    for (int r = 0; r < B; ++r) {
      ctx[r] = 1 + rng() % 5000;
      mode[r] = rng() % 3 == 0;
    }
    std::vector<int32_t> owner(static_cast<size_t>(B) * H), dp(B);
    std::vector<int64_t> load(R, 0), dload(R, 0);
    if (g_case % 2 == 0) {
      REQUIRE(fs_build_placement(&sh, ctx.data(), mode.data(), nullptr, static_cast<int32_t>(rng() % 50) - 10,
                                 owner.data(), dp.data(), load.data()) == FS_OK);
    } else {
      REQUIRE(fs_build_placement_hybrid_heads(&sh, ctx.data(), static_cast<int32_t>(rng() % 50) - 10, nullptr,
                                              owner.data(), dp.data(), load.data(), dload.data()) == FS_OK);
    }
    int64_t total = 0;
    for (int r = 0; r < B; ++r) total += static_cast<int64_t>(ctx[r]) * H;
    int64_t sum = 0;
    for (int64_t x : load) sum += x;
    REQUIRE(sum == total);
    const int chunks[] = {0, 16, 64, 1024};
    const int chunk = chunks[rng() % 4];
    int64_t covered = 0;
    for (int k = 0; k < R; ++k) {
      int64_t ni = -1, np = -1;
      REQUIRE(fs_build_worklist(&sh, ctx.data(), owner.data(), k, chunk, nullptr, 0, nullptr, 0, nullptr, nullptr,
                                &ni, &np) == FS_OK);
      std::vector<fs_work_item> items(ni);
      std::vector<fs_pair> pairs(np);
      std::vector<int32_t> sched(ni);
      std::vector<int64_t> indptr(np + 1);
      REQUIRE(fs_build_worklist(&sh, ctx.data(), owner.data(), k, chunk, items.data(), ni, pairs.data(), np,
                                sched.data(), indptr.data(), &ni, &np) == FS_OK);
      int64_t toks = 0;
      for (const auto& it : items) toks += it.tok_end - it.tok_begin;
      REQUIRE(toks == load[k]);
      for (int64_t j = 1; j < ni; ++j) {
        const auto& a = items[sched[j - 1]];
        const auto& b = items[sched[j]];
        REQUIRE(a.tok_end - a.tok_begin >= b.tok_end - b.tok_begin);
      }
      REQUIRE(indptr[np] == ni);
      covered += np;
      {   // the chunk chooser agrees with the builder on the list's length and stays inside its bounds
        int32_t chosen = -1;
        int64_t n_chosen = -1, n_check = -1, p_check = -1;
        const int64_t slots = 1 + rng() % 64;
        REQUIRE(fs_choose_chunk_tokens(&sh, ctx.data(), owner.data(), k, 1024, 16, slots, &chosen, &n_chosen) == FS_OK);
        REQUIRE(chosen >= 16 && chosen <= 1024 && chosen % 16 == 0);
        REQUIRE(fs_build_worklist(&sh, ctx.data(), owner.data(), k, chosen, nullptr, 0, nullptr, 0, nullptr, nullptr,
                                  &n_check, &p_check) == FS_OK);
        REQUIRE(n_check == n_chosen);
      }
      if (ni > 0) {   // one slot too few must be refused, not overrun
        std::vector<fs_work_item> small(ni - 1);
        std::vector<int32_t> ssched(ni - 1);
        int64_t a = 0, b = 0;
        REQUIRE(fs_build_worklist(&sh, ctx.data(), owner.data(), k, chunk, small.data(), ni - 1, pairs.data(), np,
                                  ssched.data(), indptr.data(), &a, &b) == FS_ECAPACITY);
        REQUIRE(a == ni && b == np);
      }
    }
    REQUIRE(covered == static_cast<int64_t>(B) * H);
  }
  // the list cut into equal runs: exactly-sized arrays, runs equal to within a page, every pair tiled
  for (g_case = 500; g_case < 900; ++g_case) {
    const int R = 1 + rng() % 5, H = 1 + rng() % 8, G = 1 + rng() % 4, B = rng() % 14;
    fs_shape sh{B, H * G, H, 128, 16, R};
    std::vector<int32_t> ctx(B), owner(static_cast<size_t>(B) * H);
    for (auto& c : ctx) c = 1 + rng() % (rng() % 2 ? 60 : 3000);
    for (auto& o : owner) o = rng() % R;
    const int32_t rank = rng() % R, n_units = 1 + rng() % (rng() % 2 ? 8 : 700);
    int64_t ni = -1, np = -1, nu = -1;
    REQUIRE(fs_build_worklist_units(&sh, ctx.data(), owner.data(), rank, n_units, nullptr, 0, nullptr, 0, nullptr, 0,
                                    nullptr, &ni, &np, &nu) == FS_OK);
    std::vector<fs_work_item> items(ni);
    std::vector<fs_pair> pairs(np);
    std::vector<int64_t> unit_indptr(nu + 1), chunk_indptr(np + 1);
    int64_t ni2 = -1, np2 = -1, nu2 = -1;
    REQUIRE(fs_build_worklist_units(&sh, ctx.data(), owner.data(), rank, n_units, items.data(), ni, pairs.data(), np,
                                    unit_indptr.data(), nu, chunk_indptr.data(), &ni2, &np2, &nu2) == FS_OK);
    REQUIRE(ni2 == ni && np2 == np && nu2 == nu && unit_indptr[0] == 0 && unit_indptr[nu] == ni && chunk_indptr[np] == ni);
    REQUIRE(ni <= np + (nu > 0 ? nu - 1 : 0));
    int64_t lo = INT64_MAX, hi = 0;
    for (int64_t u = 0; u < nu; ++u) {
      int64_t pages = 0;
      REQUIRE(unit_indptr[u + 1] > unit_indptr[u]);
      for (int64_t i = unit_indptr[u]; i < unit_indptr[u + 1]; ++i) pages += (items[i].tok_end - items[i].tok_begin + 15) / 16;
      lo = pages < lo ? pages : lo;
      hi = pages > hi ? pages : hi;
    }
    REQUIRE(nu == 0 || hi - lo <= 1);
    for (int64_t p = 0; p < np; ++p) {
      REQUIRE(items[chunk_indptr[p]].tok_begin == 0 && items[chunk_indptr[p + 1] - 1].tok_end == pairs[p].ctx_len);
      for (int64_t i = chunk_indptr[p] + 1; i < chunk_indptr[p + 1]; ++i) REQUIRE(items[i].tok_begin == items[i - 1].tok_end);
    }
    {   // launch records of the same list: exactly-sized output, every record restates its item
      std::vector<int64_t> page_indptr(np + 1, 0);
      for (int64_t p = 0; p < np; ++p) page_indptr[p + 1] = page_indptr[p] + (pairs[p].ctx_len + 15) / 16;
      std::vector<int32_t> page_ids(page_indptr[np]);
      for (size_t j = 0; j < page_ids.size(); ++j) page_ids[j] = static_cast<int32_t>(1000 + j);
      std::vector<fs_launch_record> rec(ni);
      REQUIRE(fs_build_launch_records(&sh, items.data(), nullptr, ni, chunk_indptr.data(), np, page_indptr.data(),
                                      page_ids.data(), static_cast<int64_t>(page_ids.size()), 1, rec.data()) == FS_OK);
      for (int64_t i = 0; i < ni; ++i) {
        REQUIRE(rec[i].n_tok == items[i].tok_end - items[i].tok_begin && rec[i].q_row == items[i].q_row);
        REQUIRE(rec[i].first_page == page_indptr[items[i].pair] + items[i].tok_begin / 16);
        REQUIRE(rec[i].first_slots[0] == 1000 + rec[i].first_page);
        const bool single = chunk_indptr[items[i].pair + 1] - chunk_indptr[items[i].pair] == 1;
        REQUIRE(rec[i].row == (single ? -(items[i].pair * G) - 1 : items[i].part_row));
      }
    }
    if (ni > 1) {
      std::vector<fs_work_item> small(ni - 1);
      REQUIRE(fs_build_worklist_units(&sh, ctx.data(), owner.data(), rank, n_units, small.data(), ni - 1, pairs.data(), np,
                                      unit_indptr.data(), nu, chunk_indptr.data(), &ni2, &np2, &nu2) == FS_ECAPACITY);
    }
  }
  // router and prefill scheduler: exactly-sized arrays, token conservation, budget respected
  for (g_case = 1000; g_case < 1300; ++g_case) {
    const int R = 1 + rng() % 12, n = rng() % 12;   // up to 8 ranks: packed keys; beyond: the linear search
    std::vector<int64_t> pending(R, 0);
    std::vector<fs_prefill_entry> ent(n);
    int64_t waiting = 0;
    for (int e = 0; e < n; ++e) {
      const int32_t n_new = rng() % 50;
      int32_t rank = -1;
      REQUIRE(fs_route_request(R, pending.data(), n_new, &rank) == FS_OK);
      REQUIRE(rank >= 0 && rank < R);
      ent[e] = fs_prefill_entry{e, rank, static_cast<int32_t>(rng() % 100000), n_new};
      waiting += n_new;
    }
    {   // the queue form places the same requests the same way
      std::vector<int64_t> pending2(R, 0), work(n);
      std::vector<int32_t> ranks(n);
      for (int e = 0; e < n; ++e) work[e] = ent[e].n_new;
      REQUIRE(fs_route_requests(R, pending2.data(), work.data(), n, ranks.data()) == FS_OK);
      for (int e = 0; e < n; ++e) REQUIRE(ranks[e] == ent[e].rank);
      REQUIRE(pending2 == pending);
    }
    const int budget = rng() % 200, floor_tokens = rng() % 220;
    std::vector<int32_t> take(n);
    std::vector<int64_t> load(R);
    int32_t n_tok = -1;
    REQUIRE(fs_schedule_prefill(R, budget, floor_tokens, ent.data(), n, nullptr, take.data(), load.data(), &n_tok) == FS_OK);
    int64_t sum = 0;
    for (int e = 0; e < n; ++e) {
      REQUIRE(take[e] >= 0 && take[e] <= ent[e].n_new);
      sum += take[e];
    }
    REQUIRE(sum == n_tok && n_tok <= budget && n_tok <= waiting);
    if (floor_tokens >= budget) REQUIRE(n_tok == (waiting < budget ? waiting : budget));
  }
  // recovery planner: exactly-sized arrays, conservation of slices and shards
  for (g_case = 2000; g_case < 2300; ++g_case) {
    const int n = 1 + rng() % 8, B = rng() % 16, H = 1 + rng() % 8, S = rng() % 40;
    std::vector<uint8_t> alive(n);
    for (auto& a : alive) a = rng() % 2;
    alive[rng() % n] = 1;
    std::vector<int32_t> ctx(B), old_owner(static_cast<size_t>(B) * H), old_dp(B), new_owner(old_owner.size()), new_dp(B);
    for (auto& c : ctx) c = 1 + rng() % 3000;
    for (auto& o : old_owner) o = rng() % n;
    for (auto& d : old_dp) d = static_cast<int32_t>(rng() % (n + 1)) - 1;
    std::vector<int64_t> dload(n, 0), reload(n), reuse(n);
    REQUIRE(fs_replace_failed_gpu(B, H, ctx.data(), old_owner.data(), old_dp.data(), n, alive.data(), new_owner.data(),
                                  new_dp.data(), dload.data()) == FS_OK);
    REQUIRE(fs_plan_kv_reload(B, H, ctx.data(), old_owner.data(), new_owner.data(), n, alive.data(), reload.data(),
                              reuse.data()) == FS_OK);
    int64_t moved = 0, kept = 0, lost = 0, total = 0;
    for (int g = 0; g < n; ++g) { moved += reload[g]; kept += reuse[g]; }
    for (int r = 0; r < B; ++r)
      for (int h = 0; h < H; ++h) {
        total += ctx[r];
        if (!alive[old_owner[static_cast<size_t>(r) * H + h]]) lost += ctx[r];
        REQUIRE(alive[new_owner[static_cast<size_t>(r) * H + h]]);
      }
    REQUIRE(moved == lost && moved + kept == total);
    std::vector<int32_t> shard_owner(S), shard_new(S), n_load(n);
    for (auto& o : shard_owner) o = rng() % n;
    REQUIRE(fs_plan_ffn_reload(S, shard_owner.data(), n, alive.data(), shard_new.data(), n_load.data()) == FS_OK);
    int loaded = 0, dead = 0;
    for (int g = 0; g < n; ++g) loaded += n_load[g];
    for (int s = 0; s < S; ++s) { dead += !alive[shard_owner[s]]; REQUIRE(alive[shard_new[s]]); }
    REQUIRE(loaded == dead);
  }
  // prefill tile list: exactly-sized arrays, every new token of every owned pair in exactly one tile,
  // every tile's keys tiled by its chunks without gap or overlap
  for (g_case = 3000; g_case < 3300; ++g_case) {
    const int R = 1 + rng() % 5, H = 1 + rng() % 6, G = 1 + rng() % 8, B = rng() % 10;
    fs_shape sh{B, H * G, H, 128, 16, R};
    std::vector<int32_t> n_done(B), n_new(B), owner(static_cast<size_t>(B) * H);
    for (int r = 0; r < B; ++r) {
      n_done[r] = rng() % 3 ? static_cast<int32_t>(rng() % 2000) : 0;
      n_new[r] = rng() % 4 ? static_cast<int32_t>(rng() % 300) : 0;
    }
    for (auto& o : owner) o = rng() % R;
    const int32_t rank = rng() % R, tile = 1 + rng() % 40, chunk = 32 * (rng() % 9);
    int64_t ni = -1, np = -1, nt = -1;
    REQUIRE(fs_build_prefill_worklist(&sh, n_done.data(), n_new.data(), owner.data(), rank, tile, chunk, nullptr, 0,
                                      nullptr, 0, nullptr, nullptr, 0, nullptr, &ni, &np, &nt) == FS_OK);
    std::vector<fs_prefill_item> items(ni);
    std::vector<fs_prefill_pair> pairs(np);
    std::vector<int32_t> sched(ni);
    std::vector<int64_t> chunk_indptr(nt + 1), out_indptr(np + 1);
    int64_t ni2 = -1, np2 = -1, nt2 = -1;
    REQUIRE(fs_build_prefill_worklist(&sh, n_done.data(), n_new.data(), owner.data(), rank, tile, chunk, items.data(), ni,
                                      pairs.data(), np, sched.data(), chunk_indptr.data(), nt, out_indptr.data(), &ni2,
                                      &np2, &nt2) == FS_OK);
    REQUIRE(ni2 == ni && np2 == np && nt2 == nt && chunk_indptr[0] == 0 && chunk_indptr[nt] == ni);
    int64_t tokens = 0, want = 0;
    for (int r = 0; r < B; ++r)
      for (int h = 0; h < H; ++h)
        if (owner[static_cast<size_t>(r) * H + h] == rank) want += n_new[r];
    for (int64_t t = 0; t < nt; ++t) {
      const int64_t a = chunk_indptr[t], b = chunk_indptr[t + 1];
      REQUIRE(b > a);
      const fs_prefill_item& first = items[a];
      tokens += first.q_end - first.q_begin;
      REQUIRE(first.kv_begin == 0 && items[b - 1].kv_end == first.n_done + first.q_end);
      for (int64_t i = a + 1; i < b; ++i) REQUIRE(items[i].kv_begin == items[i - 1].kv_end && items[i].pair == first.pair);
    }
    REQUIRE(tokens == want);
    std::vector<char> seen(ni, 0);
    for (int64_t i = 0; i < ni; ++i) {
      REQUIRE(sched[i] >= 0 && sched[i] < ni && !seen[sched[i]]);
      seen[sched[i]] = 1;
    }
    if (ni > 1) {   // one item short: the call must refuse, not write past the end
      std::vector<fs_prefill_item> small(ni - 1);
      std::vector<int32_t> sched_small(ni - 1);
      REQUIRE(fs_build_prefill_worklist(&sh, n_done.data(), n_new.data(), owner.data(), rank, tile, chunk, small.data(),
                                        ni - 1, pairs.data(), np, sched_small.data(), chunk_indptr.data(), nt,
                                        out_indptr.data(), &ni2, &np2, &nt2) == FS_ECAPACITY);
    }
  }
  // error paths leave a message
  fs_shape bad{1, 4, 2, 128, 16, 0};
  int32_t one = 5;
  uint8_t m = 0;
  int32_t o[2], d;
  int64_t l[1] = {0};
  REQUIRE(fs_build_placement(&bad, &one, &m, nullptr, 0, o, &d, l) == FS_EINVAL);
  REQUIRE(fs_last_error()[0] != 0);
  REQUIRE(fs_kv_elem_offset(FS_KV_BF16, 0, 15, 127) == 2047 && fs_kv_elem_offset(FS_KV_BF16, 1, 16, 0) == -1);
  std::puts("host sanitizer run: ok");
  return 0;
}
