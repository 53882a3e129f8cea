// Host-side recovery planning after a GPU fault (integer only, never touches the GPU).
//
// Section 3.2 of the paper, "Lightning Recovery", as plans: which KVCache slices a surviving
// GPU keeps and which it reloads from the host copy (Proactive KVCache Backup), a placement
// that moves nothing but the lost slices (hybrid attention absorbing the lost worker, Fig. 5),
// and the deal of the lost FFN shards over the survivors (On-Demand Weight Recovery: the
// shard order along the reduction dimension is free).  GPU ids are physical ids.
#include <vector>

#include "fs_internal.h"

namespace {

fs_status check_alive(int32_t n_gpus, const uint8_t* alive, const char* who) {
  if (n_gpus < 1) return fs::fail(FS_EINVAL, "%s: n_gpus %d < 1", who, n_gpus);
  if (!alive) return fs::fail(FS_EINVAL, "%s: alive is NULL", who);
  for (int32_t g = 0; g < n_gpus; ++g)
    if (alive[g]) return FS_OK;
  return fs::fail(FS_EINVAL, "%s: no GPU survives", who);
}

}  // namespace

extern "C" fs_status fs_plan_kv_reload(int32_t n_req, int32_t n_kv_heads, const int32_t* ctx_len,
                                       const int32_t* old_owner, const int32_t* new_owner,
                                       int32_t n_gpus, const uint8_t* alive, int64_t* reload, int64_t* reuse) {
  if (fs_status st = check_alive(n_gpus, alive, "fs_plan_kv_reload")) return st;
  if (n_req < 0 || n_kv_heads < 1) return fs::fail(FS_EINVAL, "fs_plan_kv_reload: n_req %d, n_kv_heads %d", n_req, n_kv_heads);
  if (!reload || !reuse || (n_req > 0 && (!ctx_len || !old_owner || !new_owner)))
    return fs::fail(FS_EINVAL, "fs_plan_kv_reload: NULL pointer");
  for (int32_t g = 0; g < n_gpus; ++g) reload[g] = reuse[g] = 0;
  for (int32_t r = 0; r < n_req; ++r) {
    const int64_t L = ctx_len[r];
    if (L < 1) return fs::fail(FS_EINVAL, "fs_plan_kv_reload: ctx_len[%d] = %d < 1", r, ctx_len[r]);
    for (int32_t h = 0; h < n_kv_heads; ++h) {
      const int64_t i = static_cast<int64_t>(r) * n_kv_heads + h;
      const int32_t a = old_owner[i], b = new_owner[i];
      if (a < 0 || a >= n_gpus || b < 0 || b >= n_gpus || !alive[b])
        return fs::fail(FS_EINVAL, "fs_plan_kv_reload: slice (%d, %d) goes from GPU %d to GPU %d (outside [0, %d) or dead)",
                        r, h, a, b, n_gpus);
      (a == b ? reuse : reload)[b] += L;
    }
  }
  return FS_OK;
}

extern "C" fs_status fs_replace_failed_gpu(int32_t n_req, int32_t n_kv_heads, const int32_t* ctx_len,
                                           const int32_t* old_owner, const int32_t* old_dp_rank,
                                           int32_t n_gpus, const uint8_t* alive, int32_t* new_owner,
                                           int32_t* new_dp_rank, int64_t* dp_load) {
  if (fs_status st = check_alive(n_gpus, alive, "fs_replace_failed_gpu")) return st;
  if (n_req < 0 || n_kv_heads < 1)
    return fs::fail(FS_EINVAL, "fs_replace_failed_gpu: n_req %d, n_kv_heads %d", n_req, n_kv_heads);
  if (!dp_load || (n_req > 0 && (!ctx_len || !old_owner || !old_dp_rank || !new_owner || !new_dp_rank)))
    return fs::fail(FS_EINVAL, "fs_replace_failed_gpu: NULL pointer");
  for (int32_t r = 0; r < n_req; ++r) {
    const int64_t L = ctx_len[r];
    if (L < 1) return fs::fail(FS_EINVAL, "fs_replace_failed_gpu: ctx_len[%d] = %d < 1", r, ctx_len[r]);
    const int32_t* own = old_owner + static_cast<int64_t>(r) * n_kv_heads;
    int32_t* out = new_owner + static_cast<int64_t>(r) * n_kv_heads;
    int32_t n_lost = 0;
    for (int32_t h = 0; h < n_kv_heads; ++h) {
      if (own[h] < 0 || own[h] >= n_gpus)
        return fs::fail(FS_EINVAL, "fs_replace_failed_gpu: owner of (%d, %d) is %d, outside [0, %d)", r, h, own[h], n_gpus);
      out[h] = own[h];
      n_lost += !alive[own[h]];
    }
    int32_t d = old_dp_rank[r];
    if (d >= n_gpus) return fs::fail(FS_EINVAL, "fs_replace_failed_gpu: dp_rank[%d] = %d outside [0, %d)", r, d, n_gpus);
    new_dp_rank[r] = d;
    if (n_lost == 0) continue;
    if (d < 0 || !alive[d]) {            // no DP rank survives for this request: route it afresh
      d = -1;
      for (int32_t g = 0; g < n_gpus; ++g)
        if (alive[g] && (d < 0 || dp_load[g] < dp_load[d])) d = g;
      new_dp_rank[r] = d;
    }
    for (int32_t h = 0; h < n_kv_heads; ++h)
      if (!alive[own[h]]) out[h] = d;
    dp_load[d] += n_lost * L;
  }
  return FS_OK;
}

extern "C" fs_status fs_plan_ffn_reload(int32_t n_shards, const int32_t* shard_owner, int32_t n_gpus,
                                        const uint8_t* alive, int32_t* new_owner, int32_t* n_load) {
  if (fs_status st = check_alive(n_gpus, alive, "fs_plan_ffn_reload")) return st;
  if (n_shards < 0) return fs::fail(FS_EINVAL, "fs_plan_ffn_reload: n_shards %d < 0", n_shards);
  if (!n_load || (n_shards > 0 && (!shard_owner || !new_owner)))
    return fs::fail(FS_EINVAL, "fs_plan_ffn_reload: NULL pointer");
  std::vector<int32_t> held(n_gpus, 0);
  for (int32_t s = 0; s < n_shards; ++s) {
    if (shard_owner[s] < 0 || shard_owner[s] >= n_gpus)
      return fs::fail(FS_EINVAL, "fs_plan_ffn_reload: owner of shard %d is %d, outside [0, %d)", s, shard_owner[s], n_gpus);
    ++held[shard_owner[s]];
  }
  for (int32_t g = 0; g < n_gpus; ++g) n_load[g] = 0;
  for (int32_t s = 0; s < n_shards; ++s) {
    new_owner[s] = shard_owner[s];
    if (alive[shard_owner[s]]) continue;
    int32_t k = -1;
    for (int32_t g = 0; g < n_gpus; ++g)
      if (alive[g] && (k < 0 || held[g] < held[k])) k = g;   // fewest shards, lowest id among equals
    new_owner[s] = k;
    ++held[k];
    ++n_load[k];
  }
  return FS_OK;
}
