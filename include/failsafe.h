/*
 * failsafe.h - C ABI of the cyclic/hybrid decode-attention share for MI355X (gfx950).
 *
 * One GPU's share of one batched decode-attention step over a paged KVCache when
 * the KV heads of a model are spread over R surviving tensor-parallel ranks:
 *
 *   fs_build_placement   which rank owns each (request, KV head)        host
 *   (fs_build_placement_hybrid_heads: the paper's head-level variant)   host
 *   fs_build_worklist    one rank's ragged (request, head, chunk) list  host
 *   (fs_choose_chunk_tokens: a chunk size where the caller leaves it open) host
 *   fs_decode_attention  per-item partial attention (out, lse)          device
 *   fs_merge_lse         split-K partials -> final (out, lse)           device
 *   (fs_decode_attention_fused: the last two in one call, unsplit pairs unmerged) device
 *
 * and, before the decode step, the host side of the paper's router and prefill
 * scheduler: fs_route_request(s), fs_schedule_prefill; after a fault, the recovery
 * plans: fs_plan_kv_reload, fs_replace_failed_gpu, fs_plan_ffn_reload; and the
 * attention of the prefill batches: fs_build_prefill_worklist, fs_prefill_attention.
 *
 * The placement rules are those of the paper's Section 3.1 ("Memory and
 * Computation Balancer": Cyclic Placement, Hybrid Attention, Load-Aware DP-Rank
 * Routing); attention is the decode phase of Section 2.1.1 over KVCache blocks.
 *
 * General rules
 *  - Plain C types only.  Every pointer is marked HOST or DEVICE below.
 *  - The caller owns every buffer.  The library allocates nothing that outlives
 *    a call and frees nothing of the caller's.
 *  - Host builders never touch the GPU and are pure functions of their inputs.
 *  - Device calls enqueue work on `stream` (a hipStream_t passed as void*, NULL
 *    = the null stream) and return without synchronising.
 *  - Every call returns an fs_status; nothing throws or aborts.  After a
 *    non-OK status fs_last_error() gives a message (thread-local).
 */
#ifndef FAILSAFE_H
#define FAILSAFE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_ABI_VERSION 4

#if defined(__GNUC__)
#define FS_API __attribute__((visibility("default")))
#else
#define FS_API
#endif

typedef enum {
  FS_OK = 0,
  FS_EINVAL = -1,       /* an argument is out of range or inconsistent            */
  FS_ECAPACITY = -2,    /* an output array is too small; needed counts returned   */
  FS_EHIP = -3,         /* a HIP runtime call failed                              */
  FS_EUNSUPPORTED = -4  /* valid in principle, not built (e.g. head_dim != 128)   */
} fs_status;

enum { FS_MODE_TP = 0, FS_MODE_DP = 1 };          /* per request                  */
enum { FS_KV_BF16 = 0, FS_KV_FP8_E4M3 = 1 };      /* storage type of K and V      */
/* What the caller states about the V values a call can read (fs_kv_view.v_range; used by
 * fs_prefill_attention, ignored by the decode calls):
 *   FS_V_ANY         nothing: any finite value.  V stays bf16 in the P.V product (fp8: its codes,
 *                    which are bf16 values, the slot's scale going to the weights) and the softmax
 *                    weights enter as a sum of two bf16 terms.
 *   FS_V_FP16_RANGE  every V value (fp8: code times the slot's scale) is 0 or has a magnitude in
 *                    [2^-14, 65504], i.e. a bf16 value converts to fp16 exactly (an fp8 one is rounded
 *                    toward zero to fp16's 11 bits).  The product then runs on fp16 weights and fp16 V
 *                    (~20% faster).  A value that breaks the statement is not detected: a larger
 *                    magnitude counts as 65504, a smaller one is rounded toward zero on fp16's
 *                    subnormal grid. */
enum { FS_V_ANY = 0, FS_V_FP16_RANGE = 1 };

/* Shape of one decode batch. */
typedef struct {
  int32_t n_req;        /* B   requests in the batch, >= 0                        */
  int32_t n_q_heads;    /* H_q query heads, a multiple of n_kv_heads              */
  int32_t n_kv_heads;   /* H_kv                                                   */
  int32_t head_dim;     /* d, 128 is the only size built                          */
  int32_t page_tokens;  /* tokens per KVCache block, 16 is the only size built    */
  int32_t n_ranks;      /* R   surviving tensor-parallel ranks, >= 1              */
} fs_shape;

/* One unit of kernel work: tokens [tok_begin, tok_end) of one (request, KV head).
 * 32 bytes; arrays of these are compared bit for bit against the oracle. */
typedef struct {
  int32_t req;          /* request index                                          */
  int32_t kv_head;      /* KV head index                                          */
  int32_t tok_begin;    /* first token, a multiple of page_tokens                 */
  int32_t tok_end;      /* one past the last token, <= ctx_len[req]               */
  int32_t pair;         /* index of the (request, head) pair in this rank's list  */
  int32_t chunk;        /* index of this chunk within its pair                    */
  int32_t q_row;        /* first query row: req*H_q + kv_head*G  (G = H_q/H_kv)   */
  int32_t part_row;     /* first partial-output row: item_index*G                 */
} fs_work_item;

typedef struct {
  int32_t req, kv_head, ctx_len, n_chunks;
} fs_pair;

/* ---------------------------------------------------------------------------
 * fs_build_placement - Section 3.1, Cyclic Placement + Hybrid Attention +
 * Load-Aware DP-Rank Routing, at request granularity.
 *
 * Requests are taken in index order (arrival order).  A tensor-parallel
 * request r puts KV head h on rank (h + rot[r] + layer) mod R (mathematical
 * mod, rot may be negative) and adds ctx_len[r] to that rank's load per head.
 * rot == NULL means rot[r] = r.  The paper's layer-by-layer rotation is
 * rot[r] = 0 with layer = the layer index.  A data-parallel request puts all
 * H_kv heads on the rank whose running load is smallest (lowest rank among
 * equals) and adds H_kv*ctx_len[r] there.  Load is counted in KV tokens x KV
 * heads and includes everything placed so far, tensor-parallel shares too.
 *
 *  ctx_len   HOST in   [n_req]            cached tokens per request, each >= 1
 *  mode      HOST in   [n_req]            FS_MODE_TP or FS_MODE_DP
 *  rot       HOST in   [n_req] or NULL
 *  owner     HOST out  [n_req*n_kv_heads] owning rank of (r, h) at r*H_kv + h
 *  dp_rank   HOST out  [n_req]            the rank of a DP request, -1 for TP
 *  rank_load HOST in/out [n_ranks]        running load; zero it for a fresh batch
 *
 * FS_EINVAL: NULL pointer, n_ranks < 1, n_kv_heads < 1, n_req < 0,
 * ctx_len < 1, mode not 0/1.  On error the outputs are unspecified.
 */
FS_API fs_status fs_build_placement(const fs_shape* shape, const int32_t* ctx_len, const uint8_t* mode,
                             const int32_t* rot, int32_t layer,
                             int32_t* owner, int32_t* dp_rank, int64_t* rank_load);

/* ---------------------------------------------------------------------------
 * fs_build_placement_hybrid_heads - Section 3.1, Hybrid Attention exactly as the
 * paper states it (Fig. 3), at head granularity, with Cyclic Placement's
 * layer-by-layer rotation.
 *
 * Every tensor-parallel worker gets floor(H_kv/R) heads: heads [0, R*floor(H_kv/R))
 * of every request go to rank (h + layer) mod R.  The remaining H_kv mod R heads
 * are replicated and run data-parallel: all of a request's leftover heads go to
 * the request's DP rank, which is route[r] when route is given, else the rank
 * with the least pending DP work in token units (Load-Aware DP-Rank Routing:
 * dp_load only, ties to the lowest rank, requests in index order).  When R divides
 * H_kv nothing is left over and this is uniform TP (dp_rank = -1).
 *
 *  ctx_len   HOST in   [n_req]            each >= 1
 *  route     HOST in   [n_req] or NULL    DP rank per request, each in [0, R)
 *  owner     HOST out  [n_req*n_kv_heads]
 *  dp_rank   HOST out  [n_req]
 *  rank_load HOST in/out [n_ranks]        total load, KV tokens x KV heads
 *  dp_load   HOST in/out [n_ranks]        the DP part of it (what the router balances)
 *
 * The result feeds fs_build_worklist unchanged.  FS_EINVAL: NULL pointer, bad
 * shape, ctx_len < 1, route outside [0, R).
 */
FS_API fs_status fs_build_placement_hybrid_heads(const fs_shape* shape, const int32_t* ctx_len,
                                                 int32_t layer, const int32_t* route,
                                                 int32_t* owner, int32_t* dp_rank,
                                                 int64_t* rank_load, int64_t* dp_load);

/* ---------------------------------------------------------------------------
 * fs_build_worklist - the ragged per-(request, head) list that hybrid attention
 * (Section 3.1) leaves on one rank, cut into split-K chunks.
 *
 * Pairs (r, h) with owner == rank are numbered in ascending (r, h).  Pair p is
 * cut into ceil(ctx_len/chunk_tokens) items of chunk_tokens tokens (the last
 * may be shorter); chunk_tokens == 0 means one item per pair.  Items of a pair
 * are consecutive; chunk_indptr[p] is the first item of pair p.  sched lists
 * item indices by decreasing token count, equal counts by increasing index
 * (longest first, so the short ones fill the tail of the launch).
 *
 *  owner        HOST in  [n_req*n_kv_heads]
 *  chunk_tokens 0 or a positive multiple of page_tokens
 *  items        HOST out [items_cap]
 *  pairs        HOST out [pairs_cap]
 *  sched        HOST out [items_cap]
 *  chunk_indptr HOST out [pairs_cap+1]
 *               All four NULL (capacities 0): count only.  Otherwise all are filled; an
 *               array with capacity 0 may be NULL (a rank that owns nothing), except
 *               chunk_indptr, which always has at least one entry.
 *  n_items, n_pairs  HOST out  always written when the shape is valid
 *
 * FS_ECAPACITY: a non-NULL array is too small; nothing but the counts is valid.
 * FS_EINVAL: bad shape, rank outside [0, R), bad chunk_tokens, owner outside
 * [0, R), ctx_len < 1, counts beyond int32 rows.
 */
FS_API fs_status fs_build_worklist(const fs_shape* shape, const int32_t* ctx_len, const int32_t* owner,
                            int32_t rank, int32_t chunk_tokens,
                            fs_work_item* items, int64_t items_cap,
                            fs_pair* pairs, int64_t pairs_cap,
                            int32_t* sched, int64_t* chunk_indptr,
                            int64_t* n_items, int64_t* n_pairs);

/* ---------------------------------------------------------------------------
 * fs_build_worklist_units - the same ragged share (Section 3.1) cut for a launch without
 * stragglers.  The rank's pairs, in ascending (r, h), are laid end to end as one stream of
 * KVCache pages and the stream is cut into n_units runs of equal length (to within one page), one
 * per resident workgroup of fs_decode_attention_units: with P pages in all and U = min(n_units, P)
 * units, unit u holds stream pages [floor(u*P/U), floor((u+1)*P/U)).  Where a run crosses from
 * one pair into the next it is cut there too, so an item is still tokens [tok_begin, tok_end) of
 * one pair, a pair inside one run is a single item, and the list has at most n_pairs + U - 1 items.
 * Items are numbered in stream order: the items of a unit are consecutive (unit_indptr[u] is the
 * first of unit u) and so are the items of a pair (chunk_indptr[p]); fs_work_item.chunk is the
 * item's index within its pair and fs_pair.n_chunks the pair's item count.
 *
 *  items        HOST out [items_cap]
 *  pairs        HOST out [pairs_cap]
 *  unit_indptr  HOST out [units_cap+1]
 *  chunk_indptr HOST out [pairs_cap+1]
 *               All four NULL (capacities 0): count only.
 *  n_items, n_pairs, n_units_out  HOST out  always written when the arguments are valid (n_units_out = U)
 *
 * FS_ECAPACITY: an array is too small; nothing but the counts is valid.  FS_EINVAL: bad shape,
 * rank outside [0, R), n_units < 1, owner outside [0, R), ctx_len < 1, counts beyond int32 rows.
 */
FS_API fs_status fs_build_worklist_units(const fs_shape* shape, const int32_t* ctx_len, const int32_t* owner,
                                         int32_t rank, int32_t n_units,
                                         fs_work_item* items, int64_t items_cap,
                                         fs_pair* pairs, int64_t pairs_cap,
                                         int64_t* unit_indptr, int64_t units_cap, int64_t* chunk_indptr,
                                         int64_t* n_items, int64_t* n_pairs, int64_t* n_units_out);

/* ---------------------------------------------------------------------------
 * fs_choose_chunk_tokens - a split-K chunk size for one rank's share.  The ragged share of
 * Section 3.1 can be a handful of very long contexts (the skew the paper's load-aware routing is
 * there for), and a launch runs as long as its longest item.  The chunk is four thirds of a slot's fair
 * share of the whole: with T the cached tokens of rank's (request, KV head) pairs, all told,
 * ceil(4 T / (3 n_slots)), rounded up to whole pages and held within [min_chunk, max_chunk].
 *
 *  ctx_len, owner   HOST in   as for fs_build_worklist
 *  max_chunk, min_chunk       multiples of page_tokens, page_tokens <= min_chunk <= max_chunk
 *  n_slots          what the whole is shared among, >= 1.  Measured best for the decode sweep: the number of
 *                   compute units with max_chunk 2048 for a share of less than ~2 M token-heads; for a larger
 *                   one, with max_chunk 32768, 16/3 per compute unit when resident workgroups claim the launch
 *                   records (items of half of what one of a compute unit's two workgroups gets) and 3 per
 *                   compute unit with one workgroup per record (8/9 of it)
 *  chunk_tokens     HOST out  the chosen chunk
 *  n_items          HOST out  the list's length with it
 *
 * FS_EINVAL: bad shape, rank, chunk bounds, n_slots < 1, owner outside [0, R), ctx_len < 1.
 */
FS_API fs_status fs_choose_chunk_tokens(const fs_shape* shape, const int32_t* ctx_len, const int32_t* owner,
                                        int32_t rank, int32_t max_chunk, int32_t min_chunk, int64_t n_slots,
                                        int32_t* chunk_tokens, int64_t* n_items);

/* ---------------------------------------------------------------------------
 * fs_route_request - Section 3.1, Load-Aware DP-Rank Routing: the incoming request
 * goes to the rank whose pending DP work (token units) is smallest, the lowest rank
 * among equals; `work` is added to that rank's pending work.
 *
 *  pending  HOST in/out [n_ranks]   pending work per rank
 *  work     the request's work in token units, >= 0
 *  rank     HOST out                the chosen rank
 *
 * FS_EINVAL: NULL pointer, n_ranks < 1, work < 0.
 */
FS_API fs_status fs_route_request(int32_t n_ranks, int64_t* pending, int64_t work, int32_t* rank);

/* fs_route_requests - the same rule (Section 3.1, Load-Aware DP-Rank Routing) for a queue of
 * requests in arrival order, one call: request i goes to the rank with the least pending work
 * after requests 0..i-1 were placed (lowest rank among equals), exactly as n calls of
 * fs_route_request would place them.
 *
 *  pending  HOST in/out [n_ranks]   pending work per rank
 *  work     HOST in     [n]         work of each request in token units, >= 0
 *  rank     HOST out    [n]         the chosen ranks
 *
 * FS_EINVAL: NULL pointer (with n > 0), n_ranks < 1, n < 0, a negative work (nothing is changed).
 */
FS_API fs_status fs_route_requests(int32_t n_ranks, int64_t* pending, const int64_t* work, int32_t n, int32_t* rank);

/* One waiting request of the prefill queue: n_new tokens wait behind n_done tokens
 * that are already processed; rank is the request's DP rank. */
typedef struct {
  int32_t req, rank, n_done, n_new;
} fs_prefill_entry;

/* ---------------------------------------------------------------------------
 * fs_schedule_prefill - Section 3.1, Algorithm 1 (DP-aware Adaptive Chunked
 * Prefill): form the next prefill batch under a global token budget.
 *
 * S_r, the schedulable tokens of rank r, is the concatenation in array order of
 * the waiting tokens of the entries with that rank.  While the batch holds fewer
 * than `budget` tokens and some S_r is not empty: take the first token of S_r for
 * the least-loaded such r (lowest rank among equals), add the token's cost to
 * that rank's load, and remember the batch so far as a candidate.  Return the
 * best candidate.  Fixed here where the paper is open:
 *   cost of a token = tokens of its request before it + 1 (the keys it attends
 *     to); a chunk of N tokens after L processed ones then costs
 *     N*L + N*(N+1)/2, the paper's O(N^2 + N*L + N);
 *   best candidate = among the candidates of at least min(min_tokens, all taken)
 *     tokens, the one with the smallest (largest load)/(mean load); the larger
 *     batch among equals;
 *   loads start at init_load[r], or at 0 when init_load is NULL (the printed
 *     initialisation; the algorithm lists per-rank workloads as an input).
 *
 *  entries   HOST in  [n_entries]
 *  init_load HOST in  [n_ranks] or NULL   each >= 0
 *  take      HOST out [n_entries]  leading waiting tokens of each entry in the batch
 *  load      HOST out [n_ranks]    rank loads of the chosen batch (init_load included)
 *  n_tokens  HOST out              tokens in the chosen batch (0 when nothing waits or budget is 0)
 *
 * FS_EINVAL: NULL pointer, n_ranks < 1, negative budget/min_tokens/n_entries,
 * entry with rank outside [0, n_ranks) or negative counts, a negative init_load.
 */
FS_API fs_status fs_schedule_prefill(int32_t n_ranks, int32_t budget, int32_t min_tokens,
                                     const fs_prefill_entry* entries, int32_t n_entries,
                                     const int64_t* init_load, int32_t* take, int64_t* load,
                                     int32_t* n_tokens);

/* ---------------------------------------------------------------------------
 * Recovery planning after a GPU fault - Section 3.2, "Lightning Recovery", as
 * plans (what moves where); the transfers themselves are not part of this library.
 * GPU ids are physical ids in [0, n_gpus); alive[g] != 0 marks the GPUs that live
 * (HOST in [n_gpus], at least one), so a later fault is planned with the earlier
 * dead GPUs still marked dead.
 *
 * fs_plan_kv_reload - Proactive KVCache Backup: a surviving GPU keeps the KVCache
 * it holds and reloads from the host copy only what it newly needs.  For one layer
 * and any two placements: slice (r, h) is reused when new_owner == old_owner and
 * reloaded by new_owner otherwise.
 *
 *  ctx_len    HOST in  [n_req]             each >= 1
 *  old_owner  HOST in  [n_req*n_kv_heads]  GPU holding (r, h) before the fault
 *  new_owner  HOST in  [n_req*n_kv_heads]  GPU holding it afterwards, a live one
 *  reload     HOST out [n_gpus]            KV tokens x KV heads each GPU reads from the host copy
 *  reuse      HOST out [n_gpus]            KV tokens x KV heads each GPU keeps in place
 *
 * fs_replace_failed_gpu - the placement that moves nothing but the lost slices,
 * the way hybrid attention (Section 3.1; Fig. 5) absorbs a lost worker: slices on
 * surviving GPUs stay; the lost slices of request r become data-parallel work on
 * r's DP rank; a request whose DP rank is -1 or dead is routed to the
 * live GPU with the least dp_load (lowest id among equals), in request
 * order; dp_load grows by (lost heads)*ctx_len[r].  Meant for the case where the
 * tensor-parallel share per worker stays, floor(H/(R-1)) == floor(H/R); otherwise
 * build a fresh placement and diff it with fs_plan_kv_reload.
 *
 *  old_dp_rank HOST in  [n_req]            -1 for a request without one
 *  new_owner   HOST out [n_req*n_kv_heads]
 *  new_dp_rank HOST out [n_req]
 *  dp_load     HOST in/out [n_gpus]        pending DP work per GPU (entries of dead GPUs are ignored)
 *
 * fs_plan_ffn_reload - On-Demand Weight Recovery: FFN shards (slices along the
 * intermediate dimension, whose order is free) stay where they are; each lost
 * shard, in ascending index, goes to the live GPU that holds the fewest
 * shards (lowest id among equals).
 *
 *  shard_owner HOST in  [n_shards]
 *  new_owner   HOST out [n_shards]
 *  n_load      HOST out [n_gpus]           shards each GPU reads from the host
 *
 * All three: FS_EINVAL for NULL pointers, n_gpus < 1, no live GPU, an owner
 * outside [0, n_gpus), ctx_len < 1, a new owner that is dead.
 */
FS_API fs_status fs_plan_kv_reload(int32_t n_req, int32_t n_kv_heads, const int32_t* ctx_len,
                                   const int32_t* old_owner, const int32_t* new_owner,
                                   int32_t n_gpus, const uint8_t* alive, int64_t* reload, int64_t* reuse);
FS_API fs_status fs_replace_failed_gpu(int32_t n_req, int32_t n_kv_heads, const int32_t* ctx_len,
                                       const int32_t* old_owner, const int32_t* old_dp_rank,
                                       int32_t n_gpus, const uint8_t* alive, int32_t* new_owner,
                                       int32_t* new_dp_rank, int64_t* dp_load);
FS_API fs_status fs_plan_ffn_reload(int32_t n_shards, const int32_t* shard_owner, int32_t n_gpus,
                                    const uint8_t* alive, int32_t* new_owner, int32_t* n_load);

/* ---------------------------------------------------------------------------
 * The paged KVCache as the kernels read it.
 *
 * A slot is one KVCache block of one KV head: page_tokens x head_dim elements
 * of K and as many of V.  Slot s of K starts at k_pool + s*k_slot_stride bytes
 * (likewise V), so K and V may live in two pools or interleaved in one.  Slot
 * starts must be 16-byte aligned.  page_ids[page_indptr[p] + i] is the slot of
 * page i of this rank's pair p.
 *
 * Element order inside a slot is chosen for the gfx950 matrix cores so that a
 * wavefront's 16-byte loads are contiguous 1 KiB runs AND land directly in MFMA
 * operand registers; fs_kv_elem_offset() is the definition:
 *
 *  bf16 K (16 tok x 128):  [d/32][(d%32)/8][tok][d%8]
 *  bf16 V (16 tok x 128):  [d/32][tok/4][d%16][(d/16)%2][tok%4]
 *  fp8  K and V         :  [d/64][(d%64)/16][tok][d%16]   (a 16-byte piece per (token, 16 d))
 *
 * fp8 is OCP e4m3 (finite-only, max 448); element value = code * scale[slot]
 * with one fp32 scale per slot for K and one for V.
 */
typedef struct {
  const void* q;               /* DEVICE [n_req][n_q_heads][head_dim] bf16        */
  const void* k_pool;          /* DEVICE                                          */
  const void* v_pool;          /* DEVICE                                          */
  int64_t k_slot_stride;       /* bytes between consecutive K slots               */
  int64_t v_slot_stride;       /* bytes between consecutive V slots               */
  const float* k_scale;        /* DEVICE [n_slots], fp8 only, else NULL           */
  const float* v_scale;        /* DEVICE [n_slots], fp8 only, else NULL           */
  const int64_t* page_indptr;  /* DEVICE [n_pairs+1]                              */
  const int32_t* page_ids;     /* DEVICE [page_indptr[n_pairs]]                   */
  int32_t kv_dtype;            /* FS_KV_BF16 or FS_KV_FP8_E4M3                    */
  float sm_scale;              /* softmax scale, 1/sqrt(head_dim) in the paper's models */
  const float* page_scales;    /* DEVICE [page_indptr[n_pairs]][2] or NULL: fp8 only, the same scales in
                                  page-table order, entry j = (K scale, V scale) of slot page_ids[j].  When
                                  given, the kernels read these (a contiguous run along an item,
                                  0.2% of the K/V bytes) and k_scale/v_scale may be NULL; the by-slot
                                  arrays cost one memory line per slot and scale, ~4% of the bytes.      */
  int32_t v_range;             /* FS_V_ANY (0) or FS_V_FP16_RANGE: see the enum                           */
} fs_kv_view;

/* Element offset (in elements) of (tok, d) inside a slot; is_v selects the V
 * order.  Returns -1 for arguments out of range or an unknown kv_dtype. */
FS_API int32_t fs_kv_elem_offset(int32_t kv_dtype, int32_t is_v, int32_t tok, int32_t d);

/* fs_pack_kv_slots - KVCache blocks (Section 2.1.1) from token-major order [tok][d] into the element order
 * above, on the device: slot s is read at src_dev + s*src_slot_stride and written at dst_dev +
 * s*dst_slot_stride (so the destination may be the K or the V half of an interleaved pool).  The stand-in
 * for an engine's KV-append step, which would write the kernels' order directly.
 *
 *  src_dev  DEVICE in   n_slots slots of 16 x 128 elements, token-major
 *  dst_dev  DEVICE out  the same slots in kernel order; the two pools must not overlap
 *  is_v     0: the K order, else the V order
 *
 * n_slots == 0 is a no-op.  FS_EINVAL: NULL or misaligned (16 bytes) pointers or strides, a stride below one
 * slot, overlapping pools, unknown kv_dtype.  FS_EHIP: launch failure. */
FS_API fs_status fs_pack_kv_slots(const void* src_dev, int64_t src_slot_stride, void* dst_dev, int64_t dst_slot_stride,
                                  int64_t n_slots, int32_t kv_dtype, int32_t is_v, void* stream);

/* ---------------------------------------------------------------------------
 * fs_decode_attention - decode-phase attention (Section 2.1.1) for every item
 * of the list, one launch.  For item i and g in [0, G), with q = query row
 * q_row+g and t over the item's tokens:
 *     s_t = sm_scale * <q, K_t>
 *     part_lse[part_row+g] = ln sum_t exp(s_t)
 *     part_o[part_row+g][:] = sum_t exp(s_t - lse) * V_t
 * Scores, softmax and accumulation are fp32; the softmax weights enter the
 * P.V product as a sum of two bf16 terms (16 significant bits).  Tokens at or beyond tok_end are never used,
 * whatever their bits.
 *
 *  items_dev  DEVICE in  [n_items]     as built by fs_build_worklist
 *  sched_dev  DEVICE in  [n_items]     launch order, or NULL for index order
 *  part_o     DEVICE out [n_items*G][head_dim] fp32
 *  part_lse   DEVICE out [n_items*G]   fp32
 *
 * n_items == 0 is a no-op.  FS_EINVAL: NULL pointers, bad shape, G > 16,
 * misaligned pools/strides.  FS_EUNSUPPORTED: head_dim != 128, page_tokens !=
 * 16.  FS_EHIP: launch failure.  Item contents are trusted
 * (they are device memory); build them with fs_build_worklist.
 */
FS_API fs_status fs_decode_attention(const fs_shape* shape, const fs_kv_view* kv,
                              const fs_work_item* items_dev, const int32_t* sched_dev,
                              int64_t n_items, float* part_o, float* part_lse, void* stream);

/* ---------------------------------------------------------------------------
 * fs_decode_attention_persistent - the same computation as fs_decode_attention,
 * by a fixed set of workgroups (two per CU) that claim items from a counter
 * in list order and write their partial rows in bursts (decode phase, Section 2.1.1;
 * the ragged list of Section 3.1).  An item's pages are split over four wavefronts as
 * in fs_decode_attention's default launch shape ("waves_per_group" = 4), so the two
 * give the same bits there; with another "waves_per_group" the plain call sums in
 * another order and agrees only within rounding.
 *
 *  claim_dev  DEVICE in/out  two int32 (8-byte aligned): the item counter and the count
 *             of workgroups that have left.  Both must be 0 before the first launch that
 *             uses them; every launch leaves them at 0 again, so launches that follow
 *             one another on a stream (or replays of a captured graph) share one pair
 *             without clearing it.  Two launches that overlap in time need two pairs.
 *
 * Everything else as for fs_decode_attention (bf16 or fp8 K/V).
 */
FS_API fs_status fs_decode_attention_persistent(const fs_shape* shape, const fs_kv_view* kv,
                                                const fs_work_item* items_dev, const int32_t* sched_dev,
                                                int64_t n_items, int32_t* claim_dev, float* part_o,
                                                float* part_lse, void* stream);

/* ---------------------------------------------------------------------------
 * fs_decode_attention_fused - the decode attention of the whole list (Section 2.1.1) and the
 * split-K merge of its partials in one call: what fs_decode_attention (or
 * fs_decode_attention_persistent) followed by fs_merge_lse leave in out/lse, bit for bit, for
 * the ragged list of Section 3.1.  A pair that is a single item (chunk_indptr[p+1] -
 * chunk_indptr[p] == 1) gets its final rows [p*G, p*G+G) straight from the sweep and writes no
 * partial rows; the merge runs only for the pairs that are split, and is not launched at all when
 * n_items == n_pairs.
 *
 *  chunk_indptr_dev  DEVICE in   [n_pairs+1]  as built by fs_build_worklist
 *  part_o, part_lse  DEVICE scratch, sized and indexed as for fs_decode_attention (rows of
 *                    unsplit pairs stay untouched); may be NULL when n_items == n_pairs
 *  claim_dev         DEVICE in/out, as for fs_decode_attention_persistent, or NULL.  With bf16
 *                    K/V, a non-NULL claim_dev and at least 1024 items the persistent sweep runs,
 *                    otherwise one workgroup per item
 *  out, lse          DEVICE out  [n_pairs*G][head_dim], [n_pairs*G] fp32
 *
 * n_items == 0 is a no-op.  Errors as for fs_decode_attention, and FS_EINVAL for n_pairs
 * outside [1, n_items] or a NULL chunk_indptr_dev, out or lse.
 */
FS_API fs_status fs_decode_attention_fused(const fs_shape* shape, const fs_kv_view* kv,
                                           const fs_work_item* items_dev, const int32_t* sched_dev,
                                           int64_t n_items, const int64_t* chunk_indptr_dev, int64_t n_pairs,
                                           float* part_o, float* part_lse, int32_t* claim_dev,
                                           float* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------
 * fs_decode_attention_units - decode attention (Section 2.1.1) and split-K merge of a list that
 * fs_build_worklist_units has cut into equal runs: one resident workgroup per unit
 * walks its unit's items in order (no counter, nothing handed out at run time: every workgroup
 * streams the same number of pages), a pair that is one item gets its final rows from the sweep,
 * the others are merged as by fs_merge_lse.  out/lse hold, to rounding (another order of sums
 * wherever the cuts differ), what fs_decode_attention + fs_merge_lse give for the same pairs.
 * Choose n_units as the number of workgroups the GPU holds at once (two per compute unit).
 *
 *  items_dev         DEVICE in   [n_items]     as built by fs_build_worklist_units
 *  unit_indptr_dev   DEVICE in   [n_units+1]
 *  chunk_indptr_dev  DEVICE in   [n_pairs+1], or NULL: the sweep alone - every item's rows go to
 *                    part_o/part_lse as in fs_decode_attention, nothing is merged, n_pairs, out
 *                    and lse are ignored (fs_merge_lse can follow)
 *  part_o, part_lse  DEVICE scratch [n_items*G][head_dim], [n_items*G]; may be NULL when n_items == n_pairs
 *  out, lse          DEVICE out  [n_pairs*G][head_dim], [n_pairs*G] fp32
 *
 * n_items == 0 is a no-op.  Errors as for fs_decode_attention_fused (bf16 or fp8 K/V).
 * List contents are trusted (device memory): no unit may be empty.
 */
FS_API fs_status fs_decode_attention_units(const fs_shape* shape, const fs_kv_view* kv,
                                           const fs_work_item* items_dev, int64_t n_items,
                                           const int64_t* unit_indptr_dev, int64_t n_units,
                                           const int64_t* chunk_indptr_dev, int64_t n_pairs,
                                           float* part_o, float* part_lse, float* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------
 * Launch records - a work list written out the way a kernel wants to find it.  A kernel that is
 * handed items looks each one up itself: the list entry, the item, the pair's offset in the page
 * table and its chunk count, then the page ids - four dependent reads before the first page of
 * K/V can be asked for, at the start of every workgroup.  A record holds all of that for one item,
 * resolved on the host, with the slots of the item's first eight pages: one 64-byte read.
 * (The ragged list is Section 3.1's; the record is this library's device.) */
typedef struct {
  int64_t first_page;      /* index into page_ids of the item's first page:
                              page_indptr[pair] + tok_begin / page_tokens                    */
  int32_t n_tok;           /* tok_end - tok_begin                                            */
  int32_t q_row;           /* first query row, as in the item                                */
  int32_t row;             /* first partial row (part_row); or, for an item that is all of
                              its pair, -(pair*G) - 1: its rows are the pair's final rows    */
  int32_t n_chunks;        /* chunks (items) of the item's pair                              */
  int32_t first_slots[8];  /* page_ids[first_page + j], j = 0..7 (0 beyond the last page)    */
  int32_t pair;            /* the item's pair                                                */
  int32_t pair_row;        /* first partial row of the pair's first chunk:
                              chunk_indptr[pair] * G (chunk c's rows start G*c further on)   */
} fs_launch_record;        /* 64 bytes; arrays of these are compared bit for bit             */

/* fs_build_launch_records - record k describes item order[k] (order == NULL: item k).
 *
 *  items        HOST in  [n_items]    from fs_build_worklist or fs_build_worklist_units
 *  order        HOST in  [n_items] or NULL   launch order (fs_build_worklist's sched)
 *  chunk_indptr HOST in  [n_pairs+1]
 *  page_indptr  HOST in  [n_pairs+1]  the page table the kernels will be given, host copy
 *  page_ids     HOST in  [n_page_ids]
 *  direct_rows  nonzero: an item that is all of its pair gets row = -(pair*G) - 1 (what
 *               fs_decode_attention_records expects); 0: every row is the item's part_row
 *  records      HOST out [n_items]
 *
 * FS_EINVAL: NULL pointer, negative counts, an order entry or a pair outside its range, an item
 * whose pages do not lie inside its pair's part of the page table, or whose part_row is not
 * (chunk_indptr[pair] + chunk) * G (the rows the merge reads). */
FS_API fs_status fs_build_launch_records(const fs_shape* shape, const fs_work_item* items, const int32_t* order,
                                         int64_t n_items, const int64_t* chunk_indptr, int64_t n_pairs,
                                         const int64_t* page_indptr, const int32_t* page_ids, int64_t n_page_ids,
                                         int32_t direct_rows, fs_launch_record* records);

/* fs_decode_attention_records - decode attention (Section 2.1.1) and split-K merge in one call,
 * from launch records built with direct_rows != 0.  unit_indptr_dev == NULL: one workgroup per
 * record, in the order of the array, or with claim_dev resident workgroups that claim the records
 * in that order (bf16 or fp8 K/V).  unit_indptr_dev given: records of a list
 * from fs_build_worklist_units in item order, one resident workgroup per unit, as
 * fs_decode_attention_units.  Rows of unsplit pairs come final from the sweep; the merge runs for
 * split pairs and is not launched when n_items == n_pairs.  out/lse hold what the calls that take
 * items leave for the same list, bit for bit.
 *
 *  records_dev       DEVICE in   [n_items]
 *  unit_indptr_dev   DEVICE in   [n_units+1] or NULL
 *  chunk_indptr_dev  DEVICE in   [n_pairs+1]  (read by the merge only), or NULL: the sweep alone - no merge is
 *                    launched, n_pairs is ignored and every row goes where its record says (records built
 *                    with direct_rows == 0 send all of them to part_o/part_lse)
 *  part_o, part_lse  DEVICE scratch [n_items*G][head_dim], [n_items*G]; may be NULL when n_items == n_pairs
 *  out, lse          DEVICE out
 *  pair_counters_dev DEVICE scratch [n_pairs] int32, or NULL.  Given (with chunk_indptr_dev): split pairs are
 *                    merged inside the sweep and no merge kernel is launched - every workgroup that has
 *                    written partial rows of a split pair counts itself in on the pair's counter, and the one
 *                    that completes the count merges the pair's chunks into its final rows (nobody waits).
 *                    The counters must all be zero when the call is made; every call leaves them zero
 *                    (a launch that did not run to its end may not).  Calls that share counters must not
 *                    overlap.  Same bits in out/lse as with NULL.
 *  claim_dev         DEVICE scratch, two int32, 8-byte aligned, or NULL.  Given (unit_indptr_dev NULL): two
 *                    resident workgroups per compute unit claim the records in the order of the array and
 *                    write their rows in bursts, as fs_decode_attention_persistent does with items; whatever
 *                    the length of the list (the caller chooses the form).  Both counters must be zero when
 *                    the call is made and every call leaves them zero; calls that share them must not
 *                    overlap.  Same bits in out/lse as with NULL.
 *
 * The page table of kv must be the one the records were built from.  Errors as for
 * fs_decode_attention_fused; FS_EINVAL also for pair_counters_dev without chunk_indptr_dev and for
 * claim_dev together with unit_indptr_dev or not 8-byte aligned. */
FS_API fs_status fs_decode_attention_records(const fs_shape* shape, const fs_kv_view* kv,
                                             const fs_launch_record* records_dev, int64_t n_items,
                                             const int64_t* unit_indptr_dev, int64_t n_units,
                                             const int64_t* chunk_indptr_dev, int64_t n_pairs,
                                             float* part_o, float* part_lse, float* out, float* lse,
                                             int32_t* pair_counters_dev, int32_t* claim_dev, void* stream);

/* ---------------------------------------------------------------------------
 * fs_decode_attention_fused_static - fs_decode_attention_fused for callers that cannot allocate
 * device memory or hand over a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The counters of the persistent sweep and the partial rows of
 * split pairs live in a fixed array inside the library (16 MiB + 128 KiB + 256 B of device memory,
 * held on every GPU the library runs on until the process ends) instead of in part_o, part_lse and
 * claim_dev; the call allocates and frees nothing.  The sweep is the persistent one for bf16 K/V
 * from 1024 items on, one workgroup per item otherwise; out/lse are, bit for bit, what
 * fs_decode_attention_fused leaves with the same sweep.
 *
 *  Limit: a list with a split pair (n_items > n_pairs) may have at most 32768 partial rows,
 *  n_items * G <= 32768, else FS_ECAPACITY and nothing is launched.  A list without a split pair
 *  has no such limit.
 *  Every call on one GPU uses that GPU's one array: calls that may overlap in time on one GPU
 *  (two streams, two threads) race and must be serialised by the caller.  The array keeps the last
 *  call's contents; the call clears the counters it needs at zero itself (a fill kernel).
 *  The first call on a device looks up the array's address (not a stream operation): make one
 *  call on each device before capturing a graph that contains this call.
 *
 * Everything else (arguments, errors) as for fs_decode_attention_fused.
 */
FS_API fs_status fs_decode_attention_fused_static(const fs_shape* shape, const fs_kv_view* kv,
                                                  const fs_work_item* items_dev, const int32_t* sched_dev,
                                                  int64_t n_items, const int64_t* chunk_indptr_dev,
                                                  int64_t n_pairs, float* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------
 * fs_merge_lse - combine the chunk partials of each pair (split-K merge):
 *     lse = ln sum_c exp(lse_c),   out = sum_c exp(lse_c - lse) * o_c
 * Rows [p*G, p*G+G) of out/lse belong to pair p; its partial rows are
 * [chunk_indptr[p]*G, chunk_indptr[p+1]*G).
 *
 *  part_o, part_lse  DEVICE in   as written by fs_decode_attention
 *  chunk_indptr_dev  DEVICE in   [n_pairs+1]
 *  out               DEVICE out  [n_pairs*G][head_dim] fp32
 *  lse               DEVICE out  [n_pairs*G] fp32
 *
 * n_pairs == 0 is a no-op.  FS_EINVAL: NULL pointers, group < 1.
 * FS_EUNSUPPORTED: head_dim != 128.
 */
FS_API fs_status fs_merge_lse(const float* part_o, const float* part_lse, const int64_t* chunk_indptr_dev,
                       int64_t n_pairs, int32_t group, int32_t head_dim,
                       float* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------
 * Chunked-prefill attention - the attention of the batches that the paper's
 * fine-grained chunked prefill (Section 3.1) forms: n_new[r] new tokens of request
 * r behind n_done[r] processed ones, chunks of several requests in one batch.
 * New token i of the chunk sits at position n_done + i and attends to the cached
 * tokens [0, n_done + i] (prefill phase, Section 2.1.1); the cache already holds
 * the chunk's own K and V.
 *
 * Q of the batch is the ragged concatenation of the new tokens in request order:
 * [sum n_new][n_q_heads][head_dim] bf16, passed as fs_kv_view.q.  The page table
 * of fs_kv_view follows the pair order of the list built here and covers
 * n_done + n_new tokens per pair.
 *
 * One unit of kernel work: query tokens [q_begin, q_end) of one pair's chunk (a
 * tile) against the cached tokens [kv_begin, kv_end) (a split-K chunk of the keys
 * the tile sees).  32 bytes, compared bit for bit against the oracle. */
typedef struct {
  int32_t pair;         /* index of the (request, head) pair in this rank's list  */
  int32_t q_begin;      /* first new token of the tile, within the chunk          */
  int32_t q_end;        /* one past the last                                      */
  int32_t n_done;       /* tokens of the request before the chunk                 */
  int32_t kv_begin;     /* first cached token of this item, a multiple of 32      */
  int32_t kv_end;       /* one past the last, <= n_done + q_end                   */
  int32_t q_row;        /* Q row of (token q_begin, first q-head of the group)    */
  int32_t part_row;     /* first partial-output row: item_index * T               */
} fs_prefill_item;

typedef struct {
  int32_t req, kv_head, n_done, n_new;
} fs_prefill_pair;

/* fs_build_prefill_worklist - pairs (r, h) with owner == rank and n_new[r] > 0, in
 * ascending (r, h).  Pair p is cut into ceil(n_new/tile_tokens) tiles; a tile ending
 * at token q_end sees the keys [0, n_done + q_end), cut into chunks of
 * kv_chunk_tokens keys (0 = one chunk), one item each, consecutive per tile;
 * chunk_indptr[k] is the first item of tile k (tiles numbered in list order).
 * With T = tile_tokens*G rows per tile: item i writes partial rows [i*T, (i+1)*T),
 * tile k owns final rows [k*T, (k+1)*T), both token-major and q-head-minor within
 * the tile; so pair p's final rows are contiguous from out_indptr[p]:
 * row(token i, group member g) = out_indptr[p] + i*G + g (rows between the end of a
 * pair's short last tile and the next pair are padding).  sched lists items by
 * decreasing kv_end - kv_begin, equal ones by increasing index.
 *
 *  n_done, n_new HOST in [n_req]      each >= 0
 *  owner         HOST in [n_req*n_kv_heads]
 *  tile_tokens   query tokens per tile, >= 1 (fs_prefill_tile_tokens(G) is the kernel's size)
 *  kv_chunk_tokens  0 or a positive multiple of 32
 *  items, sched  HOST out [items_cap]
 *  pairs         HOST out [pairs_cap]
 *  chunk_indptr  HOST out [tiles_cap+1]
 *  out_indptr    HOST out [pairs_cap+1]
 *                All five NULL (capacities 0): count only.
 *  n_items, n_pairs, n_tiles  HOST out, always written when the arguments are valid
 *
 * FS_ECAPACITY: an array is too small (nothing but the counts is valid).
 * FS_EINVAL: bad shape, rank, tile or chunk size, negative counts, owner outside
 * [0, R), more Q or partial rows than int32 holds. */
FS_API fs_status fs_build_prefill_worklist(const fs_shape* shape, const int32_t* n_done, const int32_t* n_new,
                                           const int32_t* owner, int32_t rank, int32_t tile_tokens,
                                           int32_t kv_chunk_tokens,
                                           fs_prefill_item* items, int64_t items_cap,
                                           fs_prefill_pair* pairs, int64_t pairs_cap,
                                           int32_t* sched, int64_t* chunk_indptr, int64_t tiles_cap,
                                           int64_t* out_indptr,
                                           int64_t* n_items, int64_t* n_pairs, int64_t* n_tiles);

/* fs_choose_prefill_chunk - a split-K chunk for one rank's prefill batch.  A batch with few long contexts (the
 * fine-grained chunked prefill of Section 3.1 forms such batches when little is waiting) runs as long as its
 * longest tile takes unless the keys are cut; a large batch needs no cut, and every cut costs partial rows and
 * merge work.  The chunk is four thirds of a slot's fair share of the whole: with T the keys the rank's tiles
 * see, all told, ceil(4 T / (3 n_slots)), rounded up to a multiple of 32 keys and held within
 * [min_chunk, max_chunk].
 *
 *  max_chunk, min_chunk   multiples of 32, 32 <= min_chunk <= max_chunk
 *  n_slots          workgroups the GPU runs at a time (two per compute unit for the default kernel shape), >= 1
 *  kv_chunk_tokens  HOST out  the chosen chunk
 *  n_items          HOST out  the list's length with it
 *
 * FS_EINVAL: bad chunk bounds, n_slots < 1, and whatever fs_build_prefill_worklist refuses. */
FS_API fs_status fs_choose_prefill_chunk(const fs_shape* shape, const int32_t* n_done, const int32_t* n_new,
                                         const int32_t* owner, int32_t rank, int32_t tile_tokens,
                                         int32_t max_chunk, int32_t min_chunk, int64_t n_slots,
                                         int32_t* kv_chunk_tokens, int64_t* n_items);

/* Query tokens one kernel workgroup covers for a group of G q-heads per KV head
 * (the natural tile_tokens; depends on the "prefill_waves" and "prefill_col_tiles"
 * options).  -1 for a group outside [1, 16]. */
FS_API int32_t fs_prefill_tile_tokens(int32_t group);

/* fs_prefill_attention - for every item, every token i in [q_begin, q_end) and g in
 * [0, G), with q = Q row q_row + (i - q_begin)*n_q_heads + g and t over the item's
 * cached tokens the query may see, [kv_begin, min(kv_end, n_done + i + 1)):
 *     s_t = sm_scale * <q, K_t>
 *     part_lse[row] = ln sum_t exp(s_t),   part_o[row][:] = sum_t exp(s_t - lse) * V_t
 * with row = part_row + (i - q_begin)*G + g; a row that sees none of the item's keys
 * gets part_o = 0 and part_lse = -inf.  Rows of a short last tile beyond its tokens
 * are written as zeros (part_lse = 0).  fs_merge_lse(part_o, part_lse,
 * chunk_indptr, n_tiles, T, head_dim, out, lse) then gives the final rows.  fp32
 * scores, softmax and accumulation; in P.V, V enters as bf16 and the softmax weights as
 * a sum of two bf16 terms, or, when kv->v_range == FS_V_FP16_RANGE, both as fp16.
 *
 *  items_dev  DEVICE in  [n_items]   as built by fs_build_prefill_worklist
 *  sched_dev  DEVICE in  [n_items]   launch order, or NULL for index order
 *  tile_tokens  the value the list was built with, == fs_prefill_tile_tokens(G)
 *               or smaller
 *  part_o     DEVICE out [n_items*T][head_dim] fp32, T = tile_tokens*G
 *  part_lse   DEVICE out [n_items*T] fp32
 *
 * n_items == 0 is a no-op.  FS_EINVAL: NULL pointers, bad shape, G > 16,
 * tile_tokens out of range, misaligned pools, sm_scale not finite or <= 0 (the kernel's
 * lazy running maximum is taken on the raw scores), unknown v_range or kv_dtype, fp8 K/V without scales.
 * FS_EUNSUPPORTED: head_dim != 128, page_tokens != 16.  FS_EHIP: launch failure.
 * bf16 or fp8 K/V.  With fp8 the K scales must be positive (a quantisation scale is; the same lazy maximum
 * is taken per page before the page's scale is applied), and scales are read by slot or, when
 * kv->page_scales is given, in page-table order, as in the decode calls. */
FS_API fs_status fs_prefill_attention(const fs_shape* shape, const fs_kv_view* kv,
                                      const fs_prefill_item* items_dev, const int32_t* sched_dev,
                                      int64_t n_items, int32_t tile_tokens, float* part_o, float* part_lse,
                                      void* stream);

/* fs_prefill_attention_fused - fs_prefill_attention and the split-K merge in one call (prefill phase,
 * Section 2.1.1; the batches of Section 3.1's chunked prefill).  An item that is all of its tile (kv_begin
 * == 0 and kv_end == n_done + q_end) writes the tile's final rows, out_indptr[pair] + token*G + g,
 * straight from the kernel; the merge runs for the tiles that are split and is not launched when n_items ==
 * n_tiles.  out/lse hold, bit for bit, what fs_prefill_attention followed by fs_merge_lse over all tiles
 * leaves.
 *
 *  chunk_indptr_dev  DEVICE in   [n_tiles+1]   as built by fs_build_prefill_worklist
 *  out_indptr_dev    DEVICE in   [n_pairs+1]   likewise
 *  part_o, part_lse  DEVICE scratch, sized and indexed as for fs_prefill_attention (rows of unsplit tiles stay
 *                    untouched); may be NULL when n_items == n_tiles
 *  out, lse          DEVICE out  [n_tiles*T][head_dim], [n_tiles*T] fp32
 *
 * Errors as for fs_prefill_attention, and FS_EINVAL for n_tiles outside [1, n_items] or a NULL
 * chunk_indptr_dev, out_indptr_dev, out or lse. */
FS_API fs_status fs_prefill_attention_fused(const fs_shape* shape, const fs_kv_view* kv,
                                            const fs_prefill_item* items_dev, const int32_t* sched_dev,
                                            int64_t n_items, int32_t tile_tokens,
                                            const int64_t* chunk_indptr_dev, int64_t n_tiles,
                                            const int64_t* out_indptr_dev, float* part_o, float* part_lse,
                                            float* out, float* lse, void* stream);

/* ---------------------------------------------------------------------------
 * fs_stream_read_probe - measurement aid, not a step of the path: read `bytes`
 * bytes once with the access pattern of the attention sweep (16 bytes per lane,
 * contiguous per wavefront) and discard them.  Timing it gives the read rate this
 * GPU actually reaches, to set beside the nominal HBM peak.
 *
 *  buf_dev   DEVICE in   16-byte aligned, bytes a positive multiple of 16
 *  sink_dev  DEVICE out  at least 4 bytes (written only in a 1-in-2^32 case)
 *
 * FS_EINVAL: NULL pointer, bad size or alignment.  FS_EHIP: launch failure.
 */
FS_API fs_status fs_stream_read_probe(const void* buf_dev, int64_t bytes, void* sink_dev, void* stream);

/* Launch-shape knobs for measurement sweeps: "waves_per_group" in {1,2,4}, "prefetch_pages" in [1,3],
 * "prefill_col_tiles" in {1,2,4}, "prefill_waves" in {4,8} (the pair (8,4) has no kernel).  They select
 * among kernels that compute the same thing (sums in another order); nothing numeric is an option.
 * The table is process-wide and not synchronised: set it before launching from several threads, not
 * while another thread is inside a call.
 * Unknown key or a value outside the documented range: FS_EINVAL, nothing changes. */
FS_API fs_status fs_set_option(const char* key, int32_t value);
FS_API int32_t   fs_get_option(const char* key);   /* -1 for an unknown key */

FS_API const char* fs_last_error(void);   /* message of this thread's last non-OK status */
FS_API int32_t     fs_abi_version(void);  /* FS_ABI_VERSION the library was built with   */

#ifdef __cplusplus
}
#endif
#endif /* FAILSAFE_H */
