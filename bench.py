#!/usr/bin/env python3
"""Benchmark: one GPU's cyclic/hybrid decode-attention share on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--rank k]

A step is one pass of the whole hot path over one synthetic batch: placement (S1+S2) and the
rank's work list (S3) built on the host by the library, the list copied to the GPU, the
attention sweep (S4) and the split-K merge (S5) - the last two as one library call
(fs_decode_attention_fused: pairs that are a single item need no merge).  Q, the paged K/V pool and the page table are
resident in HBM before the timed region starts.  Host work for step t+1 overlaps the GPU work
of step t (nothing synchronises inside the timed region), as it would in a serving loop.

Prints ONE JSON line.  `value` is algorithmic GB/s of the whole step; `roofline` is the
attention kernel alone against the HBM peak; `cpu_baseline` is the fp64 oracle timed on this
box's host cores (context, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published

# HBM bytes per attention launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this script (see
# profiles/).  A figure belongs to one kernel on one list: the key is (config, rank, seed, chunk, placement,
# kernel); any other run reports null.
MEASURED_TRAFFIC_BYTES = {
    (2, 0, 20251116, 3728, "requests", "decode_bf16_persistent_kernel"): 1972031652,          # profiles/decode_bf16_persistent_kernel_cfg2_70b_claimed_records_rank0.txt
    (2, 0, 20251116, 6640, "requests", "decode_bf16_kernel"): 1966162992,                     # profiles/decode_bf16_kernel_cfg2_70b_chunk6640_rank0.txt (--classic --chunk 6640)
    (2, 0, 20251116, "512 units", "requests", "decode_bf16_persistent_kernel"): 1965815821,   # profiles/decode_bf16_units_kernel_cfg2_70b_rank0.txt (--units 0)
    (2, 0, 20251116, 2048, "requests", "decode_bf16_persistent_kernel"): 1971410666,          # profiles/decode_bf16_persistent_kernel_cfg2_70b_rank0.txt (--chunked --persistent)
    (2, 0, 20251116, 2048, "requests", "decode_bf16_kernel"): 1981789512,                     # profiles/decode_bf16_kernel_cfg2_70b_rank0.txt (--chunked --classic)
    (1, 0, 20251115, "512 units", "requests", "decode_bf16_persistent_kernel"): 408077179,    # profiles/decode_bf16_units_kernel_cfg1_8b_hybrid_rank0.txt (--units 512)
    (1, 0, 20251115, 2048, "requests", "decode_bf16_kernel"): 407940537,                      # profiles/decode_bf16_kernel_cfg1_8b_hybrid_rank0.txt
    (3, 0, 20251117, 688, "requests", "decode_bf16_kernel"): 69265433,                        # profiles/decode_bf16_kernel_cfg3_skew_rank0.txt
    (0, 0, 20251114, 0, "requests", "decode_bf16_kernel"): 3205046,                           # profiles/decode_bf16_kernel_cfg0_tiny_rank0.txt
    (4, 0, 20251118, 0, "requests", "decode_fp8_kernel"): 1561925135,                         # profiles/decode_fp8_kernel_cfg4_mha_fp8_rank0.txt
    (2, 0, 20251116, 2048, "requests", "decode_fp8_kernel"): 1007783948,                      # profiles/decode_fp8_kernel_cfg2_70b_as_fp8_rank0.txt (--kv-dtype fp8 --chunked)
    (2, 0, 20251116, 6640, "requests", "decode_fp8_kernel"): 992022007,                       # profiles/decode_fp8_kernel_cfg2_70b_as_fp8_builders_chunk_rank0.txt (--kv-dtype fp8)
}
KERNEL_LAUNCHES = 30       # launches of the attention kernel timed one by one for the roofline figure


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="synthetic batch 0..4 (2 = 70B-shaped, the target)")
    ap.add_argument("--rank", type=int, default=0)
    ap.add_argument("--chunk", type=int, default=None, help="override the split-K chunk (tokens)")
    ap.add_argument("--waves", type=int, default=None)
    ap.add_argument("--prefetch", type=int, default=None)
    ap.add_argument("--separate-kv", action="store_true", help="K and V in two pools instead of interleaved")
    ap.add_argument("--scales-by-slot", action="store_true",
                    help="fp8: the kernels gather the scales from the by-slot arrays instead of reading them in page-table order")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="replay the GPU side of a step as a HIP graph per slot instead of launching it eagerly (measured "
                         "slower here: ~14 us pass between the end of one graph and the first kernel of the next)")
    ap.add_argument("--list", choices=["host", "device"], default="host",
                    help="where the kernels read the step's work list: host = in place from the pinned host memory the "
                         "builder writes (no upload; default); device = a copy uploaded every step")
    ap.add_argument("--classic", action="store_true",
                    help="one workgroup per item (fs_decode_attention) even for long lists")
    ap.add_argument("--persistent", action="store_true",
                    help="the persistent form of the sweep (fs_decode_attention_persistent: workgroups claim items, "
                         "partial rows leave in bursts) even for short lists; by default it is used from 1024 items on")
    ap.add_argument("--units", type=int, default=None, metavar="N",
                    help="cut the share into N equal runs of pages (0 = two per compute unit) and sweep them with one "
                         "resident workgroup each (fs_build_worklist_units + fs_decode_attention_units).  Default: the chunked list")
    ap.add_argument("--chunked", action="store_true",
                    help="the chunked list (fs_build_worklist) on the config's own chunk also for a large share (default there: "
                         "a chunk of the builder's choice, one workgroup per item)")
    ap.add_argument("--claim-records", action="store_true",
                    help="launch records claimed in order by two resident workgroups per compute unit instead of one workgroup "
                         "per record (default on a large bf16 share)")
    ap.add_argument("--no-records", action="store_true",
                    help="hand the kernels the items (they look each one up themselves) instead of launch records")
    ap.add_argument("--merge-kernel", action="store_true",
                    help="launch records: merge split pairs with a second kernel also where the default merges inside the sweep")
    ap.add_argument("--merge-in-sweep", action="store_true",
                    help="launch records: merge split pairs inside the sweep also on equal runs (default there: a second kernel)")
    ap.add_argument("--two-calls", action="store_true",
                    help="the step calls fs_decode_attention[_persistent] and fs_merge_lse instead of fs_decode_attention_fused")
    ap.add_argument("--placement", choices=["requests", "heads"], default="requests",
                    help="requests: the batch's TP/DP mix per request; heads: the paper's head-level hybrid (layer 0)")
    ap.add_argument("--cold", action="store_true", help="also time the kernels with L2 and the memory-side cache scrubbed before every launch")
    ap.add_argument("--all-ranks", action="store_true", help="also time every rank's share in turn (kernels only) and report the spread")
    ap.add_argument("--force-tail", action="store_true", help="config 3: request 0 gets 131072 tokens")
    ap.add_argument("--seed", type=int, default=None, help="draw the batch from this seed instead of the config's own")
    ap.add_argument("--kv-dtype", choices=["bf16", "fp8"], default=None,
                    help="keep the config's batch but hold its K/V in this type (fp8: e4m3 with a scale per slot)")
    ap.add_argument("--path", choices=["decode", "prefill"], default="decode",
                    help="decode: the measured decode-attention share (default); prefill: the chunked-prefill attention share")
    ap.add_argument("--prefill-waves", type=int, default=None)
    ap.add_argument("--prefill-col-tiles", type=int, default=None)
    ap.add_argument("--prefill-wide-v", action="store_true",
                    help="prefill: keep V in bf16 and feed the weights as bf16 hi + lo (for values beyond fp16's range)")
    ap.add_argument("--prefill-budget", type=int, default=8192, help="prefill path: token budget of the batch")
    ap.add_argument("--prefill-queue", type=int, default=64, help="prefill path: waiting prompts")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (one rank's share at its real shape); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        return 2

    if args.path == "prefill":
        import bench_prefill
        return bench_prefill.run(args)

    import torch
    import paper_2511_14116_amd as fs
    from workloads import make_requests, make_q, make_kv_pool

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path to time", file=sys.stderr)
        return 2
    if not os.path.exists(fs.library_path()):
        from paper_2511_14116_amd.build import build
        build(verbose=False)
    fs.load_library()
    if args.waves:
        fs.fs_set_option("waves_per_group", args.waves)
    if args.prefetch:
        fs.fs_set_option("prefetch_pages", args.prefetch)

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()
    sptr = stream.cuda_stream

    # ---- synthetic batch ---------------------------------------------------------------------
    kw = dict(force_first_len=131072) if (args.config == 3 and args.force_tail) else {}
    w = make_requests(args.config, seed=args.seed, **kw)
    if args.kv_dtype:
        w["kv_dtype"] = args.kv_dtype
    MIN_CHUNK = 256          # floor of the adaptive split-K chunk (tokens)
    B, Hq, Hkv, R, G = w["n_req"], w["n_q_heads"], w["n_kv_heads"], w["n_ranks"], w["group"]
    shape = fs.FsShape(B, Hq, Hkv, w["head_dim"], w["page_tokens"], R)
    ctx, mode = w["ctx_len"], w["mode"]
    q_bits = make_q(w["seed"], B, Hq, w["head_dim"])
    if args.placement == "heads":
        owner, dp_rank, rank_load, _dp_load = fs.fs_build_placement_hybrid_heads(shape, ctx, layer=0)
    else:
        owner, dp_rank, rank_load = fs.fs_build_placement(shape, ctx, mode)
    n_cu = torch.cuda.get_device_properties(dev).multi_processor_count

    def chunk_for(rank):
        """The config's chunk; where it is the builder's choice, four thirds of a compute unit's share of the rank's tokens."""
        if args.chunk is not None:
            return args.chunk
        if w.get("chunk_adaptive") and w["chunk_tokens"] > MIN_CHUNK:
            return fs.fs_choose_chunk_tokens(shape, ctx, owner, rank, w["chunk_tokens"], MIN_CHUNK, n_cu)[0]
        return w["chunk_tokens"]

    # A share is large when each of the 2 x n_cu workgroups the chip runs at a time has this many pages to read.
    UNIT_MIN_PAGES = 256

    def pages_of(rank):
        return sum(-(-int(ctx[r]) // w["page_tokens"]) for r in range(B) for h in range(Hkv) if owner[r, h] == rank)

    def units_for(rank):
        """Two resident workgroups per compute unit, but at least 16 pages (256 tokens) to a run."""
        if args.units:
            return args.units
        return max(1, min(2 * n_cu, pages_of(rank) // 16))

    # A large share, left to the builder (no flag that names a list or a sweep): the chunked list launched from records,
    # split pairs merged inside the sweep, on a chunk that is a fraction of what one of a compute unit's two resident
    # workgroups gets of the rank's tokens (no item may stick out at the end, and no finer than that, since every cut
    # costs partial rows and an item start).
    #  bf16: resident workgroups claim the records (half a workgroup's share per item: they take 2-3 each and their rows
    #    leave in bursts); same box, config 2, step: 300-305 us against 301-308 with one workgroup per record on 8/9 of
    #    a share, 304-311 on 512 equal runs (--units 0) and 309-314 on the config's own 2048-token chunks (--chunked).
    #  fp8: one workgroup per record on 8/9 of a share (the resident forms measure no faster with fp8 K/V).
    # Small shares: one workgroup per record on the config's chunk, or four thirds of a compute unit's share.
    large = pages_of(args.rank) >= UNIT_MIN_PAGES * 2 * n_cu
    auto_large = (large and args.units is None and not args.chunked and not args.classic and not args.persistent
                  and args.chunk is None and w["chunk_tokens"] > 0 and not args.no_records and not args.two_calls)
    if args.claim_records and (args.units is not None or args.no_records or args.two_calls or args.persistent):
        print("bench.py: --claim-records goes with the chunked list launched from records in one call", file=sys.stderr)
        return 2
    claim_records = args.claim_records or (auto_large and w["kv_dtype"] == "bf16")
    if auto_large:
        large_slots = 16 * n_cu // 3 if claim_records else 3 * n_cu
        if not claim_records:
            args.classic = True

        def chunk_for(rank):      # noqa: F811
            return fs.fs_choose_chunk_tokens(shape, ctx, owner, rank, 32768, MIN_CHUNK, large_slots)[0]
    chunk = chunk_for(args.rank)
    # (fp8 K/V: the resident forms run and measure no faster than one workgroup per item)
    units = args.units is not None

    if units:
        n_units_req = units_for(args.rank)
        items, pairs, unit_indptr, chunk_indptr = fs.fs_build_worklist_units(shape, ctx, owner, args.rank, n_units_req)
        n_units = len(unit_indptr) - 1
        sched = None
        chunk = 0
    else:
        items, pairs, sched, chunk_indptr = fs.fs_build_worklist(shape, ctx, owner, args.rank, chunk)
    n_items, n_pairs = len(items), len(pairs)
    if n_items == 0:
        print("bench.py: this rank's share is empty", file=sys.stderr)
        return 2
    kv = make_kv_pool(w["seed"], np.stack([pairs["req"], pairs["kv_head"]], axis=1), ctx, kv_dtype=w["kv_dtype"])

    from paper_2511_14116_amd.device import DeviceShare
    ds = DeviceShare(shape, q_bits, kv, w["sm_scale"], interleave_kv=not args.separate_kv,
                     scales_by_page=not args.scales_by_slot)

    # ---- algorithmic bytes ---------------------------------------------------------------------
    tok_heads = int(rank_load[args.rank])
    n_pages = int(kv["page_indptr"][-1])
    elt = 2 if w["kv_dtype"] == "bf16" else 1
    kv_bytes = tok_heads * 2 * w["head_dim"] * elt          # K and V rows actually attended
    scale_bytes = n_pages * 8 if w["kv_dtype"] == "fp8" else 0
    q_bytes = n_pairs * G * w["head_dim"] * 2
    # list bytes the sweep reads: 64-byte records, or 32-byte items + launch order; run boundaries for equal runs
    table_bytes = n_pages * 4 + (n_items * 64 if not (args.no_records or args.two_calls) else n_items * 32 + (0 if units else n_items * 4)) \
        + ((n_units + 1) * 8 if units else 0)
    row_bytes = w["head_dim"] * 4 + 4                       # one fp32 output row and its lse
    counts = np.diff(chunk_indptr)
    if args.two_calls:                                      # every item writes partial rows, the merge reads them all
        n_part_items, n_direct_pairs = n_items, 0
    else:                                                   # fused: only split pairs go through partial rows
        n_part_items, n_direct_pairs = int(counts[counts > 1].sum()), int((counts == 1).sum())
    part_bytes = n_part_items * G * row_bytes
    decode_bytes = (kv_bytes + scale_bytes + q_bytes + table_bytes + part_bytes + n_direct_pairs * G * row_bytes
                    + (0 if args.two_calls else (n_pairs + 1) * 8))
    merge_bytes = part_bytes + (n_pairs - n_direct_pairs) * G * row_bytes + (n_pairs + 1) * 8
    if not args.two_calls and n_part_items == 0:
        merge_bytes = 0                                     # nothing is split: no merge is launched
    step_bytes = decode_bytes + merge_bytes

    # ---- buffers for the per-step work list --------------------------------------------------------
    # One blob per step holds items | sched | chunk_indptr.  The host builds it in pinned memory (N_SLOTS
    # buffers in rotation), which is mapped into the GPU's address space: by default the kernels read the
    # list in place (85 KB per step on the 70B-shaped batch, fetched once per item while the previous item's
    # rows are merged), so a step is one library call, launched eagerly.  --list device uploads the blob
    # into HBM every step instead; --graph replays sweep, merge (and upload) as one HIP graph per slot.
    def up(x):
        return (x + 255) & ~255
    off_items = 0
    off_sched = up(off_items + n_items * 32)
    off_indptr = up(off_sched + ((n_units + 1) * 8 if units else n_items * 4))      # units: unit_indptr sits where sched would
    off_records = up(off_indptr + (n_pairs + 1) * 8)          # launch records of the step's list (one-call form)
    off_records2 = up(off_records + n_items * 64)             # and records that send every row to part_o (the sweep timed alone)
    blob_bytes = up(off_records2 + n_items * 64)
    N_SLOTS = 4
    dev_blobs = [torch.empty(blob_bytes, dtype=torch.uint8, device=dev) for _ in range(N_SLOTS)]
    host_blobs = [torch.zeros(blob_bytes, dtype=torch.uint8, pin_memory=True) for _ in range(N_SLOTS)]
    slot_done = [torch.cuda.Event() for _ in range(N_SLOTS)]     # the step that last used this slot finished
    host_views = []
    for hb in host_blobs:
        a = hb.numpy()
        host_views.append((a[off_items:off_items + n_items * 32].view(fs.ITEM_DTYPE),
                           np.empty(n_pairs, dtype=fs.PAIR_DTYPE),
                           a[off_sched:off_sched + (n_units + 1) * 8].view(np.int64) if units else
                           a[off_sched:off_sched + n_items * 4].view(np.int32),
                           a[off_indptr:off_indptr + (n_pairs + 1) * 8].view(np.int64)))
    host_rec = [hb.numpy()[off_records:off_records + n_items * 64].view(fs.RECORD_DTYPE) for hb in host_blobs]
    host_rec2 = [hb.numpy()[off_records2:off_records2 + n_items * 64].view(fs.RECORD_DTYPE) for hb in host_blobs]
    part_o = torch.empty((n_items * G, w["head_dim"]), dtype=torch.float32, device=dev)
    part_lse = torch.empty(n_items * G, dtype=torch.float32, device=dev)
    out = torch.empty((n_pairs * G, w["head_dim"]), dtype=torch.float32, device=dev)
    lse = torch.empty(n_pairs * G, dtype=torch.float32, device=dev)

    # Every library call of the step, with its arguments marshalled once.
    owner_buf = np.empty((B, Hkv), dtype=np.int32)
    dp_buf = np.empty(B, dtype=np.int32)
    load_buf = np.zeros(R, dtype=np.int64)
    ctx_c = np.ascontiguousarray(ctx, dtype=np.int32)
    mode_c = np.ascontiguousarray(mode, dtype=np.uint8)
    if args.placement == "heads":
        dpl_buf = np.zeros(R, dtype=np.int64)
        call_place = fs.bind_build_placement_hybrid_heads(shape, ctx_c, owner_buf, dp_buf, load_buf, dpl_buf)
    else:
        dpl_buf = None
        call_place = fs.bind_build_placement(shape, ctx_c, mode_c, owner_buf, dp_buf, load_buf)
    if units:
        call_list = [fs.bind_build_worklist_units(shape, ctx_c, owner_buf, args.rank, n_units_req, *hv) for hv in host_views]
    else:
        call_list = [fs.bind_build_worklist(shape, ctx_c, owner_buf, args.rank, chunk, *hv) for hv in host_views]

    # The persistent form pays off once every workgroup walks several items (it saves the scattered stores
    # and the relaunches); with one item or fewer per workgroup slot it is the same work plus a counter.
    persistent = not args.classic and not units and not claim_records and (args.persistent or (w["kv_dtype"] == "bf16" and n_items >= 1024))
    if args.persistent and n_items < 1024 and not args.two_calls:
        print("bench.py: --persistent below 1024 items needs --two-calls (the fused call picks the sweep by list length)",
              file=sys.stderr)
        return 2
    claim = torch.zeros(2, dtype=torch.int32, device=dev)    # the persistent sweep's counters; every launch leaves them at zero
    pair_counters = torch.zeros(n_pairs, dtype=torch.int32, device=dev)   # one per pair for the merge inside the sweep; likewise
    # Split pairs merged by the sweep itself (no second kernel): pays on a short launch (config 3: 21.7 -> 18.4 us per
    # step), where the merge kernel's launch is a third of the time; on the equal-run sweeps of the large shares the
    # hand-over at the end of every workgroup's life costs what the second launch cost (config 2: 311.5 against 310.0).
    merge_in_sweep = args.merge_in_sweep or (not units and not args.merge_kernel)
    # Launch records: the host resolves every item (page-table offset, chunk count, first slots) while it builds the
    # list, so a workgroup starts with one read instead of four dependent ones.  The counter form takes items only.
    use_records = not args.no_records and not persistent and not args.two_calls
    page_indptr_h = np.ascontiguousarray(kv["page_indptr"], dtype=np.int64)
    page_ids_h = np.ascontiguousarray(kv["page_ids"], dtype=np.int32)
    call_records = [fs.bind_build_launch_records(shape, hv[0], None if units else hv[2], hv[3], n_pairs, page_indptr_h,
                                                 page_ids_h, host_rec[s_]) for s_, hv in enumerate(host_views)]

    def bind_gpu_calls(stream_ptr):
        """Per blob: the sweep alone, the merge alone, and the one-call form of both."""
        dec, mrg, fused = [], [], []
        for db in (host_blobs if host_list else dev_blobs):
            base = db.data_ptr()        # a pinned host blob is mapped into the GPU's address space at the same address
            if use_records:
                ui = (base + off_sched) if units else None
                dec.append(fs.bind_decode_attention_records(shape, ds.view, base + off_records2, n_items, ui, n_units if units else 0,
                                                            None, 0, part_o, part_lse, out, lse, None,
                                                            claim if claim_records else None, stream_ptr))
                mrg.append(fs.bind_merge_lse(part_o, part_lse, base + off_indptr, n_pairs, G, w["head_dim"], out, lse, stream_ptr))
                fused.append(fs.bind_decode_attention_records(shape, ds.view, base + off_records, n_items, ui, n_units if units else 0,
                                                              base + off_indptr, n_pairs, part_o, part_lse, out, lse,
                                                              pair_counters if merge_in_sweep else None,
                                                              claim if claim_records else None, stream_ptr))
                continue
            if units:
                dec.append(fs.bind_decode_attention_units(shape, ds.view, base + off_items, n_items, base + off_sched, n_units,
                                                          None, 0, part_o, part_lse, None, None, stream_ptr))
                mrg.append(fs.bind_merge_lse(part_o, part_lse, base + off_indptr, n_pairs, G, w["head_dim"], out, lse, stream_ptr))
                fused.append(fs.bind_decode_attention_units(shape, ds.view, base + off_items, n_items, base + off_sched, n_units,
                                                            base + off_indptr, n_pairs, part_o, part_lse, out, lse, stream_ptr))
                continue
            if persistent:
                dec.append(fs.bind_decode_attention_persistent(shape, ds.view, base + off_items, base + off_sched,
                                                               n_items, claim, part_o, part_lse, stream_ptr))
            else:
                dec.append(fs.bind_decode_attention(shape, ds.view, base + off_items, base + off_sched, n_items,
                                                    part_o, part_lse, stream_ptr))
            mrg.append(fs.bind_merge_lse(part_o, part_lse, base + off_indptr, n_pairs, G, w["head_dim"],
                                         out, lse, stream_ptr))
            fused.append(fs.bind_decode_attention_fused(shape, ds.view, base + off_items, base + off_sched, n_items,
                                                        base + off_indptr, n_pairs, part_o, part_lse,
                                                        claim if persistent else None, out, lse, stream_ptr))
        return dec, mrg, fused

    host_list = args.list == "host"
    call_decode, call_merge, call_fused = bind_gpu_calls(sptr)

    def upload(slot: int):
        if not host_list:
            dev_blobs[slot].copy_(host_blobs[slot], non_blocking=True)

    def build_host(slot: int):
        load_buf.fill(0)
        if dpl_buf is not None:
            dpl_buf.fill(0)
        call_place()                                        # S1 + S2
        call_list[slot]()                                   # S3
        if use_records:
            call_records[slot]()                            # S3, written out for the kernels

    # The GPU side of step i reads device blob i % N_SLOTS and, next to it, uploads the blob of
    # step i+1 (which the host has built by then), so the upload never sits between two sweeps.
    def gpu_side(dec, mrg, fused, slot: int):
        if args.two_calls:
            dec[slot]()                                     # S4
            mrg[slot]()                                     # S5
        else:
            fused[slot]()                                   # S4 + S5

    def enqueue_eager(slot: int):
        gpu_side(call_decode, call_merge, call_fused, slot)
        upload((slot + 1) % N_SLOTS)

    for slot in range(N_SLOTS):                             # warm everything up eagerly once
        build_host(slot)
    upload(0)
    for slot in range(N_SLOTS):
        enqueue_eager(slot)
    torch.cuda.synchronize()

    # one HIP graph per slot: sweep -> merge -> upload of the next step's blob
    graphs = None
    if args.graph:
        cap_stream = torch.cuda.Stream()
        cap_decode, cap_merge, cap_fused = bind_gpu_calls(cap_stream.cuda_stream)
        graphs = []
        for slot in range(N_SLOTS):
            g = torch.cuda.CUDAGraph()
            nxt = (slot + 1) % N_SLOTS
            with torch.cuda.graph(g, stream=cap_stream):
                gpu_side(cap_decode, cap_merge, cap_fused, slot)
                upload(nxt)
            graphs.append(g)
        torch.cuda.synchronize()

    host_us, wait_us, enqueue_us = [], [], []

    def step(i: int):
        # on entry the blob of step i is built and its upload is enqueued; build the one of step i+1
        t0 = time.perf_counter()
        slot, nxt = i % N_SLOTS, (i + 1) % N_SLOTS
        # the last reader of pinned blob nxt must be done: the upload in step i-N_SLOTS, or, when the kernels read the
        # list in place, step i+1-N_SLOTS itself (busy poll: a blocking wait costs a timer tick)
        while not slot_done[nxt if host_list else slot].query():
            pass
        t1 = time.perf_counter()
        build_host(nxt)
        t2 = time.perf_counter()
        if graphs is None:
            enqueue_eager(slot)
        else:
            graphs[slot].replay()
        slot_done[slot].record(stream)
        t3 = time.perf_counter()
        wait_us.append((t1 - t0) * 1e6)
        host_us.append((t2 - t1) * 1e6)
        enqueue_us.append((t3 - t2) * 1e6)

    build_host(0)
    upload(0)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    host_us.clear(); wait_us.clear(); enqueue_us.clear()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    # The attention kernel alone, after the region (events inside it would only add gaps): KERNEL_LAUNCHES launches
    # whatever --steps is, each between its own pair of HIP events on the stream it is launched on.  It is the sweep the
    # step runs (same kernel, same list); in the fused step the rows of unsplit pairs go to out instead of part_o.
    def time_each(call, n):
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(n)]
        for a, b in evs:
            a.record(stream)
            call()
            b.record(stream)
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in evs])

    build_host(0)
    if use_records:     # for the sweep timed alone: records that send every item's rows to part_o
        hv0 = host_views[0]
        fs.fs_build_launch_records(shape, hv0[0], None if units else hv0[2], hv0[3], page_indptr_h, page_ids_h,
                                   direct_rows=False, out=host_rec2[0])
    upload(0)
    for _ in range(3):
        call_decode[0]()
    torch.cuda.synchronize()
    dec_ms = time_each(call_decode[0], KERNEL_LAUNCHES)
    fused_ms = time_each(call_fused[0], KERNEL_LAUNCHES)       # sweep + merge of the split pairs, as the step runs them

    def time_batch(call, n):
        """n launches back to back between one pair of events: the launch-to-launch period, without the few
        microseconds an event pair adds around a single launch."""
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(n):
            call()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    dec_batch_ms = time_batch(call_decode[0], KERNEL_LAUNCHES)

    # a graph step and an eager step must leave the same bits behind
    if graphs is not None:
        build_host(0)
        build_host(1)
        upload(0)
        graphs[0].replay()
        torch.cuda.synchronize()
        g_out, g_lse = out.clone(), lse.clone()
        out.fill_(float("nan")); lse.fill_(float("nan"))
        enqueue_eager(0)
        torch.cuda.synchronize()
        if not (torch.equal(g_out, out) and torch.equal(g_lse, lse)):
            print("bench.py: graph replay and eager launch disagree", file=sys.stderr)
            return 1
        out.fill_(float("nan")); lse.fill_(float("nan"))        # and so must the two-call and the one-call form
        call_decode[0](); call_merge[0]()
        torch.cuda.synchronize()
        if not (torch.equal(g_out, out) and torch.equal(g_lse, lse)):
            print("bench.py: fs_decode_attention_fused and the two calls disagree", file=sys.stderr)
            return 1

    # the merge kernel alone, timed after the region (its events would only add gaps inside it)
    m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    m0.record(stream)
    for _ in range(20):
        call_merge[0]()
    m1.record(stream)
    torch.cuda.synchronize()
    mrg_ms = np.array([m0.elapsed_time(m1) / 20])

    # sanity: the timed configuration produced finite numbers
    if not (torch.isfinite(out).all().item() and torch.isfinite(lse).all().item()):
        print("bench.py: non-finite output", file=sys.stderr)
        return 1

    # ---- stream-read probe over the same pool ----------------------------------------------------
    probe_gbs = None
    if not args.no_probe:
        pool = ds._pool if not isinstance(ds._pool, tuple) else ds._pool[0]
        nbytes = (pool.numel() * pool.element_size()) & ~15
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        for _ in range(3):
            fs.fs_stream_read_probe(pool, nbytes, sink, sptr)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record(stream)
        for _ in range(reps):
            fs.fs_stream_read_probe(pool, nbytes, sink, sptr)
        e1.record(stream)
        torch.cuda.synchronize()
        probe_gbs = nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9

    # ---- cold-cache kernel times: shares smaller than the 256 MB memory-side cache are otherwise
    # served from it when the same pool is swept again and again
    cold = None
    if args.cold:
        scrub = torch.empty(1 << 30, dtype=torch.uint8, device=dev)       # 1 GiB, read once before each launch
        sink2 = torch.zeros(4, dtype=torch.int32, device=dev)
        dts, mts = [], []
        for _ in range(20):
            fs.fs_stream_read_probe(scrub, scrub.numel(), sink2, sptr)
            c0, c1, c2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            c0.record(stream)
            call_decode[0]()
            c1.record(stream)
            call_merge[0]()
            c2.record(stream)
            torch.cuda.synchronize()
            dts.append(c0.elapsed_time(c1)); mts.append(c1.elapsed_time(c2))
        cold = {"decode_ms": round(float(np.mean(dts)), 5), "merge_ms": round(float(np.mean(mts)), 5),
                "decode_gbs": round(decode_bytes / (float(np.mean(dts)) * 1e-3) / 1e9, 1)}
        del scrub

    # ---- every rank's share in turn (the straggler view of the skewed batch) -----------------------
    per_rank = None
    if args.all_ranks:
        per_rank = []
        for k in range(R):
            if units:
                it_k, pr_k, ui_k, ip_k = fs.fs_build_worklist_units(shape, ctx, owner, k, units_for(k))
            else:
                it_k, pr_k, sc_k, ip_k = fs.fs_build_worklist(shape, ctx, owner, k, chunk_for(k))
            if len(it_k) == 0:
                per_rank.append({"rank": k, "kv_token_heads": 0, "n_items": 0, "kernels_us": 0.0, "gbs": 0.0})
                continue
            kv_k = make_kv_pool(w["seed"], np.stack([pr_k["req"], pr_k["kv_head"]], axis=1), ctx, kv_dtype=w["kv_dtype"])
            ds_k = DeviceShare(shape, q_bits, kv_k, w["sm_scale"], interleave_kv=not args.separate_kv)
            if units:
                ds_k.set_worklist_units(it_k, pr_k, ui_k, ip_k)
                run_k = ds_k.run_units
            else:
                ds_k.set_worklist(it_k, pr_k, sc_k, ip_k)
                if use_records:          # as the step launches it: from launch records, split pairs merged as the step merges them
                    ds_k.set_records(fs.fs_build_launch_records(shape, it_k, sc_k, ip_k, kv_k["page_indptr"], kv_k["page_ids"]))
                    pc_k = torch.zeros(max(len(pr_k), 1), dtype=torch.int32, device=dev)
                    run_k = fs.bind_decode_attention_records(shape, ds_k.view, ds_k.records, ds_k.n_items, None, 0, ds_k.chunk_indptr,
                                                             ds_k.n_pairs, ds_k.part_o, ds_k.part_lse, ds_k.out, ds_k.lse,
                                                             pc_k if merge_in_sweep else None, claim if claim_records else None, sptr)
                else:
                    run_k = (lambda: ds_k.run(persistent=persistent)) if args.two_calls else (lambda: ds_k.run_fused(persistent=persistent))
            for _ in range(5):
                run_k()
            r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 30
            r0.record(stream)
            for _ in range(reps):
                run_k()
            r1.record(stream)
            torch.cuda.synchronize()
            us = r0.elapsed_time(r1) * 1e3 / reps
            th = int(rank_load[k])
            per_rank.append({"rank": k, "kv_token_heads": th, "n_items": len(it_k), "kernels_us": round(us, 2),
                             "gbs": round(th * 2 * w["head_dim"] * elt / (us * 1e-6) / 1e9, 1)})
            del ds_k, kv_k
        times = [p_["kernels_us"] for p_ in per_rank if p_["n_items"]]
        rank_spread = {"min_us": min(times), "max_us": max(times), "mean_us": round(float(np.mean(times)), 2),
                       "max_over_mean": round(max(times) / float(np.mean(times)), 3)}

    # ---- CPU baseline: the oracle on this machine's host cores ---------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        cores = min(16, len(os.sched_getaffinity(0)))
        pr = pairs.view(np.int32).reshape(-1, 4)
        budget = 12_000_000                      # tok.heads: keeps this leg to some tens of seconds
        csum = np.cumsum(pr[:, 2].astype(np.int64))
        n_s = int(min(len(pr), max(1, np.searchsorted(csum, budget) + 1)))
        times = []
        t_leg = time.perf_counter()
        while len(times) < 9 and (len(times) < 3 or time.perf_counter() - t_leg < 10.0):   # short samples: repeat, take the median
            t1 = time.perf_counter()
            oo, ol = oracle.decode_attention_pairs(q_bits, kv, pr[:n_s], Hq, G, w["sm_scale"], workers=cores)
            times.append(time.perf_counter() - t1)
            if times[-1] > 5.0:
                break
        dt = float(np.median(times))
        s_tok = int(csum[n_s - 1])
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):        # the same sample on one core: one worker, single-threaded BLAS
            t1 = time.perf_counter()
            oracle.decode_attention_pairs(q_bits, kv, pr[:n_s], Hq, G, w["sm_scale"], workers=1)
            dt_one = time.perf_counter() - t1
        got = out[: n_s * G].cpu().numpy().astype(np.float64)
        err_ok = bool((np.abs(got - oo) <= 2e-3 + 1e-2 * np.abs(oo)).all()
                      and (np.abs(lse[: n_s * G].cpu().numpy() - ol) <= 1e-3).all())
        cpu = {"value": round(s_tok * 2 * w["head_dim"] * elt / dt / 1e9, 4), "unit": "GB/s", "cores": cores,
               "kind": "oracle", "sample": f"first {n_s} of {n_pairs} pairs of rank {args.rank} "
               f"({s_tok} KV-token-heads), fp64 numpy, median of {len(times)} runs: {dt:.2f} s",
               "kv_token_heads_per_s": round(s_tok / dt, 1), "gpu_matches_oracle_on_sample": err_ok,
               "one_core": {"value": round(s_tok * 2 * w["head_dim"] * elt / dt_one / 1e9, 4), "unit": "GB/s",
                            "seconds": round(dt_one, 2)}}

    dec_avg_ms = float(dec_batch_ms)
    achieved = decode_bytes / (dec_avg_ms * 1e-3) / 1e9
    kernel_name = ("decode_bf16" if w["kv_dtype"] == "bf16" else "decode_fp8") + ("_persistent_kernel" if persistent or units or claim_records else "_kernel")
    default_shape = (args.waves in (None, 4) and args.prefetch in (None, 2) and not args.separate_kv
                     and not args.scales_by_slot and not (args.config == 3 and args.force_tail))
    key = (args.config, args.rank, w["seed"], f"{n_units} units" if units else chunk, args.placement, kernel_name) if default_shape else None
    result = {
        "metric": "achieved HBM GB/s (% of peak) and KV-token-heads/s, rank-0 share, 1 MI355X",
        "value": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w["kv_dtype"] == "bf16" else "fp8_e4m3",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {w['name']}: B={B}, Hq={Hq}, Hkv={Hkv}, d=128, page=16, "
                               f"R={R}, rank {args.rank}, " + (f"{n_units} equal runs of pages" if units else f"chunk={chunk}") + f", seed={w['seed']}"
                               + (", head-level hybrid placement" if args.placement == "heads" else "")
                               + (f", K/V held as {args.kv_dtype}" if args.kv_dtype else ""),
                   "n_pairs": n_pairs, "n_items": n_items, "kv_token_heads": tok_heads,
                   "kv_bytes": kv_bytes, "step_bytes": step_bytes,
                   "sweep": "one resident workgroup per run of pages" if units else ("persistent" if persistent else
                            "resident workgroups claiming launch records" if claim_records else "one workgroup per item"),
                   "step_calls": "fs_build_launch_records + fs_decode_attention_records" if use_records else
                                 ("fs_decode_attention_units" + (" (sweep alone) + fs_merge_lse" if args.two_calls else "")) if units else
                                 ("fs_decode_attention[_persistent] + fs_merge_lse" if args.two_calls else "fs_decode_attention_fused"),
                   "merge_launched": bool(args.two_calls or (n_items > n_pairs and not (use_records and merge_in_sweep))),
                   "split_pairs_merged": "by a merge kernel" if (args.two_calls or not use_records or not merge_in_sweep) else
                                         "inside the sweep, by the workgroup that writes a pair's last partial rows",
                   "chunk_rule": None if units else ("given on the command line" if args.chunk is not None else
                                                     ("the builder's: items of half a resident workgroup's share of the rank's tokens" if claim_records else
                                                      "the builder's: items of 8/9 of a resident workgroup's share of the rank's tokens") if auto_large else
                                                     "the builder's: items of 4/3 of a compute unit's share, at most the config's chunk"
                                                     if (w.get("chunk_adaptive") and w["chunk_tokens"] > MIN_CHUNK) else "the config's"),
                   "kernel": kernel_name,
                   "waves_per_group": fs.fs_get_option("waves_per_group"),
                   "prefetch_pages": fs.fs_get_option("prefetch_pages"),
                   "kv_layout": "separate" if args.separate_kv else "interleaved",
                   "fp8_scales": None if w["kv_dtype"] != "fp8" else ("by slot" if args.scales_by_slot else "page-table order"),
                   "launch": "eager" if graphs is None else "hip graph per slot",
                   "work_list": "read in place from pinned host memory" if host_list else "uploaded every step"},
        "pct_of_hbm_peak": round(100.0 * step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "kv_token_heads_per_s": round(tok_heads / (ms_per_step * 1e-3), 1),
        "kernel_ms": {"decode_avg": round(dec_avg_ms, 5), "decode_avg_is": f"{KERNEL_LAUNCHES} launches back to back between one pair of events",
                      "decode_each_avg": round(float(dec_ms.mean()), 5), "decode_p50": round(float(np.median(dec_ms)), 5),
                      "decode_p10": round(float(np.percentile(dec_ms, 10)), 5),
                      "decode_p90": round(float(np.percentile(dec_ms, 90)), 5),
                      "decode_launches": int(len(dec_ms)),
                      "sweep_plus_merge_avg": round(float(fused_ms.mean()), 5),
                      "merge_alone_avg": round(float(mrg_ms.mean()), 5)},
        "host_us_per_step": {"builders_avg": round(float(np.mean(host_us)), 1),
                             "builders_p90": round(float(np.percentile(host_us, 90)), 1),
                             "enqueue_avg": round(float(np.mean(enqueue_us)), 1),
                             "wait_for_gpu_avg": round(float(np.mean(wait_us)), 1)},
        "stream_read_probe_gbs": None if probe_gbs is None else round(probe_gbs, 1),
        "roofline": {"bound": "hbm", "kernel": kernel_name,
                     "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "algorithmic_bytes_per_launch": decode_bytes,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(key)},
        "cpu_baseline": cpu,
    }
    if cold is not None:
        result["cold_cache"] = cold
    if per_rank is not None:
        result["per_rank"] = per_rank
        result["rank_time_spread"] = rank_spread
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
