"""Benchmark of the chunked-prefill attention share (`python bench.py --path prefill`).

A step is: route the waiting prompts (load-aware router), form the batch (Algorithm 1), place
the heads (head-level hybrid attention), build rank 0's tile list - all on the host by the
library - upload the list, and run the attention kernel over the batch's chunks.  Q, the paged
K/V pool and the page table are resident in HBM.  Prints ONE JSON line; `roofline` is the
attention kernel against the dense bf16 matrix-core peak.
"""
from __future__ import annotations

import gc
import json
import os
import sys
import time

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16, published
# HBM-side bytes of one prefill_bf16_kernel launch on the default batch (rocprofv3 --pmc FETCH_SIZE x 2.000 +
# WRITE_SIZE, see profiles/prefill_bf16_kernel_hybrid_batch_rank0.txt); other batches: not measured
MEASURED_TRAFFIC_DEFAULT_BATCH = 195328512
KV_CHUNK_MAX, KV_CHUNK_MIN = 32768, 512    # bounds of the split-K chunk of the keys a tile sees (fs_choose_prefill_chunk) ...
N_CU = 256                                 # compute units of an MI355X (the list is a host matter: no device query here)
N_SLOTS = 2 * N_CU                         # ... which is four thirds of the share of one of the workgroups the chip runs at a time


def prefill_workload(fs, n_req=64, n_ranks=7, rank=0, budget=8192, n_q_heads=64, n_kv_heads=8, seed=20251120,
                     median=8001, cap=123192, kv_chunk=None, queue=None):
    """Queue -> router -> Algorithm 1 -> hybrid placement -> rank's tile list (library calls only).
    ``queue``: the waiting prompts if already drawn (the draw is the synthetic input, not part of a step)."""
    if queue is None:
        from workloads import make_prefill_queue
        queue = make_prefill_queue(seed, n_req, median=median, sigma=0.9, cap=cap)
    prompt, n_done = queue["prompt_len"], queue["n_done"]
    R = n_ranks
    pending = np.zeros(R, dtype=np.int64)
    entries = np.zeros(n_req, dtype=fs.PREFILL_ENTRY_DTYPE)
    entries["req"] = np.arange(n_req)
    entries["n_done"] = n_done
    entries["n_new"] = prompt - n_done
    entries["rank"] = fs.fs_route_requests(pending, prompt - n_done)        # the waiting queue in arrival order
    take, load, n_tok = fs.fs_schedule_prefill(R, budget, budget // 2, entries)
    shape = fs.FsShape(n_req, n_q_heads, n_kv_heads, 128, 16, R)
    ctx = np.maximum(n_done + take, 1).astype(np.int32)
    owner, dp, rank_load, dp_load = fs.fs_build_placement_hybrid_heads(shape, ctx, layer=0, route=entries["rank"])
    G = n_q_heads // n_kv_heads
    tile = fs.fs_prefill_tile_tokens(G)
    if kv_chunk is None:      # an item about as long as a workgroup slot's share of the batch; a large batch is not cut at all
        kv_chunk, _ = fs.fs_choose_prefill_chunk(shape, n_done, take, owner, rank, tile, KV_CHUNK_MAX, KV_CHUNK_MIN,
                                                 N_SLOTS)
    items, pairs, sched, chunk_indptr, out_indptr = fs.fs_build_prefill_worklist(shape, n_done, take, owner, rank, tile,
                                                                                 kv_chunk)
    return dict(seed=seed, queue=queue, shape=shape, G=G, R=R, rank=rank, budget=budget, prompt=prompt, n_done=n_done,
                n_new=take.astype(np.int32), entries=entries, rank_token_load=load, n_tokens=n_tok, owner=owner,
                tile=tile, kv_chunk=kv_chunk, items=items, pairs=pairs, sched=sched, chunk_indptr=chunk_indptr,
                out_indptr=out_indptr)


def algorithmic_flops(pairs, G, d=128):
    """2 products x 2 flops x d per (query row, visible key): 4*d*G*sum over tokens of (n_done + i + 1)."""
    total = 0
    for p in pairs:
        L, N = int(p["n_done"]), int(p["n_new"])
        total += N * L + N * (N + 1) // 2
    return 4 * d * G * total


def run(args) -> int:
    import torch
    import paper_2511_14116_amd as fs
    from paper_2511_14116_amd.device import DeviceShare
    from workloads import make_kv_pool, make_prefill_q

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path to time", file=sys.stderr)
        return 2
    if not os.path.exists(fs.library_path()):
        from paper_2511_14116_amd.build import build
        build(verbose=False)
    fs.load_library()
    if args.prefill_waves:
        fs.fs_set_option("prefill_waves", args.prefill_waves)
    if args.prefill_col_tiles:
        fs.fs_set_option("prefill_col_tiles", args.prefill_col_tiles)
    v_range = fs.FS_V_ANY if args.prefill_wide_v else fs.FS_V_FP16_RANGE     # the batch's V is N(0,1): exact in fp16
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()

    wl = dict(rank=args.rank, kv_chunk=args.chunk, budget=args.prefill_budget, n_req=args.prefill_queue)
    w = prefill_workload(fs, **wl)
    kv_chunk = w["kv_chunk"]
    shape, G, pairs, items = w["shape"], w["G"], w["pairs"], w["items"]
    if len(items) == 0:
        print("bench.py: this rank's prefill share is empty", file=sys.stderr)
        return 2
    ctx = (w["n_done"] + w["n_new"]).astype(np.int32)
    kv_dtype = args.kv_dtype or "bf16"
    kv = make_kv_pool(w["seed"], np.stack([pairs["req"], pairs["kv_head"]], axis=1), ctx, kv_dtype=kv_dtype)
    q_indptr = np.concatenate([[0], np.cumsum(w["n_new"])]).astype(np.int64)
    q = make_prefill_q(w["seed"], int(q_indptr[-1]), shape.n_q_heads, 128)
    ds = DeviceShare(shape, q, kv, 1.0 / np.sqrt(128.0), v_range=v_range)
    ds.set_prefill_worklist(items, w["sched"], w["chunk_indptr"], w["tile"])
    flops = algorithmic_flops(pairs, G)
    rows = int(sum(int(p["n_new"]) for p in pairs)) * G
    kv_tokens = int(sum(int(p["n_done"]) + int(p["n_new"]) for p in pairs))

    host_us = []
    # The step's list is built by the library straight into pinned memory (items | sched | chunk_indptr in one
    # blob, three blobs in rotation).  By default the kernels read it in place and are launched eagerly (a blob is
    # reused only once the kernels that read it are done); --list device --graph uploads it as one copy and replays
    # upload, attention and merge as one HIP graph.
    n_cap, t_cap, p_cap = len(items), len(w["chunk_indptr"]) - 1, len(pairs)

    def up(x):
        return (x + 255) & ~255
    off_sched = up(n_cap * 32)
    off_indptr = up(off_sched + n_cap * 4)
    off_out_indptr = up(off_indptr + (t_cap + 1) * 8)
    blob_bytes = up(off_out_indptr + (p_cap + 1) * 8)
    dev_blob = torch.empty(blob_bytes, dtype=torch.uint8, device=dev)
    N_STAGE = 3
    n_done_buf = np.ascontiguousarray(w["n_done"], dtype=np.int32)
    n_new_buf = np.zeros(len(n_done_buf), dtype=np.int32)
    owner_buf = np.zeros((shape.n_req, shape.n_kv_heads), dtype=np.int32)
    staging = []
    for _ in range(N_STAGE):
        hb = torch.zeros(blob_bytes, dtype=torch.uint8, pin_memory=True)
        a = hb.numpy()
        views = dict(items=a[:n_cap * 32].view(fs.PREFILL_ITEM_DTYPE), sched=a[off_sched:off_sched + n_cap * 4].view(np.int32),
                     indptr=a[off_indptr:off_indptr + (t_cap + 1) * 8].view(np.int64),
                     pairs=np.empty(p_cap, dtype=fs.PREFILL_PAIR_DTYPE),
                     out_indptr=a[off_out_indptr:off_out_indptr + (p_cap + 1) * 8].view(np.int64))
        call = fs.bind_build_prefill_worklist(shape, n_done_buf, n_new_buf, owner_buf, args.rank, w["tile"], kv_chunk,
                                              views["items"], views["pairs"], views["sched"], views["indptr"],
                                              views["out_indptr"])
        staging.append(dict(host=hb, build=call))
    call_chunk = fs.bind_choose_prefill_chunk(shape, n_done_buf, n_new_buf, owner_buf, args.rank, w["tile"], KV_CHUNK_MAX,
                                              KV_CHUNK_MIN, N_SLOTS)
    n_step = [0]
    in_place = args.list == "host"
    use_graph = args.graph and not in_place
    base = dev_blob.data_ptr()
    R = w["R"]
    entries = w["entries"].copy()
    work = (w["prompt"] - w["n_done"]).astype(np.int64)

    # the host calls of a step, marshalled once (a serving loop calls them on the same buffers every step)
    pending_buf = np.zeros(R, dtype=np.int64)
    rank_buf = np.zeros(len(work), dtype=np.int32)
    load_buf = np.zeros(R, dtype=np.int64)
    ctx_buf = np.zeros(len(n_done_buf), dtype=np.int32)
    dp_buf = np.zeros((shape.n_req, shape.n_kv_heads), dtype=np.int32)
    rank_load_buf, dp_load_buf = np.zeros(R, dtype=np.int64), np.zeros(R, dtype=np.int64)
    call_route = fs.bind_route_requests(pending_buf, work, rank_buf)
    call_sched = fs.bind_schedule_prefill(R, args.prefill_budget, args.prefill_budget // 2, entries, n_new_buf, load_buf)
    call_place = fs.bind_build_placement_hybrid_heads(shape, ctx_buf, owner_buf, dp_buf, rank_load_buf, dp_load_buf, layer=0,
                                                      route=rank_buf)

    def step(ev=None):
        t0 = time.perf_counter()
        # host side of the step (library calls): router, Algorithm 1, head-level placement, rank's tile list
        pending_buf.fill(0)
        call_route()
        entries["rank"] = rank_buf
        t1 = time.perf_counter()
        call_sched()                             # the batch: tokens taken from every entry, straight into n_new_buf
        t2 = time.perf_counter()
        np.add(n_done_buf, n_new_buf, out=ctx_buf)
        np.maximum(ctx_buf, 1, out=ctx_buf)
        rank_load_buf.fill(0)
        dp_load_buf.fill(0)
        call_place()                             # owner map into owner_buf
        t3 = time.perf_counter()
        st = staging[n_step[0] % N_STAGE]
        n_step[0] += 1
        st["done"].synchronize()                 # the upload that last read this blob is done
        t4 = time.perf_counter()
        if args.chunk is None:                   # the split-K chunk is part of the step's host work (same batch, same choice)
            call_chunk()
            if call_chunk.n_tiles.value != kv_chunk:
                raise RuntimeError("the step's batch changed under the benchmark")
        st["build"]()
        n_it, n_ti = st["build"].n_items.value, st["build"].n_tiles.value
        t5 = time.perf_counter()
        if ev is None and st["graph"] is not None and (n_it, n_ti) == st["counts"]:
            st["graph"].replay()                 # upload, attention, merge: one launch
            st["done"].record(stream)
        else:
            enqueue(st, n_it, n_ti, stream, ev)
        t6 = time.perf_counter()
        host_us.append([(b - a) * 1e6 for a, b in ((t0, t6), (t0, t1), (t1, t2), (t2, t3), (t3, t4), (t4, t5), (t5, t6))])

    def enqueue(st, n_it, n_ti, on, ev=None):
        sp = on.cuda_stream
        if in_place:              # the kernels read the list where the host built it (pinned, mapped into the GPU's address space)
            b = st["host"].data_ptr()
        else:
            b = base
            dev_blob.copy_(st["host"], non_blocking=True)
            st["done"].record(on)
        if ev is not None:
            ev[0].record(on)
        if ev is not None or args.two_calls:   # the two calls, so that the attention kernel can be timed on its own
            fs.fs_prefill_attention(ds.shape, ds.view, b, b + off_sched, n_it,
                                    ds.prefill_tile_tokens, ds.prefill_part_o, ds.prefill_part_lse, sp)
            if ev is not None:
                ev[1].record(on)
            fs.fs_merge_lse(ds.prefill_part_o, ds.prefill_part_lse, b + off_indptr, n_ti,
                            ds.prefill_tile_rows, 128, ds.prefill_out, ds.prefill_lse, sp)
            if ev is not None:
                ev[2].record(on)
        else:                                  # one call: tiles of one chunk are final from the kernel, the rest is merged
            fs.fs_prefill_attention_fused(ds.shape, ds.view, b, b + off_sched, n_it, ds.prefill_tile_tokens, b + off_indptr,
                                          n_ti, b + off_out_indptr, ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_out,
                                          ds.prefill_lse, sp)
        if in_place:
            st["done"].record(on)     # the blob is free again once the kernels that read it are done

    for st in staging:
        st["done"] = torch.cuda.Event()
        st["done"].record(stream)
        st["graph"], st["counts"] = None, None
    for _ in range(max(args.warmup, N_STAGE)):
        step()
    torch.cuda.synchronize()
    # The GPU side of a step - upload of the blob, attention, merge - as one HIP graph per staging blob (the list's
    # sizes are launch arguments, so a step whose list has other sizes than the captured one is launched eagerly).
    if use_graph:
        cap_stream = torch.cuda.Stream()
        for st in staging:
            counts = (st["build"].n_items.value, st["build"].n_tiles.value)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=cap_stream):
                dev_blob.copy_(st["host"], non_blocking=True)
                sp = cap_stream.cuda_stream
                fs.fs_prefill_attention_fused(ds.shape, ds.view, base, base + off_sched, counts[0], ds.prefill_tile_tokens,
                                              base + off_indptr, counts[1], base + off_out_indptr, ds.prefill_part_o,
                                              ds.prefill_part_lse, ds.prefill_out, ds.prefill_lse, sp)
            st["graph"], st["counts"] = g, counts
        torch.cuda.synchronize()
        for _ in range(N_STAGE):
            step()
        torch.cuda.synchronize()
    host_us.clear()
    EVENT_EVERY = 8          # every 8th step runs eagerly with HIP events around the kernels
    timed = [i for i in range(args.steps) if i % EVENT_EVERY == 0]
    events = {i: [torch.cuda.Event(enable_timing=True) for _ in range(3)] for i in timed}
    torch.cuda.synchronize()
    gc.collect()
    gc.disable()             # as timeit does: a full collection in the middle of the loop is a 40 ms stall
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events.get(i))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    gc.enable()
    ms_per_step = wall * 1e3 / args.steps
    k_ms = np.array([e[0].elapsed_time(e[1]) for e in events.values()])
    m_ms = np.array([e[1].elapsed_time(e[2]) for e in events.values()])
    # The roofline's kernel time: the attention kernel launched back to back on the last step's list, one pair of
    # events around the lot (a single launch between its own events on an idle stream also counts the launch itself).
    st = staging[(n_step[0] - 1) % N_STAGE]
    b = st["host"].data_ptr() if in_place else base
    n_it = st["build"].n_items.value
    n_back = 30 if flops < 5e11 else 10
    back = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    back[0].record(stream)
    for _ in range(n_back):
        fs.fs_prefill_attention(ds.shape, ds.view, b, b + off_sched, n_it, ds.prefill_tile_tokens, ds.prefill_part_o,
                                ds.prefill_part_lse, stream.cuda_stream)
    back[1].record(stream)
    torch.cuda.synchronize()
    k_avg = back[0].elapsed_time(back[1]) / n_back
    enqueue(st, n_it, st["build"].n_tiles.value, stream)      # leave the outputs as the step's own calls leave them
    torch.cuda.synchronize()

    out = ds.prefill_out.cpu().numpy()
    lse = ds.prefill_lse.cpu().numpy()
    if not (np.isfinite(out).all() and np.isfinite(lse).all()):
        print("bench.py: non-finite prefill output", file=sys.stderr)
        return 1

    # ---- CPU baseline: the oracle on a bounded sample of (pair, token) rows ------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle                    # only this leg touches the oracle
        rng = np.random.default_rng(1)
        prs = oracle.PREFILL_PAIR_FIELDS
        pr_rows = np.stack([pairs[n] for n in prs], axis=1)
        budget_flops, done_flops, n_rows, ok = 2e11, 0, 0, True
        t0 = time.perf_counter()
        while done_flops < budget_flops and time.perf_counter() - t0 < 20:
            p = int(rng.integers(0, len(pairs)))
            tok = int(rng.integers(0, int(pairs[p]["n_new"])))
            o, l = oracle.prefill_attention_row(q, q_indptr, kv, pr_rows, shape.n_q_heads, G, 1.0 / np.sqrt(128.0), p, tok)
            row = int(w["out_indptr"][p]) + tok * G
            ok &= bool((np.abs(out[row:row + G] - o) <= 2e-3 + 1e-2 * np.abs(o)).all() and
                       (np.abs(lse[row:row + G] - l) <= 1e-3).all())
            done_flops += 4 * 128 * G * (int(pairs[p]["n_done"]) + tok + 1)
            n_rows += 1
        dt = time.perf_counter() - t0
        cpu = {"value": round(done_flops / dt / 1e12, 6), "unit": "TFLOP/s", "cores": len(os.sched_getaffinity(0)),
               "kind": "oracle", "sample": f"{n_rows} random (pair, token) rows of rank {args.rank}'s share, fp64 numpy, {dt:.1f} s",
               "gpu_matches_oracle_on_sample": ok}
        if not ok:
            print("bench.py: GPU prefill output disagrees with the oracle on the sample", file=sys.stderr)
            return 1

    res = {
        "metric": "chunked-prefill attention TFLOP/s (% of bf16 MFMA peak) and query-token-heads/s, rank-0 share, 1 MI355X",
        "value": round(flops / (ms_per_step * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": ("bf16" if kv_dtype == "bf16" else "fp8_e4m3 K/V, products in bf16") + (" (second product in fp16)" if not args.prefill_wide_v else ""), "data": "synthetic",
        "config": {"workload": f"prefill batch: {args.prefill_queue} waiting prompts (lognormal median 8001, cap 123192), budget {args.prefill_budget} tokens, "
                               f"Hq=64, Hkv=8, d=128, page=16, R=7 head-level hybrid, rank {args.rank}, seed={w['seed']}"
                               + (f", K/V held as {kv_dtype}" if kv_dtype != "bf16" else ""),
                   "n_pairs": len(pairs), "n_tiles": ds.n_prefill_tiles, "n_items": len(items), "tile_tokens": w["tile"],
                   "kv_chunk_tokens": kv_chunk, "batch_tokens": int(w["n_tokens"]),
                   "query_rows": rows, "kv_tokens_of_pairs": kv_tokens, "flops": flops,
                   "prefill_waves": fs.fs_get_option("prefill_waves"), "prefill_col_tiles": fs.fs_get_option("prefill_col_tiles"),
                   "second_product": "bf16 V, weights bf16 hi+lo (v_range FS_V_ANY)" if args.prefill_wide_v else "fp16 V and weights (v_range FS_V_FP16_RANGE)",
                   "work_list": "read in place from pinned host memory" if in_place else "uploaded every step",
                   "step_calls": "fs_prefill_attention + fs_merge_lse" if args.two_calls else "fs_prefill_attention_fused",
                   "single_chunk_tiles": int((np.diff(w["chunk_indptr"]) == 1).sum()),
                   "launch": f"hip graph per staging blob (upload, attention, merge); every {EVENT_EVERY}th step eager with events" if use_graph
                             else f"eager; every {EVENT_EVERY}th step with events around the kernels"},
        "kernel_ms": {"prefill_avg": round(k_avg, 5), "prefill_avg_is": f"{n_back} launches back to back between one pair of HIP events",
                      "prefill_each_avg": round(float(k_ms.mean()), 5), "prefill_p10": round(float(np.percentile(k_ms, 10)), 5),
                      "prefill_p90": round(float(np.percentile(k_ms, 90)), 5), "merge_avg": round(float(m_ms.mean()), 5)},
        "host_us_per_step": dict(zip(("all", "router", "scheduler", "placement", "wait_for_staging", "tile_list", "upload_enqueue"),
                                     (round(float(v), 1) for v in np.mean(np.array(host_us), axis=0)))),
        "query_token_heads_per_s": round(rows / G / (ms_per_step * 1e-3), 1),
        "roofline": {"bound": "mfma", "kernel": "prefill_bf16_kernel" if kv_dtype == "bf16" else "prefill_fp8_kernel", "achieved": round(flops / (k_avg * 1e-3) / 1e12, 2),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (k_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "algorithmic_flops_per_launch": flops,
                     "traffic": MEASURED_TRAFFIC_DEFAULT_BATCH if (args.prefill_queue, args.prefill_budget, args.rank, kv_chunk)
                     == (64, 8192, 0, 2272) and fs.fs_get_option("prefill_waves") == 8
                     and fs.fs_get_option("prefill_col_tiles") == 1 and kv_dtype == "bf16" else None},
    }
    if cpu is not None:
        res["cpu_baseline"] = cpu
    print(json.dumps(res))
    return 0
