"""Benchmark of the chunked-prefill attention share (`python bench.py --path prefill`).

A step is: route the waiting prompts (load-aware router), form the batch (Algorithm 1), place
the heads (head-level hybrid attention), build rank 0's tile list - all on the host by the
library - upload the list, and run the attention kernel over the batch's chunks.  Q, the paged
K/V pool and the page table are resident in HBM.  Prints ONE JSON line; `roofline` is the
attention kernel against the dense bf16 matrix-core peak.
"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16, published
# HBM-side bytes of one prefill_bf16_kernel launch on the default batch (rocprofv3 --pmc FETCH_SIZE x 2.000 +
# WRITE_SIZE, see profiles/prefill_bf16_kernel_hybrid_batch_rank0.txt); other batches: not measured
MEASURED_TRAFFIC_DEFAULT_BATCH = 208407450
KV_CHUNK_DEFAULT = 2048            # split-K chunk of the keys a tile sees


def prefill_workload(fs, n_req=64, n_ranks=7, rank=0, budget=8192, n_q_heads=64, n_kv_heads=8, seed=20251120,
                     median=8001, cap=123192, kv_chunk=KV_CHUNK_DEFAULT, queue=None):
    """Queue -> router -> Algorithm 1 -> hybrid placement -> rank's tile list (library calls only).
    ``queue``: the waiting prompts if already drawn (the draw is the synthetic input, not part of a step)."""
    if queue is None:
        from workloads import make_prefill_queue
        queue = make_prefill_queue(seed, n_req, median=median, sigma=0.9, cap=cap)
    prompt, n_done = queue["prompt_len"], queue["n_done"]
    R = n_ranks
    t0 = time.perf_counter()
    pending = np.zeros(R, dtype=np.int64)
    entries = np.zeros(n_req, dtype=fs.PREFILL_ENTRY_DTYPE)
    entries["req"] = np.arange(n_req)
    entries["n_done"] = n_done
    entries["n_new"] = prompt - n_done
    entries["rank"] = fs.fs_route_requests(pending, prompt - n_done)        # the waiting queue in arrival order
    t1 = time.perf_counter()
    take, load, n_tok = fs.fs_schedule_prefill(R, budget, budget // 2, entries)
    t2 = time.perf_counter()
    shape = fs.FsShape(n_req, n_q_heads, n_kv_heads, 128, 16, R)
    ctx = np.maximum(n_done + take, 1).astype(np.int32)
    owner, dp, rank_load, dp_load = fs.fs_build_placement_hybrid_heads(shape, ctx, layer=0, route=entries["rank"])
    G = n_q_heads // n_kv_heads
    tile = fs.fs_prefill_tile_tokens(G)
    items, pairs, sched, chunk_indptr, out_indptr = fs.fs_build_prefill_worklist(shape, n_done, take, owner, rank, tile,
                                                                                 kv_chunk)
    t3 = time.perf_counter()
    return dict(seed=seed, queue=queue, shape=shape, G=G, R=R, rank=rank, budget=budget, prompt=prompt, n_done=n_done,
                n_new=take.astype(np.int32), entries=entries, rank_token_load=load, n_tokens=n_tok, owner=owner,
                tile=tile, kv_chunk=kv_chunk, items=items, pairs=pairs, sched=sched, chunk_indptr=chunk_indptr,
                out_indptr=out_indptr,
                host_us=dict(router=(t1 - t0) * 1e6, scheduler=(t2 - t1) * 1e6, placement_and_list=(t3 - t2) * 1e6))


def algorithmic_flops(pairs, G, d=128):
    """2 products x 2 flops x d per (query row, visible key): 4*d*G*sum over tokens of (n_done + i + 1)."""
    total = 0
    for p in pairs:
        L, N = int(p["n_done"]), int(p["n_new"])
        total += N * L + N * (N + 1) // 2
    return 4 * d * G * total


def run(args) -> int:
    import torch
    import oracle
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
    if args.prefill_wide_v:
        fs.fs_set_option("prefill_wide_v", 1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream()

    kv_chunk = KV_CHUNK_DEFAULT if args.chunk is None else args.chunk
    wl = dict(rank=args.rank, kv_chunk=kv_chunk, budget=args.prefill_budget, n_req=args.prefill_queue)
    w = prefill_workload(fs, **wl)
    shape, G, pairs, items = w["shape"], w["G"], w["pairs"], w["items"]
    if len(items) == 0:
        print("bench.py: this rank's prefill share is empty", file=sys.stderr)
        return 2
    ctx = (w["n_done"] + w["n_new"]).astype(np.int32)
    kv = make_kv_pool(w["seed"], np.stack([pairs["req"], pairs["kv_head"]], axis=1), ctx)
    q_indptr = np.concatenate([[0], np.cumsum(w["n_new"])]).astype(np.int64)
    q = make_prefill_q(w["seed"], int(q_indptr[-1]), shape.n_q_heads, 128)
    ds = DeviceShare(shape, q, kv, 1.0 / np.sqrt(128.0))
    ds.set_prefill_worklist(items, w["sched"], w["chunk_indptr"], w["tile"])
    flops = algorithmic_flops(pairs, G)
    rows = int(sum(int(p["n_new"]) for p in pairs)) * G
    kv_tokens = int(sum(int(p["n_done"]) + int(p["n_new"]) for p in pairs))

    host_us = []
    # The step's list goes to the GPU through pinned staging buffers (a copy from pageable memory would make the
    # host wait for it); three sets, and a set is reused only once the upload that read it is done.
    N_STAGE = 3
    staging = [dict(items=torch.empty((len(items), 8), dtype=torch.int32, pin_memory=True),
                    sched=torch.empty(len(items), dtype=torch.int32, pin_memory=True),
                    indptr=torch.empty(len(w["chunk_indptr"]), dtype=torch.int64, pin_memory=True),
                    done=None) for _ in range(N_STAGE)]
    n_step = [0]

    def step(ev=None):
        t0 = time.perf_counter()
        ww = prefill_workload(fs, queue=w["queue"], **wl)                # host side of the step (library calls)
        st = staging[n_step[0] % N_STAGE]
        n_step[0] += 1
        if st["done"] is not None:
            st["done"].synchronize()
        st["items"].numpy()[...] = ww["items"].view(np.int32).reshape(-1, 8)
        st["sched"].numpy()[...] = ww["sched"]
        st["indptr"].numpy()[...] = ww["chunk_indptr"]
        ds.prefill_items.copy_(st["items"], non_blocking=True)
        ds.prefill_sched.copy_(st["sched"], non_blocking=True)
        ds.prefill_chunk_indptr.copy_(st["indptr"], non_blocking=True)
        st["done"] = torch.cuda.Event()
        st["done"].record(stream)
        host_us.append((time.perf_counter() - t0) * 1e6)
        sp = stream.cuda_stream
        if ev is not None:
            ev[0].record(stream)
        fs.fs_prefill_attention(ds.shape, ds.view, ds.prefill_items, ds.prefill_sched, ds.n_prefill_items,
                                ds.prefill_tile_tokens, ds.prefill_part_o, ds.prefill_part_lse, sp)
        if ev is not None:
            ev[1].record(stream)
        fs.fs_merge_lse(ds.prefill_part_o, ds.prefill_part_lse, ds.prefill_chunk_indptr, ds.n_prefill_tiles,
                        ds.prefill_tile_rows, 128, ds.prefill_out, ds.prefill_lse, sp)
        if ev is not None:
            ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    host_us.clear()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    k_ms = np.array([e[0].elapsed_time(e[1]) for e in events])
    m_ms = np.array([e[1].elapsed_time(e[2]) for e in events])

    out = ds.prefill_out.cpu().numpy()
    lse = ds.prefill_lse.cpu().numpy()
    if not (np.isfinite(out).all() and np.isfinite(lse).all()):
        print("bench.py: non-finite prefill output", file=sys.stderr)
        return 1

    # ---- CPU baseline: the oracle on a bounded sample of (pair, token) rows ------------------------
    cpu = None
    if not args.no_cpu_baseline:
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

    k_avg = float(k_ms.mean())
    res = {
        "metric": "chunked-prefill attention TFLOP/s (% of bf16 MFMA peak) and query-token-heads/s, rank-0 share, 1 MI355X",
        "value": round(flops / (ms_per_step * 1e-3) / 1e12, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16 (second product in fp16)" if not fs.fs_get_option("prefill_wide_v") else "bf16", "data": "synthetic",
        "config": {"workload": f"prefill batch: {args.prefill_queue} waiting prompts (lognormal median 8001, cap 123192), budget {args.prefill_budget} tokens, "
                               f"Hq=64, Hkv=8, d=128, page=16, R=7 head-level hybrid, rank {args.rank}, seed={w['seed']}",
                   "n_pairs": len(pairs), "n_tiles": ds.n_prefill_tiles, "n_items": len(items), "tile_tokens": w["tile"],
                   "kv_chunk_tokens": kv_chunk, "batch_tokens": int(w["n_tokens"]),
                   "query_rows": rows, "kv_tokens_of_pairs": kv_tokens, "flops": flops,
                   "prefill_waves": fs.fs_get_option("prefill_waves"), "prefill_col_tiles": fs.fs_get_option("prefill_col_tiles"),
                   "second_product": "bf16 V, weights bf16 hi+lo" if fs.fs_get_option("prefill_wide_v") else "fp16 V and weights"},
        "kernel_ms": {"prefill_avg": round(k_avg, 5), "prefill_p10": round(float(np.percentile(k_ms, 10)), 5),
                      "prefill_p90": round(float(np.percentile(k_ms, 90)), 5), "merge_avg": round(float(m_ms.mean()), 5)},
        "host_us_per_step": {"all_avg": round(float(np.mean(host_us)), 1), **{k: round(v, 1) for k, v in w["host_us"].items()}},
        "query_token_heads_per_s": round(rows / G / (ms_per_step * 1e-3), 1),
        "roofline": {"bound": "mfma", "kernel": "prefill_bf16_kernel", "achieved": round(flops / (k_avg * 1e-3) / 1e12, 2),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (k_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                     "algorithmic_flops_per_launch": flops,
                     "traffic": MEASURED_TRAFFIC_DEFAULT_BATCH if (args.prefill_queue, args.prefill_budget, args.rank, kv_chunk)
                     == (64, 8192, 0, KV_CHUNK_DEFAULT) and fs.fs_get_option("prefill_waves") == 8
                     and fs.fs_get_option("prefill_col_tiles") == 1 else None},
    }
    if cpu is not None:
        res["cpu_baseline"] = cpu
    print(json.dumps(res))
    return 0
