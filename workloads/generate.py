"""Seeded generators for the five synthetic decode batches.

The paper measures on a production trace sample and a reasoning dataset
(Section 4, Tables 1 and 2); neither is reproduced here.  These generators draw
stand-ins with the published length character (a median of a few thousand
tokens and a heavy tail beyond 1e5) from closed-form distributions.

Everything here is input preparation: random draws, rounding to the storage
formats, and laying pages out in a pool whose slot order is a seeded
permutation.  Which rank owns which head, what the work list looks like and
what attention computes are decided elsewhere and arrive here, where needed,
as plain arguments (``pairs``).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor

import numpy as np

BASE_SEED = 20251114

MODE_TP = 0
MODE_DP = 1

# One entry per synthetic batch.  "lengths" names the draw in _draw_lengths.
CONFIGS = {
    0: dict(name="tiny-all-tp", n_req=16, n_q_heads=32, n_kv_heads=8, head_dim=128,
            page_tokens=16, n_ranks=7, kv_dtype="bf16", lengths=("uniform", 64, 512),
            dp=("fraction", 0.0), chunk_tokens=0),
    1: dict(name="8b-hybrid", n_req=256, n_q_heads=32, n_kv_heads=8, head_dim=128,
            page_tokens=16, n_ranks=7, kv_dtype="bf16", lengths=("lognormal", 2048, 0.8, 8192),
            dp=("fraction", 0.25), chunk_tokens=2048, chunk_adaptive=True),
    2: dict(name="70b-gqa", n_req=512, n_q_heads=64, n_kv_heads=8, head_dim=128,
            page_tokens=16, n_ranks=6, kv_dtype="bf16", lengths=("lognormal", 4096, 0.7, 32768),
            dp=("fraction", 0.20), chunk_tokens=2048),
    3: dict(name="long-context-skew", n_req=64, n_q_heads=32, n_kv_heads=8, head_dim=128,
            page_tokens=16, n_ranks=5, kv_dtype="bf16", lengths=("pareto", 1.2, 512, 131072),
            dp=("shorter_than", 16384), chunk_tokens=2048, chunk_adaptive=True),
    4: dict(name="mha-fp8", n_req=1024, n_q_heads=32, n_kv_heads=32, head_dim=128,
            page_tokens=16, n_ranks=7, kv_dtype="fp8", lengths=("uniform", 512, 2048),
            dp=("fraction", 0.0), chunk_tokens=0),
}


def _draw_lengths(rng: np.random.Generator, spec, n: int) -> np.ndarray:
    kind = spec[0]
    if kind == "uniform":
        return rng.integers(spec[1], spec[2], size=n, endpoint=True).astype(np.int32)
    if kind == "lognormal":
        median, sigma, cap = spec[1], spec[2], spec[3]
        x = np.exp(rng.normal(np.log(median), sigma, size=n))
        return np.clip(np.rint(x), 1, cap).astype(np.int32)
    if kind == "pareto":
        alpha, lo, cap = spec[1], spec[2], spec[3]
        u = 1.0 - rng.random(size=n)            # (0, 1]
        x = np.floor(lo * u ** (-1.0 / alpha))
        return np.minimum(x, cap).astype(np.int32)
    raise ValueError(kind)


def make_requests(cfg_id: int, seed: int | None = None, n_req: int | None = None,
                  max_len: int | None = None, force_first_len: int | None = None) -> dict:
    """Draw one batch: context lengths and the TP/DP mode of each request.

    ``n_req`` and ``max_len`` shrink a config for tests; ``force_first_len``
    overrides request 0's length (the forced-tail variant of the skew batch).
    """
    cfg = dict(CONFIGS[cfg_id])
    seed = BASE_SEED + cfg_id if seed is None else seed
    rng = np.random.Generator(np.random.PCG64(seed))
    n = cfg["n_req"] if n_req is None else n_req
    ctx = _draw_lengths(rng, cfg["lengths"], n)
    if max_len is not None:
        ctx = np.minimum(ctx, max_len).astype(np.int32)
    if force_first_len is not None:
        ctx[0] = force_first_len
    mode = np.zeros(n, dtype=np.uint8)
    if cfg["dp"][0] == "fraction":
        n_dp = int(round(cfg["dp"][1] * n))
        perm = rng.permutation(n)
        mode[perm[:n_dp]] = MODE_DP
    else:  # "shorter_than": long requests stay tensor-parallel
        mode[ctx < cfg["dp"][1]] = MODE_DP
    cfg.update(cfg_id=cfg_id, seed=seed, n_req=n, ctx_len=ctx, mode=mode,
               group=cfg["n_q_heads"] // cfg["n_kv_heads"],
               sm_scale=1.0 / float(np.sqrt(cfg["head_dim"])))
    return cfg


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def make_q(seed: int, n_req: int, n_q_heads: int, head_dim: int) -> np.ndarray:
    """Query rows [n_req][n_q_heads][head_dim] as bf16 bit patterns, N(0,1)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 11])))
    return f32_to_bf16_bits(rng.standard_normal((n_req, n_q_heads, head_dim), dtype=np.float32))


def _f32_to_e4m3_bytes(y: np.ndarray) -> np.ndarray:
    """fp32 -> fp8 e4m3fn bytes, nearest-even, saturating at +-448."""
    import torch
    t = torch.from_numpy(np.clip(y, -448.0, 448.0).astype(np.float32))
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy()


BF16_NAN_BITS = np.uint16(0x7FFF)
FP8_NAN_BYTE = np.uint8(0x7F)


def make_kv_pool(seed: int, pairs: np.ndarray, ctx_len: np.ndarray, head_dim: int = 128,
                 page_tokens: int = 16, kv_dtype: str = "bf16", spare_slots: int = 3,
                 poison: bool = True, threads: int = 8) -> dict:
    """Paged K/V for the given (request, kv_head) pairs, in the order given.

    Each pair's K and V rows depend only on (seed, request, head), so the same
    pair holds the same numbers whichever rank's list it appears in.  A slot is
    one (page, kv head): ``page_tokens x head_dim`` elements in token-major
    order, once for K and once for V.  Slot numbers are a seeded permutation of
    the pool; ``spare_slots`` unused slots, and the unused tail of every last
    page, hold NaN patterns when ``poison`` is set so that a stray read shows.

    Returns k_pool/v_pool [n_slots][page_tokens][head_dim] (uint16 bf16 bits or
    uint8 e4m3 bytes), k_scale/v_scale [n_slots] fp32 (fp8 only, else None),
    page_indptr int64 [n_pairs+1] and page_ids int32 [total pages].
    """
    pairs = np.asarray(pairs, dtype=np.int64).reshape(-1, 2)
    n_pairs = len(pairs)
    lens = ctx_len[pairs[:, 0]].astype(np.int64) if n_pairs else np.zeros(0, np.int64)
    n_pages = (lens + page_tokens - 1) // page_tokens
    page_indptr = np.zeros(n_pairs + 1, dtype=np.int64)
    np.cumsum(n_pages, out=page_indptr[1:])
    total = int(page_indptr[-1])
    n_slots = total + spare_slots
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 13])))
    page_ids = rng.permutation(n_slots)[:total].astype(np.int32)

    fp8 = kv_dtype == "fp8"
    elt = np.uint8 if fp8 else np.uint16
    fill = FP8_NAN_BYTE if fp8 else BF16_NAN_BITS
    shape = (n_slots, page_tokens, head_dim)
    if poison:
        k_pool = np.full(shape, fill, dtype=elt)
        v_pool = np.full(shape, fill, dtype=elt)
    else:
        k_pool = np.zeros(shape, dtype=elt)
        v_pool = np.zeros(shape, dtype=elt)
    k_scale = v_scale = None
    if fp8:
        k_scale = np.full(n_slots, np.nan if poison else 1.0, dtype=np.float32)
        v_scale = np.full(n_slots, np.nan if poison else 1.0, dtype=np.float32)

    def fill_pair(p: int) -> None:
        r, h = int(pairs[p, 0]), int(pairs[p, 1])
        L, npg = int(lens[p]), int(n_pages[p])
        slots = page_ids[page_indptr[p]:page_indptr[p + 1]]
        prng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 17, r, h])))
        for pool, scale in ((k_pool, k_scale), (v_pool, v_scale)):
            x = np.zeros((npg * page_tokens, head_dim), dtype=np.float32)
            x[:L] = prng.standard_normal((L, head_dim), dtype=np.float32)
            x = x.reshape(npg, page_tokens, head_dim)
            if fp8:
                amax = np.abs(x).max(axis=(1, 2))          # padding rows are zero
                s = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
                enc = _f32_to_e4m3_bytes(x / s[:, None, None])
                scale[slots] = s
            else:
                enc = f32_to_bf16_bits(x)
            if poison and L % page_tokens:
                enc[-1, L % page_tokens:, :] = fill
            pool[slots] = enc

    if n_pairs:
        if threads > 1 and n_pairs > 1:
            with ThreadPoolExecutor(max_workers=threads) as ex:
                list(ex.map(fill_pair, range(n_pairs)))
        else:
            for p in range(n_pairs):
                fill_pair(p)

    return dict(k_pool=k_pool, v_pool=v_pool, k_scale=k_scale, v_scale=v_scale,
                page_indptr=page_indptr, page_ids=page_ids, n_slots=n_slots,
                kv_dtype=kv_dtype, head_dim=head_dim, page_tokens=page_tokens)


def make_prefill_queue(seed: int, n_req: int, median: int = 8001, sigma: float = 0.9, cap: int = 123192,
                       progress: float = 0.5) -> dict:
    """Waiting prompts for a prefill batch: prompt length per request (lognormal with the median
    and cap of the paper's online trace, Table 2) and how many of its tokens are already
    processed (a multiple of 16; a fraction ``progress`` of the requests has made some progress).
    Routing and batch forming are not done here."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 23])))
    prompt = np.clip(np.rint(np.exp(rng.normal(np.log(median), sigma, size=n_req))), 1, cap).astype(np.int32)
    started = rng.random(n_req) < progress
    done = np.where(started, (rng.random(n_req) * prompt).astype(np.int64) // 16 * 16, 0).astype(np.int32)
    done = np.minimum(done, prompt - 1).astype(np.int32) // 16 * 16
    return dict(seed=seed, prompt_len=prompt, n_done=done.astype(np.int32))


def make_prefill_q(seed: int, n_tokens: int, n_q_heads: int, head_dim: int) -> np.ndarray:
    """Query rows of a prefill batch [n_tokens][n_q_heads][head_dim] as bf16 bit patterns, N(0,1)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 29])))
    return f32_to_bf16_bits(rng.standard_normal((n_tokens, n_q_heads, head_dim), dtype=np.float32))
