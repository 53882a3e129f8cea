"""The C++ router and prefill scheduler against the oracle, value for value (no GPU needed)."""
import json
import os
import time

import numpy as np
import pytest

import paper_2511_14116_amd as fs
from oracle.scheduler import adaptive_chunked_prefill, route_request

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        from paper_2511_14116_amd.build import build
        build(verbose=False)
    return fs.load_library()


def test_fig4_through_the_library():
    with open(os.path.join(GOLD, "fig4_router_scheduler.json")) as f:
        g = json.load(f)
    R = g["n_ranks"]
    pending = np.zeros(R, dtype=np.int64)
    for _req, gpu, toks in g["queued"]:
        pending[gpu] += toks
    gpu3 = fs.fs_route_request(pending, g["new_request_tokens"])
    assert gpu3 == g["load_aware_gpu_of_request_3"] and pending.tolist() == [4, 2, 1]
    entries = [(req, gpu, 0, toks) for req, gpu, toks in g["queued"]] + [(3, gpu3, 0, 1)]
    take, load, n = fs.fs_schedule_prefill(R, g["budget"], (g["budget"] + 1) // 2, entries)
    assert take.tolist() == g["adaptive_batch_tokens_per_request"] and n == 3 and load.tolist() == [1, 1, 1]


@pytest.mark.parametrize("seed", range(60))
def test_scheduler_matches_oracle_on_random_queues(seed):
    rng = np.random.default_rng(1000 + seed)
    R = int(rng.integers(1, 9))
    n = int(rng.integers(0, 14))
    entries = [(i, int(rng.integers(0, R)), int(rng.integers(0, 3000)), int(rng.integers(0, 40))) for i in range(n)]
    budget = int(rng.integers(0, 150))
    min_tokens = int(rng.integers(0, budget + 3))
    init = None if seed % 2 else [int(x) for x in rng.integers(0, 5000, size=R)]
    want = adaptive_chunked_prefill(budget, R, entries, min_tokens, init)
    take, load, n_tok = fs.fs_schedule_prefill(R, budget, min_tokens, entries, init)
    assert take.tolist() == want[0] and load.tolist() == list(want[1]) and n_tok == want[2]


@pytest.mark.parametrize("seed", range(40))
def test_scheduler_search_forms_agree_with_the_oracle(seed):
    """Up to 8 ranks with modest loads the library searches packed (load, rank) keys; more ranks or loads
    near 2^59 take the linear search.  Both against the oracle, on queues full of equal loads (ties go to the
    lowest rank) and of ranks that run dry.  A negative starting load is an error on both sides."""
    rng = np.random.default_rng(7000 + seed)
    kind = seed % 4
    R = int(rng.integers(9, 21)) if kind == 0 else int(rng.integers(1, 9))
    n = int(rng.integers(1, 20))
    entries = [(i, int(rng.integers(0, R)), int(rng.choice([0, 0, 7, 512])), int(rng.integers(0, 12))) for i in range(n)]
    budget = int(rng.integers(1, 120))
    min_tokens = int(rng.integers(0, budget + 1))
    init = None
    if kind == 1:
        init = [int(x) for x in rng.integers(0, 50, size=R)]
        bad = list(init); bad[int(rng.integers(0, R))] = -1 - int(rng.integers(0, 40))
        with pytest.raises(ValueError):
            adaptive_chunked_prefill(budget, R, entries, min_tokens, bad)
        with pytest.raises(fs.FsError):
            fs.fs_schedule_prefill(R, budget, min_tokens, entries, bad)
    elif kind == 2:
        init = [int(x) for x in (1 << 59) + rng.integers(0, 3, size=R)]   # no room for the rank bits: linear search
    elif kind == 3:
        init = [int(x) for x in rng.integers(0, 2, size=R)]               # packed keys, nearly all equal
    want = adaptive_chunked_prefill(budget, R, entries, min_tokens, init)
    take, load, n_tok = fs.fs_schedule_prefill(R, budget, min_tokens, entries, init)
    assert take.tolist() == want[0] and load.tolist() == list(want[1]) and n_tok == want[2]


def test_router_matches_oracle():
    rng = np.random.default_rng(5)
    for R in (1, 3, 7):
        a = np.zeros(R, dtype=np.int64)
        b = [0] * R
        for w in rng.integers(0, 10000, size=300):
            assert fs.fs_route_request(a, int(w)) == route_request(b, int(w))
        assert a.tolist() == b


def test_queue_router_matches_oracle_and_single_calls():
    rng = np.random.default_rng(6)
    for R in (1, 2, 7):
        work = rng.integers(0, 10000, size=257)
        work[::9] = 0                                   # zero-work requests still take the lowest least-loaded rank
        start = rng.integers(0, 3000, size=R).astype(np.int64)
        a, b, c = start.copy(), [int(x) for x in start], start.copy()
        ranks = fs.fs_route_requests(a, work)
        assert ranks.dtype == np.int32
        assert ranks.tolist() == [route_request(b, int(w)) for w in work]
        assert ranks.tolist() == [fs.fs_route_request(c, int(w)) for w in work]
        assert a.tolist() == b == c.tolist()
    assert len(fs.fs_route_requests(np.zeros(3, dtype=np.int64), [])) == 0
    keep = np.array([5, 1, 9], dtype=np.int64)
    with pytest.raises(fs.FsError):
        fs.fs_route_requests(keep, [4, -1, 2])          # a negative work: nothing is placed
    assert keep.tolist() == [5, 1, 9]
    with pytest.raises(TypeError):
        fs.fs_route_requests([0, 0], [1])


def test_serving_sized_budget_is_fast_and_balanced():
    # 7 ranks, 64 waiting prompts shaped like the paper's online trace (mean ~13.5K tokens), budget 8192
    rng = np.random.default_rng(11)
    R = 7
    lens = np.clip(np.round(np.exp(rng.normal(np.log(8001), 0.9, size=64))), 1, 123192).astype(np.int64)
    pending = np.zeros(R, dtype=np.int64)
    entries = np.zeros(64, dtype=fs.PREFILL_ENTRY_DTYPE)
    for i, L in enumerate(lens):
        entries[i] = (i, fs.fs_route_request(pending, int(L)), 0, int(L))
    assert pending.max() - pending.min() <= lens.max()
    t0 = time.perf_counter()
    take, load, n = fs.fs_schedule_prefill(R, 8192, 4096, entries)
    dt = time.perf_counter() - t0
    assert n >= 4096 and take.sum() == n
    assert load.max() * R / load.sum() < 1.01          # a token budget spread evenly over the ranks
    assert dt < 0.05


def test_bound_router_and_scheduler_reuse_their_buffers():
    """The pre-marshalled forms (what a serving loop calls every step) give what the plain calls give, and see
    changed inputs on the next call."""
    rng = np.random.default_rng(31)
    R, n = 5, 40
    work = rng.integers(1, 9000, size=n).astype(np.int64)
    pending = np.zeros(R, dtype=np.int64); ranks = np.zeros(n, dtype=np.int32)
    route = fs.bind_route_requests(pending, work, ranks)
    entries = np.zeros(n, dtype=fs.PREFILL_ENTRY_DTYPE)
    entries["req"] = np.arange(n); entries["n_done"] = rng.integers(0, 3000, size=n); entries["n_new"] = work
    take = np.zeros(n, dtype=np.int32); load = np.zeros(R, dtype=np.int64)
    sched = fs.bind_schedule_prefill(R, 4096, 2048, entries, take, load)
    for rep in range(3):
        pending[:] = rep * 100
        want_pending = pending.copy()
        want_ranks = fs.fs_route_requests(want_pending, work)
        route()
        assert ranks.tobytes() == want_ranks.tobytes() and pending.tobytes() == want_pending.tobytes()
        entries["rank"] = ranks
        want_take, want_load, want_n = fs.fs_schedule_prefill(R, 4096, 2048, entries)
        sched()
        assert take.tobytes() == want_take.tobytes() and load.tobytes() == want_load.tobytes()
        assert sched.n_items.value == want_n == int(take.sum())
        work[rep] += 777; entries["n_new"][rep] = work[rep]          # the next call sees the change
    with pytest.raises(TypeError):
        fs.bind_route_requests(pending.astype(np.int32), work, ranks)
    with pytest.raises(TypeError):
        fs.bind_schedule_prefill(R, 4096, 2048, entries, take.astype(np.int64), load)


def test_errors():
    with pytest.raises(fs.FsError):
        fs.fs_schedule_prefill(0, 4, 0, [])
    with pytest.raises(fs.FsError):
        fs.fs_schedule_prefill(2, 4, 0, [(0, 2, 0, 1)])
    with pytest.raises(fs.FsError):
        fs.fs_schedule_prefill(2, -1, 0, [(0, 1, 0, 1)])
    with pytest.raises(fs.FsError):
        fs.fs_route_request(np.zeros(3, dtype=np.int64), -5)
    with pytest.raises(TypeError):
        fs.fs_route_request([0, 0], 1)
    take, load, n = fs.fs_schedule_prefill(3, 10, 5, [])
    assert len(take) == 0 and n == 0 and load.tolist() == [0, 0, 0]
