"""The synthetic input generators: determinism, encodings, poison, shapes."""
import numpy as np
import torch

from oracle import E4M3_TABLE
from workloads import CONFIGS, BASE_SEED, make_requests, make_q, make_kv_pool, f32_to_bf16_bits


def test_bf16_rounding_matches_library_nearest_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 3,
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 65504.0], dtype=np.float32)])
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(f32_to_bf16_bits(x), lib)


def test_requests_follow_the_recipe():
    for cid, cfg in CONFIGS.items():
        w = make_requests(cid)
        assert w["seed"] == BASE_SEED + cid and len(w["ctx_len"]) == cfg["n_req"]
        assert w["ctx_len"].min() >= 1
        again = make_requests(cid)
        assert np.array_equal(w["ctx_len"], again["ctx_len"]) and np.array_equal(w["mode"], again["mode"])
    w0 = make_requests(0); assert w0["ctx_len"].min() >= 64 and w0["ctx_len"].max() <= 512 and w0["mode"].sum() == 0
    w1 = make_requests(1); assert w1["mode"].sum() == 64 and w1["ctx_len"].max() <= 8192
    w2 = make_requests(2); assert w2["mode"].sum() == 102 and w2["ctx_len"].max() <= 32768 and w2["group"] == 8
    assert 3000 < np.median(w2["ctx_len"]) < 5500
    w3 = make_requests(3); assert w3["ctx_len"].min() >= 512 and w3["ctx_len"].max() <= 131072
    assert np.array_equal(w3["mode"] == 0, w3["ctx_len"] >= 16384)
    w3f = make_requests(3, force_first_len=131072); assert w3f["ctx_len"][0] == 131072 and w3f["mode"][0] == 0
    w4 = make_requests(4); assert w4["ctx_len"].min() >= 512 and w4["ctx_len"].max() <= 2048 and w4["group"] == 1


def test_pool_is_deterministic_per_pair_and_poisoned():
    ctx = np.array([40, 7, 16], dtype=np.int32)
    a = make_kv_pool(3, [(0, 1), (2, 0), (1, 1)], ctx)
    b = make_kv_pool(3, [(1, 1), (0, 1)], ctx, spare_slots=9)
    # pair (0,1) holds the same K/V rows in both pools, wherever its pages landed
    def rows(kv, p, name):
        s = kv["page_ids"][kv["page_indptr"][p]:kv["page_indptr"][p + 1]]
        return kv[name][s].reshape(-1, 128)
    for name in ("k_pool", "v_pool"):
        assert np.array_equal(rows(a, 0, name)[:40], rows(b, 1, name)[:40])
        assert np.array_equal(rows(a, 2, name)[:7], rows(b, 0, name)[:7])
        assert (rows(a, 0, name)[40:] == 0x7FFF).all()        # tail of the last page
        assert not np.array_equal(rows(a, 0, "k_pool")[:40], rows(a, 0, "v_pool")[:40])
    assert a["page_indptr"].tolist() == [0, 3, 4, 5]
    assert sorted(a["page_ids"].tolist()) != list(range(5)) or a["n_slots"] == 8
    used = np.zeros(a["n_slots"], bool); used[a["page_ids"]] = True
    assert (a["k_pool"][~used] == 0x7FFF).all() and len(set(a["page_ids"].tolist())) == 5


def test_fp8_pool_quantisation_is_nearest_and_scaled_to_448():
    ctx = np.array([50], dtype=np.int32)
    kv = make_kv_pool(5, [(0, 0)], ctx, kv_dtype="fp8")
    slots = kv["page_ids"]
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([5, 17, 0, 0])))
    K = rng.standard_normal((50, 128), dtype=np.float32)
    Kp = np.zeros((64, 128), np.float32); Kp[:50] = K; Kp = Kp.reshape(4, 16, 128)
    finite = np.sort(E4M3_TABLE[~np.isnan(E4M3_TABLE)])
    for i, s in enumerate(slots):
        amax = np.abs(Kp[i]).max()
        assert kv["k_scale"][s] == np.float32(amax / np.float32(448.0))
        valid = 16 if i < 3 else 2
        y = (Kp[i][:valid] / kv["k_scale"][s]).astype(np.float64)
        dec = E4M3_TABLE[kv["k_pool"][s][:valid]]
        # nearest representable: no other code is closer
        best = np.abs(finite[None, :] - y.reshape(-1, 1)).min(axis=1)
        assert np.allclose(np.abs(dec.reshape(-1) - y.reshape(-1)), best, rtol=0, atol=1e-12)
        assert np.abs(dec).max() == 448.0
        assert (kv["k_pool"][s][valid:] == 0x7F).all()


def test_q_is_bf16_normal():
    q = make_q(1, 4, 8, 128)
    assert q.shape == (4, 8, 128) and q.dtype == np.uint16
    x = (q.astype(np.uint32) << 16).view(np.float32)
    assert abs(x.mean()) < 0.1 and 0.9 < x.std() < 1.1
