"""The C++ prefill tile-list builder against the oracle, bit for bit (no GPU needed)."""
import os

import numpy as np
import pytest

import oracle
import paper_2511_14116_amd as fs


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(fs.library_path()):
        from paper_2511_14116_amd.build import build
        build(verbose=False)
    return fs.load_library()


@pytest.mark.parametrize("seed", range(30))
def test_prefill_worklist_matches_oracle(seed):
    rng = np.random.default_rng(3000 + seed)
    B, Hkv, G, R = int(rng.integers(0, 12)), int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 8))
    n_done = rng.integers(0, 5000, size=B).astype(np.int32)
    n_new = (rng.integers(0, 300, size=B) * (rng.random(B) < 0.7)).astype(np.int32)
    owner = rng.integers(0, R, size=(B, Hkv)).astype(np.int32)
    tile = int(rng.integers(1, 70))
    chunk = int(rng.integers(0, 40)) * 32
    shape = fs.FsShape(B, Hkv * G, Hkv, 128, 16, R)
    for k in range(R):
        w_items, w_pairs, w_sched, w_chunks, w_out = oracle.build_prefill_worklist(n_done, n_new, owner, k, Hkv * G, tile, chunk)
        items, pairs, sched, chunks, out = fs.fs_build_prefill_worklist(shape, n_done, n_new, owner, k, tile, chunk)
        assert items.view(np.int32).reshape(-1, 8).tobytes() == w_items.tobytes()
        assert pairs.view(np.int32).reshape(-1, 4).tobytes() == w_pairs.tobytes()
        assert sched.tobytes() == w_sched.tobytes() and chunks.tobytes() == w_chunks.tobytes()
        assert out.tobytes() == w_out.tobytes()


def test_field_names_follow_the_oracle():
    assert fs.PREFILL_ITEM_DTYPE.names == oracle.PREFILL_ITEM_FIELDS
    assert fs.PREFILL_PAIR_DTYPE.names == oracle.PREFILL_PAIR_FIELDS
    assert fs.PREFILL_ITEM_DTYPE.itemsize == 32 and fs.PREFILL_PAIR_DTYPE.itemsize == 16


def test_tile_tokens_and_errors():
    assert fs.fs_prefill_tile_tokens(0) == -1 and fs.fs_prefill_tile_tokens(17) == -1
    ct = fs.fs_get_option("prefill_col_tiles")
    assert (fs.fs_get_option("prefill_waves"), ct) == (8, 1)
    assert fs.fs_get_option("prefill_wide_v") == -1          # nothing numeric is a process-wide option
    with pytest.raises(fs.FsError):
        fs.fs_set_option("prefill_wide_v", 1)
    for G, per_tile in ((1, 16), (2, 8), (3, 4), (4, 4), (5, 2), (8, 2), (16, 1)):
        assert fs.fs_prefill_tile_tokens(G) == fs.fs_get_option("prefill_waves") * ct * per_tile
    shape = fs.FsShape(1, 4, 2, 128, 16, 2)
    with pytest.raises(fs.FsError):
        fs.fs_build_prefill_worklist(shape, [0], [5], [[0, 1]], 2, 4)        # rank outside
    with pytest.raises(fs.FsError):
        fs.fs_build_prefill_worklist(shape, [0], [5], [[0, 1]], 0, 0)        # tile size
    with pytest.raises(fs.FsError):
        fs.fs_build_prefill_worklist(shape, [-1], [5], [[0, 1]], 0, 4)
    with pytest.raises(fs.FsError):
        fs.fs_build_prefill_worklist(shape, [0], [5], [[0, 7]], 0, 4)
    with pytest.raises(fs.FsError):
        fs.fs_build_prefill_worklist(shape, [0], [5], [[0, 1]], 0, 4, 48)    # chunk not a multiple of 32
    items, pairs, sched, chunks, out = fs.fs_build_prefill_worklist(shape, [9], [0], [[0, 1]], 0, 4)
    assert len(items) == 0 and len(pairs) == 0 and chunks.tolist() == [0] and out.tolist() == [0]


def test_bound_builder_fills_caller_arrays_and_follows_its_inputs():
    """The pre-marshalled call writes the same list into caller-held arrays, reads its inputs anew at every
    call, and reports a list that outgrows the arrays."""
    rng = np.random.default_rng(77)
    B, Hkv, G, R, tile, chunk = 6, 4, 2, 3, 8, 64
    shape = fs.FsShape(B, Hkv * G, Hkv, 128, 16, R)
    n_done = rng.integers(0, 400, size=B).astype(np.int32)
    n_new = rng.integers(1, 60, size=B).astype(np.int32)
    owner = rng.integers(0, R, size=(B, Hkv)).astype(np.int32)
    ref = fs.fs_build_prefill_worklist(shape, n_done, n_new, owner, 1, tile, chunk)
    cap_i, cap_p, cap_t = len(ref[0]) + 5, len(ref[1]) + 2, len(ref[3]) - 1 + 3
    items = np.zeros(cap_i, dtype=fs.PREFILL_ITEM_DTYPE)
    pairs = np.zeros(cap_p, dtype=fs.PREFILL_PAIR_DTYPE)
    sched = np.zeros(cap_i, dtype=np.int32)
    chunks = np.zeros(cap_t + 1, dtype=np.int64)
    out = np.zeros(cap_p + 1, dtype=np.int64)
    call = fs.bind_build_prefill_worklist(shape, n_done, n_new, owner, 1, tile, chunk, items, pairs, sched, chunks, out)
    for _ in range(2):
        call()
        ni, npairs, nt = call.n_items.value, call.n_pairs.value, call.n_tiles.value
        assert (ni, npairs, nt) == (len(ref[0]), len(ref[1]), len(ref[3]) - 1)
        assert items[:ni].tobytes() == ref[0].tobytes() and pairs[:npairs].tobytes() == ref[1].tobytes()
        assert sched[:ni].tobytes() == ref[2].tobytes() and chunks[:nt + 1].tobytes() == ref[3].tobytes()
        assert out[:npairs + 1].tobytes() == ref[4].tobytes()
        n_new[0] += 3                                        # the next call sees the changed input
        ref = fs.fs_build_prefill_worklist(shape, n_done, n_new, owner, 1, tile, chunk)
    n_new[:] = 5000                                          # far more tiles than the arrays hold
    with pytest.raises(fs.FsError) as e:
        call()
    assert e.value.status == fs.FS_ECAPACITY
    with pytest.raises(TypeError):
        fs.bind_build_prefill_worklist(shape, n_done.astype(np.int64), n_new, owner, 1, tile, chunk, items, pairs, sched, chunks, out)


def test_chunk_choice_matches_oracle():
    rng = np.random.default_rng(22)
    for _ in range(150):
        B, H, R, G = int(rng.integers(1, 7)), int(rng.integers(1, 5)), int(rng.integers(1, 4)), int(rng.integers(1, 5))
        n_done = rng.integers(0, 5000, size=B).astype(np.int32); n_new = rng.integers(0, 300, size=B).astype(np.int32)
        owner = rng.integers(0, R, size=(B, H)).astype(np.int32)
        rank, tile, want = int(rng.integers(0, R)), int(rng.integers(1, 40)), int(rng.integers(1, 700))      # want: slots
        mx = 32 * int(rng.integers(1, 200)); mn = 32 * int(rng.integers(1, mx // 32 + 1))
        shape = fs.FsShape(B, H * G, H, 128, 16, R)
        assert fs.fs_choose_prefill_chunk(shape, n_done, n_new, owner, rank, tile, mx, mn, want) == \
            oracle.choose_prefill_chunk(n_done, n_new, owner, rank, H * G, tile, mx, mn, want)
    shape = fs.FsShape(1, 2, 1, 128, 16, 1)
    for mx, mn, want in ((100, 32, 1), (64, 128, 1), (64, 16, 1), (64, 32, 0)):
        with pytest.raises(fs.FsError) as e:
            fs.fs_choose_prefill_chunk(shape, [0], [5], [[0]], 0, 4, mx, mn, want)
        assert e.value.status == fs.FS_EINVAL
