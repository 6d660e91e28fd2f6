"""Pins for the oracle's KV commit (App. C "Acceptance": keep the prefix followed by the accepted path).  CPU only.

The oracle's row moves are checked against numpy's own gather (fancy indexing on a copy of the cache), on contiguous
and paged caches, plus the cases with a closed form: an accepted chain 0,1,2,... moves nothing, an empty path moves
nothing, and a path that is the last nodes of the tree pulls them down behind the prefix.
"""
import numpy as np
import pytest

from paper_2605_29727_amd import synth


def _path(rng, M, n):
    return np.sort(rng.choice(M, size=n, replace=False)).astype(np.int32)       # increasing node ids, as an accepted path is


@pytest.mark.parametrize("layers,L,M,n,shape", [(1, 0, 4, 2, (2, 8)), (3, 37, 64, 9, (8, 128)), (2, 500, 256, 16, (1, 64)),
                                                (4, 100, 16, 16, (2, 16)), (2, 7, 5, 0, (2, 4))])
@pytest.mark.parametrize("dtype", [np.uint16, np.float32])
def test_contiguous_equals_numpy_gather(oracle, layers, L, M, n, shape, dtype):
    rng = np.random.default_rng(1000 * layers + L + M + n)
    cache = rng.integers(0, 60000, size=(layers, L + M) + shape).astype(dtype)
    want = cache.copy()
    path = _path(rng, M, n)
    want[:, L:L + n] = cache[:, L + path]                                       # the definition, by the library
    new_len = oracle.kv_commit(cache, L, M, path)
    assert new_len == L + n
    assert np.array_equal(cache[:, :L + n], want[:, :L + n])                     # live part
    assert np.array_equal(cache[:, :L], want[:, :L])                             # prefix untouched


@pytest.mark.parametrize("layers,L,M,n", [(2, 100, 40, 7), (1, 15, 33, 12), (3, 16, 16, 16)])
def test_paged_equals_numpy_gather(oracle, layers, L, M, n):
    rng = np.random.default_rng(7 * layers + L + M + n)
    page, Hkv, D = synth.PAGE, 2, 8
    nblk_seq = -(-(L + M) // page)
    num_blocks = nblk_seq + 5
    bt = rng.permutation(num_blocks)[:nblk_seq].astype(np.int32)
    pool = rng.integers(0, 60000, size=(layers, num_blocks, page, Hkv, D)).astype(np.uint16)
    pos = np.arange(L + M)
    phys = bt[pos // page] * page + pos % page
    flat = pool.reshape(layers, num_blocks * page, Hkv, D)
    seq_before = flat[:, phys].copy()                                            # the logical sequence
    untouched = np.ones(num_blocks * page, dtype=bool); untouched[phys] = False
    other_before = flat[:, untouched].copy()
    path = _path(rng, M, n)
    new_len = oracle.kv_commit(pool, L, M, path, block_table=bt, page=page)
    seq_after = pool.reshape(layers, num_blocks * page, Hkv, D)[:, phys]
    want = seq_before.copy()
    want[:, L:L + n] = seq_before[:, L + path]
    assert new_len == L + n
    assert np.array_equal(seq_after[:, :L + n], want[:, :L + n])
    assert np.array_equal(pool.reshape(layers, num_blocks * page, Hkv, D)[:, untouched], other_before)   # other blocks


def test_chain_and_empty_paths_move_nothing(oracle):
    rng = np.random.default_rng(5)
    cache = rng.integers(0, 1000, size=(2, 30, 3, 4)).astype(np.float32)
    ref = cache.copy()
    assert oracle.kv_commit(cache, 20, 10, np.arange(6, dtype=np.int32)) == 26
    assert np.array_equal(cache, ref)
    assert oracle.kv_commit(cache, 20, 10, np.zeros(0, dtype=np.int32)) == 20
    assert np.array_equal(cache, ref)


def test_last_nodes_are_pulled_behind_the_prefix(oracle):
    cache = np.arange(2 * 12 * 2, dtype=np.float32).reshape(2, 12, 2)
    ref = cache.copy()
    oracle.kv_commit(cache, 4, 8, np.array([5, 6, 7], dtype=np.int32))
    assert np.array_equal(cache[:, 4:7], ref[:, 9:12])
    assert np.array_equal(cache[:, :4], ref[:, :4])


def test_bad_paths_are_refused(oracle):
    cache = np.zeros((1, 10, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.kv_commit(cache, 2, 8, np.array([0, 8], dtype=np.int32))           # node id out of range
    with pytest.raises(ValueError):
        oracle.kv_commit(cache, 2, 2, np.array([0, 1, 1], dtype=np.int32))        # longer than the tree
