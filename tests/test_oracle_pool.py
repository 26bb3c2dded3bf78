"""Pins for the oracle's allocator, swap, segmentation and block layouts (CPU only)."""
import os

import numpy as np
import pytest

import oracle
from oracle import OracleError

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- O1 allocator
def test_alloc_first_ids_are_0_to_n():
    a = oracle.Allocator(10)
    assert a.alloc(4).tolist() == [0, 1, 2, 3]
    assert a.alloc(3).tolist() == [4, 5, 6]
    assert a.num_free == 3


def test_alloc_lifo_closed_form():
    a = oracle.Allocator(8)
    ids = a.alloc(5)
    a.free(ids[[1, 3, 4]])               # pushed in this order: 1, 3, 4
    assert a.alloc(3).tolist() == [4, 3, 1]   # last freed is reused first
    assert a.alloc(3).tolist() == [5, 6, 7]


def test_alloc_enospc_is_all_or_nothing():
    a = oracle.Allocator(4)
    a.alloc(3)
    with pytest.raises(OracleError) as e:
        a.alloc(2)
    assert e.value.code == -2
    assert a.num_free == 1
    assert a.alloc(1).tolist() == [3]


def test_alloc_double_free_and_range():
    a = oracle.Allocator(4)
    ids = a.alloc(2)
    with pytest.raises(OracleError) as e:
        a.free([2])                      # never allocated
    assert e.value.code == -4
    with pytest.raises(OracleError) as e:
        a.free([4])
    assert e.value.code == -3
    with pytest.raises(OracleError) as e:
        a.free([ids[0], ids[0]])
    assert e.value.code == -4
    assert a.num_free == 2               # failed frees changed nothing
    a.free(ids)
    assert a.num_free == 4


def test_alloc_brute_force_against_list_model():
    rng = np.random.default_rng(1)
    n = 37
    a = oracle.Allocator(n)
    stack = list(range(n - 1, -1, -1))   # python list used as the stack; pop() takes the end
    held = []
    for _ in range(2000):
        if rng.random() < 0.5:
            k = int(rng.integers(0, 9))
            if k > len(stack):
                with pytest.raises(OracleError):
                    a.alloc(k)
                continue
            want = [stack.pop() for _ in range(k)]
            assert a.alloc(k).tolist() == want
            held += want
        elif held:
            k = int(rng.integers(1, min(len(held), 6) + 1))
            pick = [held.pop(int(rng.integers(0, len(held)))) for _ in range(k)]
            a.free(pick)
            stack += pick
        assert a.num_free == len(stack)
        assert sorted(stack + held) == list(range(n))     # ids are conserved


# ---------------------------------------------------------------- O2 swap
def test_swap_matches_fancy_indexing_and_leaves_rest():
    rng = np.random.default_rng(2)
    dev = rng.integers(0, 2 ** 16, size=(20, 64), dtype=np.uint16)
    host = rng.integers(0, 2 ** 16, size=(12, 64), dtype=np.uint16)
    dev0, host0 = dev.copy(), host.copy()
    src = np.array([3, 3, 7, 0], np.int32)       # duplicate sources are allowed
    dst = np.array([5, 19, 0, 2], np.int32)
    oracle.swap(dev, host, src, dst)
    want = dev0.copy()
    want[dst] = host0[src]
    assert np.array_equal(dev, want)
    assert np.array_equal(host, host0)           # source untouched
    untouched = np.setdiff1d(np.arange(20), dst)
    assert np.array_equal(dev[untouched], dev0[untouched])


def test_swap_round_trip_and_permutation():
    rng = np.random.default_rng(3)
    dev = rng.standard_normal((16, 32)).astype(np.float32)
    host = np.zeros((16, 32), np.float32)
    dev0 = dev.copy()
    perm = rng.permutation(16).astype(np.int32)
    oracle.swap(host, dev, np.arange(16, dtype=np.int32), perm)      # out: host[perm[k]] = dev[k]
    assert np.array_equal(host[perm], dev0)
    dev[:] = 0
    back = rng.permutation(16).astype(np.int32)
    oracle.swap(dev, host, perm, back)                                # in, to other slots
    assert np.array_equal(dev[back], dev0)


def test_swap_errors():
    dev = np.zeros((4, 8), np.uint16)
    host = np.ones((4, 8), np.uint16)
    with pytest.raises(OracleError) as e:
        oracle.swap(dev, host, [0, 1], [2, 2])
    assert e.value.code == -4
    with pytest.raises(OracleError) as e:
        oracle.swap(dev, host, [0, 4], [1, 2])
    assert e.value.code == -3
    assert not dev.any()                         # nothing copied on error
    oracle.swap(dev, host, [], [])               # empty list is a no-op


# ---------------------------------------------------------------- segmentation
def test_segment_equals_stable_argsort():
    rng = np.random.default_rng(4)
    for T, n_ad in [(1, 1), (50, 3), (1000, 40), (257, 300)]:
        ta = rng.integers(-1, n_ad, size=T).astype(np.int32)
        seg_adapter, seg_start, perm = oracle.segment(ta, n_ad)
        keep = np.flatnonzero(ta >= 0)
        want_perm = keep[np.argsort(ta[keep], kind="stable")]
        assert np.array_equal(perm, want_perm)
        ids, counts = np.unique(ta[keep], return_counts=True)
        assert np.array_equal(seg_adapter, ids)
        assert np.array_equal(np.diff(seg_start), counts)
        assert seg_start[0] == 0


# ---------------------------------------------------------------- layouts
def test_kv_block_layout_golden():
    bt, n_kv, d = 4, 2, 3
    rows = [l.split() for l in open(os.path.join(GOLD, "kv_block_layout.txt")) if l[0] in "KV"]
    # write distinct values as the "new" K/V of one sequence that fills exactly one block
    k_new = (np.arange(bt * n_kv * d, dtype=np.float32) + 1).reshape(bt, n_kv, d)
    v_new = -(np.arange(bt * n_kv * d, dtype=np.float32) + 1).reshape(bt, n_kv, d)
    pool = np.zeros((3, 2 * bt * n_kv * d), np.float32)
    oracle.kv_append(pool, "f32", bt, n_kv, d, [0, bt], [0], np.array([[1]], np.int32), k_new, v_new)
    assert not pool[0].any() and not pool[2].any()
    for kind, g, s, c, off in rows:
        g, s, c, off = int(g), int(s), int(c), int(off)
        want = k_new[s, g, c] if kind == "K" else v_new[s, g, c]
        assert pool[1, off] == want, (kind, g, s, c, off)
    # every element of the block was written exactly once (the map is a bijection)
    assert len(np.unique(pool[1])) == pool.shape[1]


def test_lora_page_layout_golden():
    lines = [l.split() for l in open(os.path.join(GOLD, "lora_page_layout.txt")) if not l.startswith("#")]
    table = [5, 2, 7]
    for row_len, rows in ((8, [l for l in lines if l[0] != "S"]), (12, [l[1:] for l in lines if l[0] == "S"])):
        for row, blk, off in rows:
            pool = np.zeros((8, 32), np.float32)
            vals = np.arange(1, row_len + 1, dtype=np.float32)
            oracle.lora_write_row(pool, "f32", table, int(row), vals)
            assert np.array_equal(pool[int(blk), int(off):int(off) + row_len], vals), (row_len, row)
            assert np.count_nonzero(pool) == row_len
            assert np.array_equal(oracle.lora_read_row(pool, "f32", table, row_len, int(row)), vals)


def test_lora_rows_are_disjoint_and_inside_their_table():
    rng = np.random.default_rng(5)
    be, row_len = 96, 20                        # 4 rows per block, 16 elements of slack
    table = rng.permutation(30)[:5].astype(np.int32)
    pool = np.zeros((30, be), np.float32)
    for row in range(20):
        oracle.lora_write_row(pool, "f32", table, row, np.full(row_len, row + 1, np.float32))
    for row in range(20):
        assert np.all(oracle.lora_read_row(pool, "f32", table, row_len, row) == row + 1)
    others = np.setdiff1d(np.arange(30), table)
    assert not pool[others].any()
    assert np.count_nonzero(pool) == 20 * row_len
