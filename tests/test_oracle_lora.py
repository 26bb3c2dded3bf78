"""Pins for the oracle's LoRA projection (Eq. 1 / Eq. 2 in row-vector form), CPU only.

The adapters here are built directly in numpy for cases where the page layout is
known without any layout code: when all rows of a table fit in its first block,
the first `n` rows of that block, reshaped [rows, row_len], are the matrix.
"""
import numpy as np
import pytest

import oracle
from oracle import OracleError
from paper_2505_03756_amd import workload as wl


def _single_block_adapters(rng, dtype, n_ad, r, d_in, d_out, be, n_blocks=16, std=0.02):
    """Each adapter owns one block for A rows and one for B rows (row_base 0)."""
    sd = wl.storage_dtype(dtype)
    pool = np.zeros((n_blocks, be), dtype=sd)
    ids = rng.permutation(n_blocks)[:2 * n_ad].astype(np.int32)
    A = rng.standard_normal((n_ad, r, d_in)).astype(np.float32) * std
    B = rng.standard_normal((n_ad, r, d_out)).astype(np.float32) * std
    for a in range(n_ad):
        pool[ids[2 * a], :r * d_in] = wl.quantize(A[a].reshape(-1), dtype)
        pool[ids[2 * a + 1], :r * d_out] = wl.quantize(B[a].reshape(-1), dtype)
    Aq = wl.dequantize(wl.quantize(A.reshape(-1), dtype), dtype).reshape(A.shape)
    Bq = wl.dequantize(wl.quantize(B.reshape(-1), dtype), dtype).reshape(B.shape)
    meta = dict(rank=np.full(n_ad, r, np.int32), scale=np.full(n_ad, 1.0, np.float32),
                a_tab_off=np.arange(n_ad, dtype=np.int32) * 2, a_row_base=np.zeros(n_ad, np.int32),
                b_tab_off=np.arange(n_ad, dtype=np.int32) * 2 + 1, b_row_base=np.zeros(n_ad, np.int32),
                block_tables=ids)
    return pool, Aq, Bq, meta


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_single_adapter_equals_two_matmuls(dtype):
    rng = np.random.default_rng(10)
    T, d_in, d_out, r, be = 9, 48, 40, 4, 256
    pool, A, B, m = _single_block_adapters(rng, dtype, 1, r, d_in, d_out, be)
    m["scale"][:] = 1.5
    x = wl.quantize(rng.standard_normal((T, d_in)).astype(np.float32), dtype)
    y0 = wl.quantize(rng.standard_normal((T, d_out)).astype(np.float32), dtype)
    got = oracle.lora_apply(pool, dtype, x, np.zeros(T, np.int32), d_out=d_out, y_in=y0, **m)
    xd, yd = wl.dequantize(x, dtype), wl.dequantize(y0, dtype)
    want = yd + 1.5 * (xd @ A[0].T) @ B[0]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_orientation_is_x_A_then_B():
    # d_in != d_out and a rank-1 adapter: delta = (x . a) * b, an outer-product closed form;
    # a transposed operand or swapped A/B cannot reproduce it.
    T, d_in, d_out, be = 3, 6, 10, 64
    a = np.arange(1, d_in + 1, dtype=np.float32)
    b = np.arange(1, d_out + 1, dtype=np.float32) * 0.5
    pool = np.zeros((4, be), np.float32)
    pool[2, :d_in] = a
    pool[0, :d_out] = b
    x = np.eye(T, d_in, dtype=np.float32) * 2.0           # token t picks out 2*a[t]
    y0 = np.zeros((T, d_out), np.float32)
    got = oracle.lora_apply(pool, "f32", x, np.zeros(T, np.int32), rank=[1], scale=[3.0], a_tab_off=[0],
                            a_row_base=[0], b_tab_off=[1], b_row_base=[0], block_tables=[2, 0], d_out=d_out,
                            y_in=y0)
    want = 3.0 * (2.0 * a[:T, None].astype(np.float64)) * b[None, :].astype(np.float64)
    np.testing.assert_allclose(got, want, rtol=0, atol=0)


def test_heterogeneous_batch_rowbase_and_multi_block_tables():
    # several adapters of different rank whose rows span blocks and start at a non-zero row_base;
    # the matrices are placed with lora_write_row and checked against per-token numpy products.
    rng = np.random.default_rng(11)
    d_in, d_out, be = 32, 24, 128                # 4 A-rows or 5 B-rows per block
    ranks = [3, 8, 5]
    n_blocks = 64
    pool = np.zeros((n_blocks, be), np.float32)
    free = list(rng.permutation(n_blocks))
    tables, meta = [], {k: [] for k in ("a_tab_off", "a_row_base", "b_tab_off", "b_row_base")}
    mats = []
    for r in ranks:
        a_base, b_base = int(rng.integers(0, 6)), int(rng.integers(0, 6))
        na = -(-(a_base + r) // (be // d_in))
        nb = -(-(b_base + r) // (be // d_out))
        ta = [free.pop() for _ in range(na)]
        tb = [free.pop() for _ in range(nb)]
        meta["a_tab_off"].append(sum(len(t) for t in tables)); tables.append(ta)
        meta["b_tab_off"].append(sum(len(t) for t in tables)); tables.append(tb)
        meta["a_row_base"].append(a_base); meta["b_row_base"].append(b_base)
        A = rng.standard_normal((r, d_in)).astype(np.float32)
        B = rng.standard_normal((r, d_out)).astype(np.float32)
        for rho in range(r):
            oracle.lora_write_row(pool, "f32", ta, a_base + rho, A[rho])
            oracle.lora_write_row(pool, "f32", tb, b_base + rho, B[rho])
        mats.append((A.astype(np.float64), B.astype(np.float64)))
    bt_all = np.concatenate([np.asarray(t, np.int32) for t in tables])
    T = 40
    ta_ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    x = rng.standard_normal((T, d_in)).astype(np.float32)
    y0 = rng.standard_normal((T, d_out)).astype(np.float32)
    scale = np.array([0.5, 2.0, -1.0], np.float32)
    got = oracle.lora_apply(pool, "f32", x, ta_ids, rank=ranks, scale=scale, block_tables=bt_all, d_out=d_out,
                            y_in=y0, **meta)
    for t in range(T):
        want = y0[t].astype(np.float64)
        if ta_ids[t] >= 0:
            A, B = mats[ta_ids[t]]
            want = want + float(scale[ta_ids[t]]) * ((x[t].astype(np.float64) @ A.T) @ B)
        np.testing.assert_allclose(got[t], want, rtol=1e-12, atol=1e-12)
    # id -1 => exactly the base term
    none = np.flatnonzero(ta_ids < 0)
    assert len(none) and np.array_equal(got[none], y0[none].astype(np.float64))
    # a selection returns the same rows
    sel = np.array([7, 0, 33], np.int32)
    got_sel = oracle.lora_apply(pool, "f32", x, ta_ids, rank=ranks, scale=scale, block_tables=bt_all,
                                d_out=d_out, y_in=y0, sel=sel, **meta)
    assert np.array_equal(got_sel, got[sel])


def _step_lora(step, p, pool, **over):
    pr = step.proj[p]
    kw = dict(rank=step.rank, scale=step.scale, a_tab_off=pr.a_tab_off, a_row_base=pr.a_row_base,
              b_tab_off=pr.b_tab_off, b_row_base=pr.b_row_base, block_tables=step.lora_tables,
              d_out=pr.d_out, y_in=step.acts["base_" + p])
    kw.update(over)
    return oracle.lora_apply(pool, step.cfg.dtype, step.acts["x"], step.token_adapter, **kw)


def _tiny_step():
    from helpers import resident_pool
    step = wl.make_step(wl.config("tiny"))
    return step, resident_pool(step)


def test_zero_B_gives_zero_delta():
    step, pool = _tiny_step()
    pr = step.proj["q"]
    for a in np.flatnonzero(step.rank):
        tb = step.lora_tables[pr.b_tab_off[a]:]
        for rho in range(step.rank[a]):
            oracle.lora_write_row(pool, "f32", tb, pr.b_row_base[a] + rho, np.zeros(pr.d_out, np.float32))
    got = _step_lora(step, "q", pool)
    assert np.array_equal(got, step.acts["base_q"].astype(np.float64))


def test_factored_equals_dense_delta():
    # Eq. 1 literally: materialise dW = A B per adapter and apply it with a library matmul
    step, pool = _tiny_step()
    for p in ("q", "v"):
        pr = step.proj[p]
        got = _step_lora(step, p, pool)
        x = step.acts["x"].astype(np.float64)
        want = step.acts["base_" + p].astype(np.float64).copy()
        for a in np.flatnonzero(step.rank):
            dW = oracle.lora_dense_delta(pool, "f32", pr.d_in, pr.d_out, int(step.rank[a]),
                                         step.lora_tables[pr.a_tab_off[a]:], int(pr.a_row_base[a]),
                                         step.lora_tables[pr.b_tab_off[a]:], int(pr.b_row_base[a]))
            rows = np.flatnonzero(step.token_adapter == a)
            want[rows] += float(step.scale[a]) * (x[rows] @ dW)
        np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
        assert np.abs(got - step.acts["base_" + p]).max() > 1e-3      # the delta is not trivially zero


def test_dense_delta_matches_numpy_on_directly_placed_adapter():
    rng = np.random.default_rng(12)
    pool, A, B, m = _single_block_adapters(rng, "f16", 2, 4, 16, 12, 128)
    for a in range(2):
        dW = oracle.lora_dense_delta(pool, "f16", 16, 12, 4, m["block_tables"][m["a_tab_off"][a]:], 0,
                                     m["block_tables"][m["b_tab_off"][a]:], 0)
        np.testing.assert_allclose(dW, A[a].T @ B[a], rtol=1e-13, atol=1e-15)


def test_scale_linearity_and_token_permutation():
    step, pool = _tiny_step()
    base = step.acts["base_q"].astype(np.float64)
    d1 = _step_lora(step, "q", pool) - base
    d2 = _step_lora(step, "q", pool, scale=step.scale * 2) - base
    np.testing.assert_allclose(d2, 2 * d1, rtol=1e-12, atol=1e-15)
    rng = np.random.default_rng(13)
    perm = rng.permutation(step.n_tokens)
    pr = step.proj["q"]
    got_p = oracle.lora_apply(pool, "f32", np.ascontiguousarray(step.acts["x"][perm]), step.token_adapter[perm],
                              rank=step.rank, scale=step.scale, a_tab_off=pr.a_tab_off,
                              a_row_base=pr.a_row_base, b_tab_off=pr.b_tab_off, b_row_base=pr.b_row_base,
                              block_tables=step.lora_tables, d_out=pr.d_out,
                              y_in=np.ascontiguousarray(step.acts["base_q"][perm]))
    assert np.array_equal(got_p, (d1 + base)[perm])


def test_physical_block_permutation_changes_nothing():
    step, pool = _tiny_step()
    ref = _step_lora(step, "v", pool)
    rng = np.random.default_rng(14)
    sigma = rng.permutation(pool.shape[0]).astype(np.int32)      # block b moves to sigma[b]
    pool2 = np.empty_like(pool)
    pool2[sigma] = pool
    got = _step_lora(step, "v", pool2, block_tables=sigma[step.lora_tables])
    assert np.array_equal(got, ref)


def test_w_base_path_equals_library_matmul():
    rng = np.random.default_rng(15)
    pool, A, B, m = _single_block_adapters(rng, "f32", 1, 2, 12, 7, 64)
    x = rng.standard_normal((5, 12)).astype(np.float32)
    W = rng.standard_normal((12, 7)).astype(np.float32)
    got = oracle.lora_apply(pool, "f32", x, np.zeros(5, np.int32), d_out=7, w_base=W, **m)
    want = x.astype(np.float64) @ W.astype(np.float64) + (x.astype(np.float64) @ A[0].T) @ B[0]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_token_with_absent_adapter_is_an_error():
    step, pool = _tiny_step()
    rank = step.rank.copy()
    rank[step.token_adapter[0]] = 0
    with pytest.raises(OracleError) as e:
        _step_lora(step, "q", pool, rank=rank)
    assert e.value.code == -1


def test_generator_distinct_adapter_count_matches_eq3_form():
    # Eq. 3's expression for the number of adapters a batch needs: sum_i 1 - (1 - p_i)^BS.
    # 100 equally likely adapters, 256 draws -> 100 * (1 - 0.99^256) = 92.37
    assert abs(wl.expected_distinct_adapters(np.full(100, 0.01), 256) - 100 * (1 - 0.99 ** 256)) < 1e-9
    cfg = wl.config("7b_decode")
    counts = [len(np.unique(wl.make_step(cfg, seed=s, with_acts=False, fill_content=False).seq_adapter))
              for s in range(20)]
    assert abs(np.mean(counts) - 92.37) < 2.0
