"""Pins for the oracle's KV append and paged prefix attention (CPU only)."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import OracleError
from paper_2505_03756_amd import workload as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _paged_from_contig(rng, K, V, bt, dtype="f32", n_blocks=None, poison=True):
    """Store contiguous K,V [L, n_kv, d] (float) for ONE sequence into a fresh pool through
    kv_append (as if all L positions were new), in shuffled physical blocks."""
    L, n_kv, d = K.shape
    nb = -(-L // bt)
    n_blocks = n_blocks or nb + 5
    sd = wl.storage_dtype(dtype)
    pool = np.zeros((n_blocks, 2 * bt * n_kv * d), dtype=sd)
    if poison:
        pool[:] = np.float32(np.nan) if dtype == "f32" else 0x7E00
    table = rng.permutation(n_blocks)[:nb].astype(np.int32)[None, :]
    kq = wl.quantize(K.reshape(-1), dtype).reshape(L, n_kv, d)
    vq = wl.quantize(V.reshape(-1), dtype).reshape(L, n_kv, d)
    oracle.kv_append(pool, dtype, bt, n_kv, d, [0, L], [0], table, kq, vq)
    return pool, table, wl.dequantize(kq, dtype), wl.dequantize(vq, dtype)


def _sdpa_reference(K, V, q, P, n_h):
    """Library scaled-dot-product attention on contiguous inputs with an explicit mask."""
    L, n_kv, d = K.shape
    N = q.shape[0]
    g = n_h // n_kv
    Kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(g, dim=0)      # [n_h, L, d]
    Vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(g, dim=0)
    qt = torch.from_numpy(q).permute(1, 0, 2)                                   # [n_h, N, d]
    mask = torch.zeros(N, L, dtype=torch.bool)
    for j in range(N):
        mask[j, :P + j + 1] = True
    out = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, attn_mask=mask)
    return out.permute(1, 0, 2).numpy()


# ---------------------------------------------------------------- O4 append
def test_append_round_trip_bit_exact_and_others_untouched():
    rng = np.random.default_rng(20)
    cfg = wl.config("tiny")
    step = wl.make_step(cfg)
    from helpers import resident_pool
    pool = resident_pool(step)
    before = pool.copy()
    bt, n_kv, d = cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim
    k_new = step.acts["k_new"].reshape(-1, n_kv, d)
    v_new = step.acts["v_new"].reshape(-1, n_kv, d)
    oracle.kv_append(pool, "f32", bt, n_kv, d, step.cu_new, step.prefix_len, step.kv_tables, k_new, v_new)
    for i in range(cfg.n_seqs):
        P, N = int(step.prefix_len[i]), int(step.new_len[i])
        K, V = oracle.kv_gather(pool, "f32", bt, n_kv, d, step.kv_tables[i], P + N)
        K0, V0 = oracle.kv_gather(before, "f32", bt, n_kv, d, step.kv_tables[i], P + N)
        lo, hi = step.cu_new[i], step.cu_new[i + 1]
        assert np.array_equal(K[P:], k_new[lo:hi].astype(np.float64))
        assert np.array_equal(V[P:], v_new[lo:hi].astype(np.float64))
        assert np.array_equal(K[:P], K0[:P]) and np.array_equal(V[:P], V0[:P])     # prefix kept
    in_tables = np.unique(step.kv_tables[step.kv_tables >= 0])
    others = np.setdiff1d(np.arange(cfg.n_dev_blocks), in_tables)
    assert np.array_equal(pool[others], before[others])
    changed = int(np.count_nonzero(pool.view(np.uint32) != before.view(np.uint32)))
    assert changed <= 2 * step.n_tokens * n_kv * d


def test_append_overflowing_table_is_an_error():
    pool = np.zeros((4, 2 * 4 * 1 * 2), np.float32)
    k = np.zeros((3, 1, 2), np.float32)
    with pytest.raises(OracleError) as e:
        oracle.kv_append(pool, "f32", 4, 1, 2, [0, 3], [6], np.array([[0, 1]], np.int32), k, k)
    assert e.value.code == -3


# ---------------------------------------------------------------- O5 attention
def test_golden_closed_forms():
    want = dict(l.split() for l in open(os.path.join(GOLD, "attention_closed_form.txt")) if not l.startswith("#"))
    rng = np.random.default_rng(21)

    def run(keys, vals, q, P):
        K = np.array(keys, np.float64).reshape(-1, 1, 1)
        V = np.array(vals, np.float64).reshape(-1, 1, 1)
        pool, table, _, _ = _paged_from_contig(rng, K, V, bt=2)
        N = len(keys) - P
        qa = np.full((N, 1), q, np.float32)
        return oracle.paged_attention(pool, "f32", 2, 1, 1, 1, [0, N], [P], table, qa, sm_scale=1.0).reshape(-1)

    assert abs(run([0, 1], [8, 4], math.log(3), 1)[0] - float(want["two_keys"])) < 1e-6
    assert abs(run([0, 1, 2], [7, 14, 21], math.log(2), 2)[0] - float(want["three_keys"])) < 1e-5
    out = run([0, 1, 2], [7, 14, 21], math.log(2), 1)
    assert abs(out[0] - float(want["causal_tok0"])) < 1e-5
    assert abs(out[1] - float(want["causal_tok1"])) < 1e-5


@pytest.mark.parametrize("n_h,n_kv", [(4, 4), (8, 2), (6, 1)])
def test_equals_library_sdpa_and_contiguous_oracle(n_h, n_kv):
    rng = np.random.default_rng(22)
    d, bt, P, N = 16, 4, 13, 7
    K = rng.standard_normal((P + N, n_kv, d))
    V = rng.standard_normal((P + N, n_kv, d))
    q = rng.standard_normal((N, n_h, d)).astype(np.float32)
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    got = oracle.paged_attention(pool, "f32", bt, n_kv, d, n_h, [0, N], [P], table, q.reshape(N, -1))
    want = _sdpa_reference(Kq, Vq, q.astype(np.float64), P, n_h)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)
    contig = oracle.contig_attention(Kq, Vq, q.astype(np.float64), P)
    np.testing.assert_allclose(got, contig, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_16bit_storage_is_decoded_exactly(dtype):
    rng = np.random.default_rng(23)
    d, bt, P, N, n_h = 8, 4, 5, 3, 2
    K = rng.standard_normal((P + N, n_h, d))
    V = rng.standard_normal((P + N, n_h, d))
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt, dtype=dtype)
    qb = wl.quantize(rng.standard_normal((N, n_h * d)).astype(np.float32), dtype)
    got = oracle.paged_attention(pool, dtype, bt, n_h, d, n_h, [0, N], [P], table, qb)
    want = _sdpa_reference(Kq, Vq, wl.dequantize(qb, dtype).reshape(N, n_h, d), P, n_h)
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


def test_brute_force_tiny():
    rng = np.random.default_rng(24)
    d, bt, P, N = 4, 2, 3, 5
    K = rng.standard_normal((P + N, 1, d))
    V = rng.standard_normal((P + N, 1, d))
    q = rng.standard_normal((N, 1, d)).astype(np.float32)
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    got = oracle.paged_attention(pool, "f32", bt, 1, d, 1, [0, N], [P], table, q.reshape(N, -1))
    for j in range(N):
        sc = [sum(float(q[j, 0, c]) * Kq[k, 0, c] for c in range(d)) / math.sqrt(d) for k in range(P + j + 1)]
        m = max(sc)
        e = [math.exp(s - m) for s in sc]
        for c in range(d):
            want = sum(e[k] * Vq[k, 0, c] for k in range(len(e))) / sum(e)
            assert abs(got[j, 0, c] - want) < 1e-12


def test_softmax_weights_sum_to_one_and_step_invariants():
    from helpers import resident_pool
    cfg = wl.config("tiny")
    step = wl.make_step(cfg, poison_fresh=True)
    pool = resident_pool(step)
    bt, n_kv, d, n_h = cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads
    oracle.kv_append(pool, "f32", bt, n_kv, d, step.cu_new, step.prefix_len, step.kv_tables,
                     step.acts["k_new"], step.acts["v_new"])
    out, wsum = oracle.paged_attention(pool, "f32", bt, n_kv, d, n_h, step.cu_new, step.prefix_len,
                                       step.kv_tables, step.acts["q"], want_wsum=True)
    assert np.isfinite(out).all()              # poisoned slots beyond each length are never read
    np.testing.assert_allclose(wsum, 1.0, rtol=0, atol=1e-12)
    # invariance under a random permutation of the physical blocks
    rng = np.random.default_rng(25)
    sigma = rng.permutation(pool.shape[0]).astype(np.int32)
    pool2 = np.empty_like(pool)
    pool2[sigma] = pool
    tab2 = np.where(step.kv_tables >= 0, sigma[np.maximum(step.kv_tables, 0)], -1).astype(np.int32)
    out2 = oracle.paged_attention(pool2, "f32", bt, n_kv, d, n_h, step.cu_new, step.prefix_len, tab2,
                                  step.acts["q"])
    assert np.array_equal(out, out2)
    # equality with contiguous attention, sequence by sequence
    q = step.acts["q"].astype(np.float64).reshape(-1, n_h, d)
    for i in range(cfg.n_seqs):
        P, N = int(step.prefix_len[i]), int(step.new_len[i])
        K, V = oracle.kv_gather(pool, "f32", bt, n_kv, d, step.kv_tables[i], P + N)
        lo, hi = step.cu_new[i], step.cu_new[i + 1]
        want = _sdpa_reference(K, V, q[lo:hi], P, n_h)
        np.testing.assert_allclose(out[lo:hi], want, rtol=1e-9, atol=1e-11)
    # a selection of tokens gives the same rows
    sel = np.array([step.n_tokens - 1, 0, 5], np.int32)
    out_sel = oracle.paged_attention(pool, "f32", bt, n_kv, d, n_h, step.cu_new, step.prefix_len,
                                     step.kv_tables, step.acts["q"], sel=sel)
    assert np.array_equal(out_sel, out[sel])


def test_zero_query_gives_running_mean_of_values():
    # q = 0: token j's output is the plain mean of V[0 .. P+j]; pins the causal boundary and
    # the prefix/fresh seam.
    rng = np.random.default_rng(26)
    d, bt, n_h = 8, 4, 2
    for P, N in [(0, 6), (5, 4), (8, 1), (3, 9)]:
        K = rng.standard_normal((P + N, n_h, d))
        V = rng.standard_normal((P + N, n_h, d))
        pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
        q = np.zeros((N, n_h * d), np.float32)
        got = oracle.paged_attention(pool, "f32", bt, n_h, d, n_h, [0, N], [P], table, q)
        for j in range(N):
            np.testing.assert_allclose(got[j], Vq[:P + j + 1].mean(axis=0), rtol=1e-12, atol=1e-13)


def test_degenerate_cases():
    rng = np.random.default_rng(27)
    d, bt, n_h = 8, 4, 2
    # P = 0, N = 1: out = v0
    K = rng.standard_normal((1, n_h, d)); V = rng.standard_normal((1, n_h, d))
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    q = rng.standard_normal((1, n_h * d)).astype(np.float32)
    got = oracle.paged_attention(pool, "f32", bt, n_h, d, n_h, [0, 1], [0], table, q)
    np.testing.assert_allclose(got[0], Vq[0], rtol=1e-15, atol=0)
    # all V rows equal: out = that row
    L = 11
    K = rng.standard_normal((L, n_h, d)); V = np.tile(rng.standard_normal((1, n_h, d)), (L, 1, 1))
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    q = rng.standard_normal((4, n_h * d)).astype(np.float32)
    got = oracle.paged_attention(pool, "f32", bt, n_h, d, n_h, [0, 4], [L - 4], table, q)
    np.testing.assert_allclose(got, np.broadcast_to(Vq[0], got.shape), rtol=1e-13, atol=1e-14)
    # one key with a huge score: out -> its V row, no overflow
    K = rng.standard_normal((L, n_h, d)); V = rng.standard_normal((L, n_h, d))
    K[4] = 300.0
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    q = np.full((1, n_h * d), 50.0, np.float32)
    got = oracle.paged_attention(pool, "f32", bt, n_h, d, n_h, [0, 1], [L - 1], table, q)
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got[0], Vq[4], rtol=1e-12, atol=1e-12)


def test_prefix_new_split_does_not_matter_for_last_token():
    rng = np.random.default_rng(28)
    d, bt, n_h, L = 8, 4, 2, 14
    K = rng.standard_normal((L, n_h, d)); V = rng.standard_normal((L, n_h, d))
    pool, table, _, _ = _paged_from_contig(rng, K, V, bt)
    qlast = rng.standard_normal((1, n_h * d)).astype(np.float32)
    rows = []
    for N in (1, 3, 7, L):
        q = np.zeros((N, n_h * d), np.float32)
        q[-1] = qlast
        rows.append(oracle.paged_attention(pool, "f32", bt, n_h, d, n_h, [0, N], [L - N], table, q)[-1])
    for r in rows[1:]:
        assert np.array_equal(r, rows[0])


def test_gqa_head_mapping():
    # query head h reads kv head h // (n_h / n_kv): make the two kv heads very different
    rng = np.random.default_rng(29)
    d, bt, L = 4, 4, 6
    K = rng.standard_normal((L, 2, d)); V = np.zeros((L, 2, d))
    V[:, 0] = 1.0
    V[:, 1] = -1.0
    pool, table, _, _ = _paged_from_contig(rng, K, V, bt)
    q = rng.standard_normal((1, 6 * d)).astype(np.float32)
    got = oracle.paged_attention(pool, "f32", bt, 2, d, 6, [0, 1], [L - 1], table, q)
    np.testing.assert_allclose(got[0, :3], 1.0, atol=1e-14)
    np.testing.assert_allclose(got[0, 3:], -1.0, atol=1e-14)


def test_explicit_scale_and_default_scale():
    rng = np.random.default_rng(30)
    d, bt, L = 16, 4, 9
    K = rng.standard_normal((L, 1, d)); V = rng.standard_normal((L, 1, d))
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    q = rng.standard_normal((1, d)).astype(np.float32)
    a = oracle.paged_attention(pool, "f32", bt, 1, d, 1, [0, 1], [L - 1], table, q)
    b = oracle.paged_attention(pool, "f32", bt, 1, d, 1, [0, 1], [L - 1], table, q, sm_scale=0.25)
    assert np.array_equal(a, b)                      # 1/sqrt(16)
    c = oracle.paged_attention(pool, "f32", bt, 1, d, 1, [0, 1], [L - 1], table, q, sm_scale=1.0)
    s = Kq[:, 0] @ q[0].astype(np.float64)
    w = np.exp(s - s.max()); w /= w.sum()
    np.testing.assert_allclose(c[0, 0], w @ Vq[:, 0], rtol=1e-12, atol=1e-14)


def test_round_to_dtype_matches_numpy_formats():
    rng = np.random.default_rng(31)
    v = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-9, 5, size=2000),
                        [0.0, 65504.0, 65520.0, 1e-8, 6e-8, 2.0 ** -24, 3 * 2.0 ** -25]])
    got = oracle.round_to_dtype(v, "f16")
    with np.errstate(over="ignore"):
        want = v.astype(np.float16).astype(np.float64)
    assert np.array_equal(got, want)
    got = oracle.round_to_dtype(v, "bf16")
    want = wl.dequantize(wl.quantize(v.astype(np.float32), "bf16"), "bf16")
    v32 = v.astype(np.float32).astype(np.float64)
    ok = v32 == v                                    # quantize() rounds from fp32; compare where that is exact
    assert np.array_equal(got[ok], want[ok])


def test_block_size_is_a_storage_detail():
    """The same keys and values stored in blocks of 16 and of 32 positions (other slot strides, other tables)
    give the same attention, and each block size places element (head, slot, channel) where the layout rule
    says (K at (g*bt + s)*d + c, V at n_kv*bt*d + (g*d + c)*bt + s)."""
    rng = np.random.default_rng(33)
    L, n_kv, d, n_h, P = 77, 2, 8, 4, 50
    K = rng.standard_normal((L, n_kv, d))
    V = rng.standard_normal((L, n_kv, d))
    q = rng.standard_normal((L - P, n_h, d)).astype(np.float32)
    outs = []
    for bt in (16, 32):
        pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
        pos, g, c = 41, 1, 5
        blk = pool[table[0, pos // bt]]
        assert blk[(g * bt + pos % bt) * d + c] == np.float32(K[pos, g, c])
        assert blk[n_kv * bt * d + (g * d + c) * bt + pos % bt] == np.float32(V[pos, g, c])
        outs.append(oracle.paged_attention(pool, "f32", bt, n_kv, d, n_h, [0, L - P], [P], table, q))
    assert np.array_equal(outs[0], outs[1])
    assert np.allclose(outs[0], _sdpa_reference(K.astype(np.float32).astype(np.float64),
                                                V.astype(np.float32).astype(np.float64), q.astype(np.float64), P, n_h),
                       atol=1e-12)


# ---------------------------------------------------------------- whole-sequence (numpy) form of O5
def test_dense_form_equals_the_per_row_oracle_and_the_library():
    """oracle/attention_dense.py evaluates the same definition for all rows of a sequence with library matrix
    products; pinned against the per-row C oracle (paged, GQA, several sequences, bf16 storage, a block of 32
    positions) and against library scaled-dot-product attention on the gathered K and V."""
    from oracle.attention_dense import paged_attention_sequence
    from helpers import resident_pool
    for dtype, bt, seed in (("bf16", 16, 5), ("f16", 32, 6), ("f32", 16, 7)):
        cfg = wl.LayerConfig("dense_pin", dtype, 256, 8, 2, 64, 300, 4, 3, (8,), ("q",), 5, (0, 150), (1, 40),
                             block_tokens=bt, seed=seed)
        step = wl.make_step(cfg, poison_fresh=False)
        pool = resident_pool(step)
        n_kv, d, n_h = cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads
        oracle.kv_append(pool, dtype, bt, n_kv, d, step.cu_new, step.prefix_len, step.kv_tables,
                         step.acts["k_new"], step.acts["v_new"])
        rows = oracle.paged_attention(pool, dtype, bt, n_kv, d, n_h, step.cu_new, step.prefix_len, step.kv_tables,
                                      step.acts["q"])
        for i in range(cfg.n_seqs):
            got = paged_attention_sequence(pool, dtype, bt, n_kv, d, n_h, step.cu_new, step.prefix_len,
                                           step.kv_tables, step.acts["q"], i)
            lo, hi = int(step.cu_new[i]), int(step.cu_new[i + 1])
            np.testing.assert_allclose(got, rows[lo:hi], rtol=1e-11, atol=1e-13)
            P = int(step.prefix_len[i])
            K, V = oracle.kv_gather(pool, dtype, bt, n_kv, d, step.kv_tables[i], P + hi - lo)
            qv = wl.dequantize(step.acts["q"], dtype).reshape(-1, n_h, d)[lo:hi]
            np.testing.assert_allclose(got, _sdpa_reference(K, V, qv, P, n_h), rtol=1e-9, atol=1e-11)


def test_dense_form_closed_forms():
    """q = 0 gives the running mean of V over positions 0..P+j (pins the causal boundary and the prefix / fresh
    seam of the dense form on its own); an explicit scale is honoured."""
    from oracle.attention_dense import paged_attention_sequence
    rng = np.random.default_rng(31)
    L, n_kv, d, bt, P = 45, 2, 8, 16, 29
    K, V = rng.standard_normal((L, n_kv, d)), rng.standard_normal((L, n_kv, d))
    pool, table, Kq, Vq = _paged_from_contig(rng, K, V, bt)
    N = L - P
    q0 = np.zeros((N, 4 * d), np.float32)
    got = paged_attention_sequence(pool, "f32", bt, n_kv, d, 4, [0, N], [P], table, q0, 0)
    for j in range(N):
        for h in range(4):
            np.testing.assert_allclose(got[j, h], Vq[:P + j + 1, h // 2].mean(axis=0), rtol=1e-12, atol=1e-13)
    q1 = rng.standard_normal((N, 4 * d)).astype(np.float32)
    a = paged_attention_sequence(pool, "f32", bt, n_kv, d, 4, [0, N], [P], table, q1, 0, sm_scale=0.3)
    b = oracle.paged_attention(pool, "f32", bt, n_kv, d, 4, [0, N], [P], table, q1, sm_scale=0.3)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)
