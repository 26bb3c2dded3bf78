"""GPU parity of the layer glue (include/fllayer.h) against oracle/layer_oracle.py: each element-wise step
on its own, then the composed decoder layer over the paged pool."""
import math

import numpy as np
import pytest

import oracle
from oracle import layer_oracle as lo
from paper_2505_03756_amd import fllayer, workload as wl
from helpers import close
from paper_2505_03756_amd.harness import GpuStep, resident_pool, to_dev, to_np

pytestmark = pytest.mark.gpu

# one rounding of the result in the element type: half a unit in the last place, plus the fp32 arithmetic
TOL = {"f32": (1e-5, 1e-6), "f16": (2e-3, 1e-2), "bf16": (2e-3, 1e-2)}
ULP = {"f32": 2.0 ** -23, "f16": 2.0 ** -10, "bf16": 2.0 ** -7}


def within_one_rounding(got, want, dtype):
    """|got - want| <= one spacing of the element type at |want| (both were rounded once from nearly equal
    fp32 / fp64 values, so they are equal or neighbours), with an absolute floor for tiny values."""
    # fp32 tensors: the kernels' own arithmetic is fp32 (a sum of H squares, a reciprocal root, two products),
    # so the result carries a few fp32 roundings instead of one: 16 spacings (2e-6 relative)
    k = 16.0 if dtype == "f32" else 1.01
    tol = ULP[dtype] * np.maximum(np.abs(want), 2.0 ** -14) * k
    bad = np.abs(got - want) > tol
    return not bad.any(), float(np.abs(got - want).max()), int(bad.sum())


@pytest.mark.parametrize("dtype,T,H", [("f16", 37, 4096), ("bf16", 5, 5120), ("f32", 9, 256), ("f16", 1, 8), ("bf16", 130, 8192)])
def test_rmsnorm_and_fused_residual(dtype, T, H):
    rng = np.random.default_rng(T * 1000 + H)
    x_st, xv = lo.round_store(rng.normal(0, 1.5, (T, H)), dtype)
    w_st, wv = lo.round_store(rng.normal(1, 0.2, H), dtype)
    d_st, dv = lo.round_store(rng.normal(0, 0.5, (T, H)), dtype)
    x, w, d = to_dev(x_st), to_dev(w_st), to_dev(d_st)
    import torch
    y = torch.zeros_like(x)
    fllayer.rmsnorm(dtype, x, w, y, T, H, eps=1e-5)
    torch.cuda.synchronize()
    want = lo.round_store(lo.rmsnorm(xv, wv, 1e-5), dtype)[1]
    ok, worst, nbad = within_one_rounding(lo.load(to_np(y, x_st.dtype), dtype), want, dtype)
    assert ok, (worst, nbad)
    # fused: the residual is updated (bit-exact: one fp32 add of two exactly representable values, one rounding) ...
    r = x.clone()
    y2 = torch.zeros_like(x)
    fllayer.add_rmsnorm(dtype, r, d, w, y2, T, H, eps=1e-5)
    torch.cuda.synchronize()
    r_want_st, r_want = lo.round_store(xv + dv, dtype)
    assert np.array_equal(to_np(r, x_st.dtype), r_want_st)
    # ... and the norm is taken over the stored residual
    want2 = lo.round_store(lo.rmsnorm(r_want, wv, 1e-5), dtype)[1]
    ok, worst, nbad = within_one_rounding(lo.load(to_np(y2, x_st.dtype), dtype), want2, dtype)
    assert ok, (worst, nbad)
    # y == NULL: only the residual update
    r3 = x.clone()
    fllayer.add_rmsnorm(dtype, r3, d, None, None, T, H)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(r3, x_st.dtype), r_want_st)


@pytest.mark.parametrize("dtype,T,nh,nkv,d", [("f16", 50, 32, 32, 128), ("bf16", 17, 64, 8, 128), ("f32", 12, 4, 4, 64),
                                              ("f16", 3, 8, 2, 64)])
def test_rope(dtype, T, nh, nkv, d):
    import torch
    rng = np.random.default_rng(T + nh)
    q_st, qv = lo.round_store(rng.normal(0, 1, (T, nh, d)), dtype)
    k_st, kv = lo.round_store(rng.normal(0, 1, (T, nkv, d)), dtype)
    pos = rng.integers(0, 20000, size=T).astype(np.int32)
    pos[0] = 0
    pos[-1] = 16383
    q, k, p = to_dev(q_st), to_dev(k_st), to_dev(pos)
    fllayer.rope(dtype, q, k, p, T, nh, nkv, d, theta=10000.0)
    torch.cuda.synchronize()
    for got_t, xv, st in ((q, qv, q_st), (k, kv, k_st)):
        want = lo.round_store(lo.rope(xv, pos, 10000.0), dtype)[1]
        got = lo.load(to_np(got_t, st.dtype), dtype)
        # the rotation adds two products: allow the element type's spacing at the larger operand
        tol = ULP[dtype] * np.maximum(np.abs(xv).max(axis=-1, keepdims=True) * (8.0 if dtype == "f32" else 1.5), 2.0 ** -14) + 1e-6
        assert (np.abs(got - want) <= tol).all(), float(np.abs(got - want).max())
    assert np.array_equal(to_np(q, q_st.dtype)[0], q_st[0])           # position 0 leaves the row as it is
    # q alone / k alone
    q2 = to_dev(q_st)
    fllayer.rope(dtype, q2, None, p, T, nh, nkv, d)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(q2, q_st.dtype), to_np(q, q_st.dtype))


@pytest.mark.parametrize("dtype,T,M", [("f16", 33, 11008), ("bf16", 7, 13824), ("f32", 5, 128)])
def test_silu_mul(dtype, T, M):
    import torch
    rng = np.random.default_rng(M)
    g_st, gv = lo.round_store(rng.normal(0, 3, (T, M)), dtype)
    u_st, uv = lo.round_store(rng.normal(0, 1, (T, M)), dtype)
    gv[0, :4] = [0.0, 30.0, -30.0, -90.0]
    g_st = lo.round_store(gv, dtype)[0]
    g, u = to_dev(g_st), to_dev(u_st)
    out = torch.zeros_like(g)
    fllayer.silu_mul(dtype, g, u, out, T, M)
    torch.cuda.synchronize()
    want = lo.round_store(lo.silu_mul(gv, uv), dtype)[1]
    got = lo.load(to_np(out, g_st.dtype), dtype)
    tol = ULP[dtype] * np.maximum(np.abs(want), 2.0 ** -14) * (16.0 if dtype == "f32" else 1.01) + 4e-7 * np.abs(want) + 1e-30
    assert (np.abs(got - want) <= tol).all(), float(np.abs(got - want).max())
    # in place, and from the two halves of one tensor
    both = to_dev(np.concatenate([g_st, u_st], axis=1))
    fllayer.silu_mul(dtype, both, both.view(-1)[M:], both, T, M, ld_gate=2 * M, ld_up=2 * M, ld_out=2 * M)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(both, g_st.dtype)[:, :M], to_np(out, g_st.dtype))


def layer_cfg(dtype, **kw):
    base = dict(name="layer_" + dtype, dtype=dtype, hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128,
                n_dev_blocks=900, n_host_blocks=8, n_adapters=5, ranks=(8, 16), projections=("q", "k", "v", "o", "gate", "up", "down"),
                n_seqs=6, prefix_range=(0, 200), new_range=(1, 90), mlp_dim=1024, seed=41)
    base.update(kw)
    return wl.LayerConfig(**base)


def make_weights(cfg, rng):
    W = {"in_norm": rng.normal(1, 0.1, cfg.hidden), "post_norm": rng.normal(1, 0.1, cfg.hidden)}
    for n in ("q", "k", "v", "o", "gate", "up", "down"):
        d_in, d_out = cfg.proj_dims(n)
        W[n] = rng.normal(0, 1 / math.sqrt(d_in), (d_out, d_in))
    return {k: lo.round_store(v, cfg.dtype)[0] for k, v in W.items()}


LAYER_CASES = {
    "f16_prefill": lambda: layer_cfg("f16"),
    "bf16_gqa_mixed": lambda: layer_cfg("bf16", n_q_heads=8, n_kv_heads=2, hidden=1024, decode_frac=0.5, seed=42),
    "f32_small": lambda: layer_cfg("f32", n_seqs=3, prefix_range=(0, 60), new_range=(1, 20), hidden=256, n_q_heads=2,
                                   n_kv_heads=2, mlp_dim=512, n_dev_blocks=300, seed=43),
    # LoRA on the attention projections only (the 7B workload): the MLP projections are dense products alone
    "bf16_attention_lora_only": lambda: layer_cfg("bf16", projections=("q", "k", "v", "o"), seed=45),
    # enough tokens for the matrix-core LoRA and attention kernels
    "f16_long": lambda: layer_cfg("f16", n_seqs=10, prefix_range=(0, 300), new_range=(100, 160), n_dev_blocks=2500, seed=44),
    # over 1024 tokens, no LoRA on the MLP and 25 x 5 tiles of 128 features x 256 tokens: gate, up and the gated SiLU
    # run as one pass of the large-batch GEMM (the last feature tile is half filled: 3136 = 24.5 x 128)
    "f16_fused_gate_up": lambda: layer_cfg("f16", projections=("q", "k", "v", "o"), n_seqs=10, prefix_range=(0, 300),
                                           new_range=(110, 160), mlp_dim=3136, n_dev_blocks=2500, seed=47),
    # 3000 tokens and more, hidden 2048: 12 x 8 tiles of 256 x 256 for q, k, v, o, so the LoRA branch of those
    # projections is added inside the large-batch GEMM (weights as [d_out, d_in]); down takes the plain large-batch GEMM
    "f16_lora_inside_gemm": lambda: layer_cfg("f16", hidden=2048, n_q_heads=16, n_kv_heads=16,
                                              projections=("q", "k", "v", "o"), n_seqs=24, prefix_range=(0, 200),
                                              new_range=(125, 150), mlp_dim=3136, n_dev_blocks=2500, seed=49),
    # the same size with LoRA on all seven projections: gate and up each get their branch inside the one gated pass,
    # down (input width 3136) inside its own product
    "bf16_all_lora_inside_gemm": lambda: layer_cfg("bf16", hidden=2048, n_q_heads=16, n_kv_heads=16, n_seqs=24,
                                                   prefix_range=(0, 200), new_range=(125, 150), mlp_dim=3136,
                                                   n_dev_blocks=3500, ranks=(8, 16, 32), seed=50),
    # the same in fp16, where the composed layer's bound (8 spacings) is 7.8e-3: tight enough that a missing rank-8
    # branch on gate or up (delta of standard deviation ~0.03 before the down projection) cannot pass
    "f16_all_lora_inside_gemm": lambda: layer_cfg("f16", hidden=2048, n_q_heads=16, n_kv_heads=16, n_seqs=24,
                                                  prefix_range=(0, 200), new_range=(125, 150), mlp_dim=3136,
                                                  n_dev_blocks=3500, ranks=(8, 16, 32), seed=51),
    "bf16_fused_gate_up": lambda: layer_cfg("bf16", projections=("q", "k", "v", "o"), n_seqs=10, prefix_range=(0, 300),
                                            new_range=(110, 160), mlp_dim=3136, n_dev_blocks=2500, seed=48),
}


@pytest.mark.parametrize("name", list(LAYER_CASES))
def test_layer_forward_matches_composed_oracle(name):
    import torch
    cfg = LAYER_CASES[name]()
    step = wl.make_step(cfg)
    T = step.n_tokens
    print("\n[layer case %s] T=%d" % (name, T), flush=True)
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    W = make_weights(cfg, np.random.default_rng(7))
    h0_st, _ = lo.round_store(np.random.default_rng(8).normal(0, 1, (T, cfg.hidden)), cfg.dtype)
    pos = np.concatenate([step.prefix_len[i] + np.arange(step.cu_new[i + 1] - step.cu_new[i])
                          for i in range(cfg.n_seqs)]).astype(np.int32)
    Wd = {k: to_dev(v) for k, v in W.items()}
    layer = fllayer.Layer(g.pool, cfg.hidden, cfg.n_q_heads, cfg.mlp_dim, Wd)
    batch = fllayer.Batch(step.cu_new, step.prefix_len, to_dev(pos), g.kv_tables, g.token_adapter, g.rank, g.scale,
                          g.lora_tables, g.proj, n_adapters=len(step.rank), max_rank=int(step.rank.max()),
                          max_blocks_per_seq=step.kv_tables.shape[1])
    nbytes = layer.scratch_bytes(T)
    scratch = torch.zeros(nbytes + 256, dtype=torch.uint8, device="cuda")
    sp = (scratch.data_ptr() + 255) & ~255
    h = to_dev(h0_st)
    layer.forward(batch, h, sp, nbytes)
    torch.cuda.synchronize()
    got = lo.load(to_np(h, h0_st.dtype), cfg.dtype)

    pool_o = dev0.copy()
    want_st, inter = lo.layer_forward(cfg, step, pool_o, W, h0_st, pos)
    want = lo.load(want_st, cfg.dtype)
    # Tolerance.  Each of the ~12 tensors between the steps is rounded to the element type on both sides; where
    # the two sides' unrounded values straddle a rounding boundary they differ by one spacing, and later steps
    # carry that on.  The residual stream has magnitude ~1-3, so a few spacings of it bound the difference:
    # 8 spacings at the value (relative) plus 8 spacings at 1 (absolute).
    # fp32 pools: the tensors are not rounded to a coarser type, the difference is the fp32 summation order of the
    # kernels against float64: the tolerance of the fp32 parity tests (rel 1e-4 + abs 1e-5).
    rtol, atol = (1e-4, 1e-5) if cfg.dtype == "f32" else (8 * ULP[cfg.dtype], 8 * ULP[cfg.dtype])
    ok, worst, nbad = close(got, want, rtol, atol)
    assert ok, "h: max err %g, %d of %d out of tolerance" % (worst, nbad, got.size)
    # the layer did something: both residual branches are far above the tolerance
    h0 = lo.load(h0_st, cfg.dtype)
    assert np.abs(want - h0).max() > 10 * atol
    # the pool received the rotated keys and the values: compare the appended blocks with the oracle's pool
    img = g.dev_image()
    fresh = step.fresh_block_ids
    if cfg.dtype == "f32":
        assert np.allclose(img[fresh], pool_o[fresh], rtol=1e-4, atol=1e-5, equal_nan=True)
    else:
        a, b = lo.load(img[fresh], cfg.dtype), lo.load(pool_o[fresh], cfg.dtype)
        m = np.isfinite(a) & np.isfinite(b)
        assert (np.isfinite(a) == np.isfinite(b)).all()
        assert np.abs(a[m] - b[m]).max() <= 4 * ULP[cfg.dtype] * max(1.0, np.abs(b[m]).max())


def test_two_layer_stack_with_per_layer_pools():
    """Two layers, each with its own pool (the same block ids and tables in both) and its own weights: the second
    layer's input is the first one's residual stream; each layer appends its K/V to its own pool."""
    import torch
    from paper_2505_03756_amd import flpool
    from paper_2505_03756_amd.harness import GpuPool
    cfg = layer_cfg("f16", seed=46)
    step = wl.make_step(cfg)
    T = step.n_tokens
    dev0 = resident_pool(step)
    stub = np.zeros((1, cfg.block_elems), dev0.dtype)
    g = GpuStep(step, dev0, stub)
    gp1 = GpuPool(cfg, dev0, stub)                                     # layer 1's pool: same blocks at the same ids
    W = [make_weights(cfg, np.random.default_rng(70 + l)) for l in range(2)]
    h0_st, _ = lo.round_store(np.random.default_rng(9).normal(0, 1, (T, cfg.hidden)), cfg.dtype)
    pos = np.concatenate([step.prefix_len[i] + np.arange(step.cu_new[i + 1] - step.cu_new[i])
                          for i in range(cfg.n_seqs)]).astype(np.int32)
    pools = [g.pool, gp1.pool]
    layers = [fllayer.Layer(pools[l], cfg.hidden, cfg.n_q_heads, cfg.mlp_dim, {k: to_dev(v) for k, v in W[l].items()})
              for l in range(2)]
    batch = fllayer.Batch(step.cu_new, step.prefix_len, to_dev(pos), g.kv_tables, g.token_adapter, g.rank, g.scale,
                          g.lora_tables, g.proj, n_adapters=len(step.rank), max_rank=int(step.rank.max()),
                          max_blocks_per_seq=step.kv_tables.shape[1])
    nbytes = layers[0].scratch_bytes(T)
    scratch = torch.zeros(nbytes + 256, dtype=torch.uint8, device="cuda")
    sp = (scratch.data_ptr() + 255) & ~255
    h = to_dev(h0_st)
    for ly in layers:
        ly.forward(batch, h, sp, nbytes)
    torch.cuda.synchronize()
    got = lo.load(to_np(h, h0_st.dtype), cfg.dtype)
    want_st, pools_o = h0_st, [dev0.copy(), dev0.copy()]
    for l in range(2):
        want_st, _ = lo.layer_forward(cfg, step, pools_o[l], W[l], want_st, pos)
    want = lo.load(want_st, cfg.dtype)
    ok, worst, nbad = close(got, want, 16 * ULP[cfg.dtype], 16 * ULP[cfg.dtype])     # two layers: twice one layer's bound
    assert ok, "h: max err %g, %d of %d out of tolerance" % (worst, nbad, got.size)
    # each pool holds its own layer's keys: the two layers appended different K rows to the same block ids
    fresh = step.fresh_block_ids
    img0, img1 = g.dev_image()[fresh], to_np(gp1.dev, dev0.dtype)[fresh]
    assert not np.array_equal(img0, img1)
    a, b = lo.load(img1, cfg.dtype), lo.load(pools_o[1][fresh], cfg.dtype)
    m = np.isfinite(a) & np.isfinite(b)
    assert (np.isfinite(a) == np.isfinite(b)).all() and np.abs(a[m] - b[m]).max() <= 16 * ULP[cfg.dtype] * max(1.0, np.abs(b[m]).max())


@pytest.mark.parametrize("workload,n_oracle_seqs", [("7b_prefill", 2), ("7b_decode", 6), ("13b", 2), ("34b_gqa", 3)])
def test_layer_full_size_against_the_oracle_on_a_few_sequences(workload, n_oracle_seqs):
    """One decoder layer at the benchmark's sizes.  7B shapes (hidden 4096, 32 heads, MLP 11008, LoRA on q, k, v, o):
    the 18 953-token prefill batch on the 4 GiB pool (large-batch GEMMs with the LoRA branch and the gate inside) and
    the 256-token decode batch over contexts of 512-4096 (split small-batch GEMMs, per-token LoRA kernels); half of
    the 13B batch (rank 32 on seven projections: gate and up with their branches in one gated pass) and a quarter of the 34B
    batch (grouped-query attention, rank 64, prefill and decode sequences mixed, contexts up to 16 k).  A
    token's output depends only on its own sequence, so the oracle runs the layer on a few of the sequences and their
    rows of the GPU's full-batch result are compared."""
    import types
    import torch
    from paper_2505_03756_amd.harness import SparseGpuPool, compact_step
    cfg = wl.config(workload)
    if workload == "7b_decode":
        cfg = cfg.scaled(n_dev_blocks=40000)
    elif workload == "13b":         # hidden 5120, MLP 13824, rank 32 on all seven projections; half of the sequences
        cfg = cfg.scaled(n_seqs=64, n_dev_blocks=65536, n_host_blocks=32768)
    elif workload == "34b_gqa":     # hidden 8192, 64 query / 8 kv heads, MLP 22016, rank 64; a quarter of the sequences
        cfg = cfg.scaled(n_seqs=128, n_dev_blocks=200000, n_host_blocks=32768)
    step = wl.make_step(cfg)
    T = step.n_tokens
    gp = SparseGpuPool(step)
    g = GpuStep(step, gpool=gp)
    pool_c, kv_c, lt_c = compact_step(step)
    g.pool.swap_in(step.swap_in_host, step.swap_in_dev)
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    H, qd, kd = cfg.hidden, cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    mlp = cfg.mlp_dim or {4096: 11008, 8192: 22016}[H]
    dims = {"q": (qd, H), "k": (kd, H), "v": (kd, H), "o": (H, qd), "gate": (mlp, H), "up": (mlp, H), "down": (H, mlp)}
    W = {"in_norm": rng.normal(1, 0.1, H), "post_norm": rng.normal(1, 0.1, H)}
    for n, (d_out, d_in) in dims.items():
        W[n] = rng.standard_normal((d_out, d_in), dtype=np.float32) / np.float32(math.sqrt(d_in))
    W = {k: lo.round_store(v, cfg.dtype)[0] for k, v in W.items()}
    h0_st, _ = lo.round_store(rng.standard_normal((T, H), dtype=np.float32), cfg.dtype)
    pos = np.concatenate([step.prefix_len[i] + np.arange(step.cu_new[i + 1] - step.cu_new[i])
                          for i in range(cfg.n_seqs)]).astype(np.int32)
    layer = fllayer.Layer(g.pool, H, cfg.n_q_heads, mlp, {k: to_dev(v) for k, v in W.items()})
    batch = fllayer.Batch(step.cu_new, step.prefix_len, to_dev(pos), g.kv_tables, g.token_adapter, g.rank, g.scale,
                          g.lora_tables, g.proj, n_adapters=len(step.rank), max_rank=int(step.rank.max()),
                          max_blocks_per_seq=step.kv_tables.shape[1])
    nbytes = layer.scratch_bytes(T)
    scratch = torch.zeros(nbytes + 256, dtype=torch.uint8, device="cuda")
    h = to_dev(h0_st)
    layer.forward(batch, h, (scratch.data_ptr() + 255) & ~255, nbytes)
    torch.cuda.synchronize()
    got_all = to_np(h, h0_st.dtype)

    # the oracle on the longest-context sequence, the last one (whose rows end the batch's last, partly filled tile)
    # and, for the decode batch, a few more
    seqs = sorted({int(np.argmax(step.prefix_len + np.diff(step.cu_new))), cfg.n_seqs - 1} |
                  set(int(i) for i in rng.choice(cfg.n_seqs, size=n_oracle_seqs - 2, replace=False)))
    rows = np.concatenate([np.arange(step.cu_new[i], step.cu_new[i + 1]) for i in seqs])
    lens = np.array([step.cu_new[i + 1] - step.cu_new[i] for i in seqs])
    sub = types.SimpleNamespace(n_tokens=int(lens.sum()), proj={n: step.proj[n] for n in cfg.projections},
                                token_adapter=step.token_adapter[rows], rank=step.rank, scale=step.scale,
                                lora_tables=lt_c, cu_new=np.concatenate([[0], np.cumsum(lens)]).astype(np.int32),
                                prefix_len=step.prefix_len[seqs], kv_tables=np.ascontiguousarray(kv_c[seqs]))
    want_st, _ = lo.layer_forward(cfg, sub, pool_c, W, h0_st[rows], pos[rows])
    got, want = lo.load(got_all[rows], cfg.dtype), lo.load(want_st, cfg.dtype)
    ok, worst, nbad = close(got, want, 8 * ULP[cfg.dtype], 8 * ULP[cfg.dtype])
    assert ok, "h: max err %g, %d of %d out of tolerance" % (worst, nbad, got.size)
    assert np.abs(want - lo.load(h0_st[rows], cfg.dtype)).max() > 1.0
    gp.pool.close()
