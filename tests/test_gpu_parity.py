"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

import oracle
from helpers import TOL, GpuStep, build_pools, close, resident_pool, to_dev, to_np
from paper_2505_03756_amd import flpool
from paper_2505_03756_amd import workload as wl

pytestmark = pytest.mark.gpu


def small_cfg(dtype, **kw):
    base = dict(name="small_" + dtype, dtype=dtype, hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128,
                n_dev_blocks=400, n_host_blocks=512, n_adapters=6, ranks=(8, 16, 32), projections=("q", "k", "v", "o"),
                n_seqs=7, prefix_range=(0, 300), new_range=(1, 70), swap_in_frac=0.4, seed=77)
    base.update(kw)
    return wl.LayerConfig(**base)


CASES = {
    "tiny": lambda: wl.config("tiny"),
    "f16_prefill": lambda: small_cfg("f16"),
    "bf16_decode": lambda: small_cfg("bf16", n_seqs=19, prefix_range=(1, 700), new_range=(1, 1), decode_frac=1.0,
                                     n_dev_blocks=1200, seed=78),
    "bf16_gqa_mixed": lambda: small_cfg("bf16", n_q_heads=8, n_kv_heads=2, hidden=1024, decode_frac=0.5,
                                        prefix_range=(0, 500), seed=79),
    "f16_d64": lambda: small_cfg("f16", head_dim=64, n_q_heads=8, n_kv_heads=8, seed=80),
    "bf16_d64_gqa": lambda: small_cfg("bf16", head_dim=64, n_q_heads=8, n_kv_heads=4, decode_frac=0.4, seed=93),
    "f32_d128": lambda: small_cfg("f32", n_seqs=4, prefix_range=(0, 120), new_range=(1, 40), seed=81),
    # blocks of 32 token positions (the block size of the paper's vLLM baseline, section 2.2) as a layout variant:
    # prefill on the matrix-core kernel, decode / mixed and fp32 on the row kernel, head_dim 64
    "f16_prefill_bt32": lambda: small_cfg("f16", block_tokens=32, seed=91),
    "bf16_gqa_mixed_bt32": lambda: small_cfg("bf16", block_tokens=32, n_q_heads=8, n_kv_heads=2, hidden=1024,
                                             decode_frac=0.5, prefix_range=(0, 500), seed=92),
    "bf16_decode_bt32": lambda: small_cfg("bf16", block_tokens=32, n_seqs=19, prefix_range=(1, 700), new_range=(1, 1),
                                          decode_frac=1.0, n_dev_blocks=1200, seed=93),
    "f32_d64_bt32": lambda: small_cfg("f32", block_tokens=32, head_dim=64, n_q_heads=8, n_kv_heads=8, n_seqs=4,
                                      prefix_range=(0, 120), new_range=(1, 40), seed=94),
}


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    cfg = CASES[request.param]()
    step = wl.make_step(cfg)
    print("\n[case %s] T=%d S=%d dtype=%s" % (request.param, step.n_tokens, cfg.n_seqs, cfg.dtype), flush=True)
    return step


def test_swap_in_out_bit_exact(case):
    step, cfg = case, case.cfg
    dev0, host0 = build_pools(step, poison_rest=True)
    g = GpuStep(step, dev0, host0)
    # oracle
    dev_ref, host_ref = dev0.copy(), host0.copy()
    oracle.swap(host_ref, dev_ref, step.swap_out_dev, step.swap_out_host)
    oracle.swap(dev_ref, host_ref, step.swap_in_host, step.swap_in_dev)
    # library: swap-out first, then swap-in (the order the paper gives when the device tier is full)
    g.pool.swap_out(step.swap_out_dev, step.swap_out_host)
    g.pool.swap_in(step.swap_in_host, step.swap_in_dev)
    assert np.array_equal(g.dev_image().view(np.uint8), dev_ref.view(np.uint8))
    assert np.array_equal(g.host_image().view(np.uint8), host_ref.view(np.uint8))
    # after the swap-in every needed block is resident with its content
    assert np.array_equal(g.dev_image()[step.content_ids].view(np.uint8), step.content.view(np.uint8))


def test_swap_round_trip_every_block():
    cfg = wl.config("tiny")
    rng = np.random.default_rng(5)
    dev0 = rng.standard_normal((cfg.n_dev_blocks, cfg.block_elems)).astype(np.float32)
    host0 = np.zeros((cfg.n_dev_blocks, cfg.block_elems), np.float32)
    step = wl.make_step(cfg, with_acts=False)
    g = GpuStep(step, dev0, host0)
    ids = np.arange(cfg.n_dev_blocks, dtype=np.int32)
    perm, back = rng.permutation(ids).astype(np.int32), rng.permutation(ids).astype(np.int32)
    g.pool.swap_out(ids, perm)
    assert np.array_equal(g.host_image()[perm], dev0)
    g.dev.zero_()
    g.pool.swap_in(perm, back)
    assert np.array_equal(g.dev_image()[back], dev0)


def test_kv_append_bit_exact(case):
    step, cfg = case, case.cfg
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    ref = dev0.copy()
    oracle.kv_append(ref, cfg.dtype, cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, step.cu_new, step.prefix_len,
                     step.kv_tables, step.acts["k_new"], step.acts["v_new"])
    g.pool.kv_append(g.acts["k_new"], g.acts["v_new"], step.cu_new, step.prefix_len, g.kv_tables)
    assert np.array_equal(g.dev_image().view(np.uint8), ref.view(np.uint8))


def test_attention_matches_oracle(case):
    step, cfg = case, case.cfg
    dev0 = resident_pool(step)       # fresh blocks hold NaN patterns until the append fills their slots
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    got = wl.dequantize(g.attention(append=True), cfg.dtype).reshape(step.n_tokens, cfg.n_q_heads, cfg.head_dim)
    ref_pool = dev0.copy()
    oracle.kv_append(ref_pool, cfg.dtype, cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, step.cu_new,
                     step.prefix_len, step.kv_tables, step.acts["k_new"], step.acts["v_new"])
    want = oracle.paged_attention(ref_pool, cfg.dtype, cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads,
                                  step.cu_new, step.prefix_len, step.kv_tables, step.acts["q"])
    rtol, atol = TOL[cfg.dtype]
    ok, worst, nbad = close(got, want, rtol, atol)
    assert ok, "max err %g, %d elements out of tolerance" % (worst, nbad)
    # second entry form: K/V already appended, k_new = v_new = NULL
    got2 = wl.dequantize(g.attention(append=False), cfg.dtype).reshape(got.shape)
    assert np.array_equal(got, got2)


def test_lora_matches_oracle(case):
    step, cfg = case, case.cfg
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    groups = [[p for p in cfg.projections if p in ("q", "k", "v")], [p for p in cfg.projections if p == "o"]]
    for names in groups:
        if not names:
            continue
        x_key = "x" if names[0] != "o" or cfg.proj_dims("o")[0] == cfg.hidden else "x_%d" % cfg.proj_dims("o")[0]
        got = g.lora(names, x_key=x_key)
        for n in names:
            pr = step.proj[n]
            want = oracle.lora_apply(dev0, cfg.dtype, step.acts[x_key], step.token_adapter, step.rank, step.scale,
                                     pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                     pr.d_out, y_in=step.acts["base_" + n])
            ok, worst, nbad = close(wl.dequantize(got[n], cfg.dtype), want, rtol, atol)
            assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
            delta = np.abs(want - wl.dequantize(step.acts["base_" + n], cfg.dtype)).max()
            assert delta > 10 * atol or cfg.dtype == "f32"      # the test would notice a missing delta


LORA_CASES = {
    # T >= 2048 selects the 32-token tiles; rank 16 -> one rank tile; Zipf gives one long segment and a tail
    "f16_long_segments": lambda: small_cfg("f16", hidden=1024, n_q_heads=8, n_kv_heads=8, n_seqs=24,
                                           prefix_range=(0, 0), new_range=(40, 180), n_adapters=12, ranks=(16,),
                                           adapter_dist="zipf", n_dev_blocks=600, swap_in_frac=0.0, seed=82),
    # ranks 8..64 mixed -> four rank tiles with partially filled ones; many short segments, 16-token tiles
    "bf16_mixed_rank": lambda: small_cfg("bf16", hidden=1024, n_q_heads=8, n_kv_heads=8, n_seqs=200,
                                         prefix_range=(0, 0), new_range=(2, 11), n_adapters=60,
                                         ranks=(8, 16, 32, 64), n_dev_blocks=2500, swap_in_frac=0.0, seed=83),
    # the same shapes as a small decode batch (per-token kernels)
    "bf16_mixed_rank_decode": lambda: small_cfg("bf16", hidden=1024, n_q_heads=8, n_kv_heads=8, n_seqs=200,
                                                prefix_range=(0, 0), new_range=(1, 1), decode_frac=1.0,
                                                n_adapters=60, ranks=(8, 16, 32, 64), n_dev_blocks=2500,
                                                swap_in_frac=0.0, seed=83),
    # rank 64 with 32-token tiles and a k/v width different from q/o (grouped-query shapes)
    # the paper's LoRA distributions at 1000-2000 LoRAs (section 6.9): adapters handed out in turn (every
    # sequence its own adapter, hundreds of short segments in one tiled launch), ...
    "f16_distinct_2000": lambda: small_cfg("f16", hidden=1024, n_q_heads=8, n_kv_heads=8, n_seqs=300,
                                           prefix_range=(0, 0), new_range=(2, 40), n_adapters=2000, ranks=(16,),
                                           adapter_dist="distinct", n_dev_blocks=4000, swap_in_frac=0.0, seed=85),
    # ... uniform over 2000 (almost all distinct), mixed ranks ...
    "bf16_uniform_2000": lambda: small_cfg("bf16", hidden=1024, n_q_heads=8, n_kv_heads=8, n_seqs=260,
                                           prefix_range=(0, 0), new_range=(1, 24), n_adapters=2000,
                                           ranks=(8, 16, 32, 64), adapter_dist="uniform", n_dev_blocks=6000,
                                           swap_in_frac=0.0, seed=86),
    # ... and a Gaussian over the ids (a few dozen adapters carry the batch), as a decode batch
    "bf16_skewed_1000_decode": lambda: small_cfg("bf16", hidden=1024, n_q_heads=8, n_kv_heads=8, n_seqs=700,
                                                 prefix_range=(0, 0), new_range=(1, 1), decode_frac=1.0,
                                                 n_adapters=1000, ranks=(16, 32), adapter_dist="skewed", skew_std=12.0,
                                                 n_dev_blocks=6000, swap_in_frac=0.0, seed=87),
    # over 1024 tokens with output widths that are not multiples of the large GEMM tile (q, o: 320 of 256; k, v: 64)
    "bf16_dense_tail": lambda: small_cfg("bf16", hidden=320, n_q_heads=5, n_kv_heads=1, head_dim=64, n_seqs=20,
                                         prefix_range=(0, 0), new_range=(40, 80), n_adapters=4, ranks=(16,),
                                         n_dev_blocks=1200, swap_in_frac=0.0, seed=88),
    # enough 256 x 256 tiles (11 token rows x 9 feature columns; 9.5 columns in the bf16 case) for the large-batch GEMM
    # when a dense base is given
    "f16_dense_large": lambda: small_cfg("f16", hidden=512, n_q_heads=18, n_kv_heads=18, n_seqs=24, prefix_range=(0, 0),
                                         new_range=(110, 160), n_adapters=6, ranks=(8, 16), n_dev_blocks=1500,
                                         swap_in_frac=0.0, seed=89),
    "bf16_dense_large_tail": lambda: small_cfg("bf16", hidden=512, n_q_heads=19, n_kv_heads=19, n_seqs=24,
                                               prefix_range=(0, 0), new_range=(110, 160), n_adapters=6, ranks=(16, 32),
                                               n_dev_blocks=1500, swap_in_frac=0.0, seed=90),
    "f16_rank64_gqa": lambda: small_cfg("f16", hidden=1024, n_q_heads=8, n_kv_heads=2, n_seqs=38,
                                        prefix_range=(0, 0), new_range=(30, 120), n_adapters=5, ranks=(64,),
                                        n_dev_blocks=1500, swap_in_frac=0.0, seed=84),
}


@pytest.mark.parametrize("name", list(LORA_CASES))
def test_lora_matrix_core_shapes(name):
    cfg = LORA_CASES[name]()
    step = wl.make_step(cfg)
    print("\n[lora case %s] T=%d adapters=%d" % (name, step.n_tokens, int((step.rank > 0).sum())), flush=True)
    if name in ("f16_long_segments", "f16_rank64_gqa", "f16_dense_large", "bf16_dense_large_tail"):
        assert step.n_tokens >= 2048, "this case is meant for the 32-token tiles"
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    got = g.lora(["q", "k", "v"])
    got.update(g.lora(["o"]))
    for n in ("q", "k", "v", "o"):
        pr = step.proj[n]
        want = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                 pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                 pr.d_out, y_in=step.acts["base_" + n])
        ok, worst, nbad = close(wl.dequantize(got[n], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
        # the delta itself (not just base + delta) must be right: compare it at a tolerance scaled to its size
        base = wl.dequantize(step.acts["base_" + n], cfg.dtype)
        ulp = 2.0 ** (-10 if cfg.dtype == "f16" else -7)
        err = np.abs((wl.dequantize(got[n], cfg.dtype) - base) - (want - base))
        assert err.max() <= ulp * (np.abs(want).max() + 1.0), (n, err.max())


@pytest.mark.parametrize("dtype,ranks", [("f16", (16,)), ("bf16", (8, 32, 64))])
def test_lora_long_batch_with_input_width_not_a_multiple_of_64(dtype, ranks):
    """32-token tiles (2048 tokens and more) with an input width of 288 = 9 x 32: the LDS-staged shrink kernels need
    whole 64-coefficient chunks, so this batch takes the shrink kernel that reads its operands from global memory."""
    cfg = small_cfg(dtype, hidden=288, n_q_heads=4, n_kv_heads=2, n_seqs=24, prefix_range=(0, 0), new_range=(90, 140),
                    n_adapters=7, ranks=ranks, n_dev_blocks=1200, swap_in_frac=0.0, seed=94)
    step = wl.make_step(cfg)
    assert step.n_tokens >= 2048 and step.proj["q"].d_in == 288
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    got = g.lora(["q", "k", "v"])
    for n in ("q", "k", "v"):
        pr = step.proj[n]
        want = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                 pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                 pr.d_out, y_in=step.acts["base_" + n])
        ok, worst, nbad = close(wl.dequantize(got[n], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
        base = wl.dequantize(step.acts["base_" + n], cfg.dtype)
        assert np.abs(want - base).max() > 10 * atol


@pytest.mark.parametrize("case", ["f16_long_segments", "bf16_dense_large_tail", "f16_rank64_gqa"])
@pytest.mark.parametrize("names", [("q", "k"), ("q", "k", "v", "o"), ("v",)])
def test_lora_call_with_one_two_or_four_projections(names, case):
    """The staged shrink kernels are compiled per number of projections in the call (they share x): calls with 1, 2
    and 4 projections on a batch long enough for the 32-token tiles (q, k, v together is covered above), at ranks
    up to 16, up to 32 and at 64 (one, two and four rank tiles; at 64 a workgroup takes two token tiles).  All
    projections read the same x here, "o" included where its input is as wide: the call does not care what x
    means."""
    cfg = LORA_CASES[case]()
    step = wl.make_step(cfg)
    assert step.n_tokens >= 2048 and cfg.hidden % 64 == 0
    assert int(step.rank.max()) == {"f16_long_segments": 16, "bf16_dense_large_tail": 32, "f16_rank64_gqa": 64}[case]
    names = tuple(n for n in names if step.proj[n].d_in == cfg.hidden)
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    got = g.lora(list(names))
    for n in names:
        pr = step.proj[n]
        assert pr.d_in == cfg.hidden
        want = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                 pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                 pr.d_out, y_in=step.acts["base_" + n])
        ok, worst, nbad = close(wl.dequantize(got[n], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
        base = wl.dequantize(step.acts["base_" + n], cfg.dtype)
        ulp = 2.0 ** (-10 if cfg.dtype == "f16" else -7)
        err = np.abs((wl.dequantize(got[n], cfg.dtype) - base) - (want - base))
        assert err.max() <= ulp * (np.abs(want).max() + 1.0), (n, err.max())
        assert np.abs(want - base).max() > 10 * atol


@pytest.mark.parametrize("dtype,T", [("bf16", 1), ("bf16", 63), ("f32", 257), ("bf16", 1023), ("f16", 1024),
                                     ("f32", 1025)])
def test_lora_small_batches_share_adapter_pages(dtype, T):
    """The per-token kernels take the tokens of one adapter four at a time (batches of up to 1024 tokens): batches
    around that limit and around the 64-token words of the kernels' bit mask, with adapters that own one token, a
    few, or a third of the batch, tokens without an adapter, and widths that do not fill the column slabs."""
    cfg = small_cfg(dtype, hidden=320, n_q_heads=5, n_kv_heads=1, head_dim=64, n_seqs=T, prefix_range=(0, 0),
                    new_range=(1, 1), decode_frac=1.0, n_adapters=40, ranks=(8, 16, 32, 64), n_dev_blocks=2600,
                    swap_in_frac=0.0, seed=300 + T)
    step = wl.make_step(cfg)
    rng = np.random.default_rng(T)
    ta = step.token_adapter.copy()
    if T > 8:
        ta[rng.choice(T, size=T // 3, replace=False)] = 3               # one heavy adapter: many fours
        ta[rng.choice(T, size=T // 10, replace=False)] = -1             # tokens without an adapter
        ta[T - 1] = 3
    step.token_adapter = ta
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    got = g.lora(["q", "k", "v"])
    got.update(g.lora(["o"]))
    for n in ("q", "k", "v", "o"):
        pr = step.proj[n]
        want = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], ta, step.rank, step.scale, pr.a_tab_off,
                                 pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables, pr.d_out,
                                 y_in=step.acts["base_" + n])
        ok, worst, nbad = close(wl.dequantize(got[n], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
        base = wl.dequantize(step.acts["base_" + n], cfg.dtype)
        none = ta < 0
        if none.any():                                                   # rows without an adapter are untouched
            assert np.array_equal(got[n][none], step.acts["base_" + n][none])
        assert np.abs(want - base)[~none].max() > 0


@pytest.mark.parametrize("name", ["tiny", "f16_prefill", "bf16_gqa_mixed", "f16_long_segments", "bf16_dense_tail",
                                  "f16_dense_large", "bf16_dense_large_tail"])
def test_lora_with_dense_base(name):
    """w_base given: y = x.W_base + delta, the library computes the base term itself (Eq. 1's W)."""
    cfg = (CASES.get(name) or LORA_CASES[name])()
    step = wl.make_step(cfg)
    rng = np.random.default_rng(55)
    if "large" in name:
        # tokens without an adapter inside the batch: one whole sequence, and single tokens inside other sequences
        # (the LoRA branch is added inside the GEMM there, per adapter present among a wave's 128 tokens)
        ta = step.token_adapter.copy()
        ta[step.cu_new[3]:step.cu_new[4]] = -1
        ta[rng.choice(step.n_tokens, size=50, replace=False)] = -1
        ta[step.cu_new[7] + 5:step.cu_new[7] + 9] = step.token_adapter[step.cu_new[9]]   # another sequence's adapter mid-sequence
        step.token_adapter = ta
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    names = [p for p in cfg.projections if p in ("q", "k", "v")]
    W = {n: wl.quantize((rng.standard_normal((cfg.hidden, step.proj[n].d_out)) / np.sqrt(cfg.hidden)).astype(np.float32),
                        cfg.dtype) for n in names}
    got = g.lora(names, w_base={n: to_dev(W[n]) for n in names})
    # a random sample, both ends of every sequence (where the adapter changes inside a tile) and the end of the batch
    T = step.n_tokens
    sel = np.unique(np.concatenate([rng.choice(T, size=min(T, 64), replace=False), step.cu_new[:-1],
                                    step.cu_new[1:] - 1, np.arange(max(0, T - 40), T)])).astype(np.int32)
    if "large" in name:
        sel = np.unique(np.concatenate([sel, np.flatnonzero(step.token_adapter < 0)[:60],
                                        np.arange(step.cu_new[7], step.cu_new[7] + 12)])).astype(np.int32)
    sel = sel[(sel >= 0) & (sel < T)]
    for n in names:
        pr = step.proj[n]
        want = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                 pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                 pr.d_out, w_base=W[n], sel=sel)
        ok, worst, nbad = close(wl.dequantize(got[n][sel], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
        assert np.abs(want).max() > 1.0          # the base term is really there


def test_segmentation_bit_exact():
    import torch
    rng = np.random.default_rng(9)
    pool = flpool.Pool("f16", 1, 64, 2, 0)
    for T, n_ad in [(1, 1), (63, 5), (64, 5), (1000, 40), (5000, 300), (20000, 2048), (257, 100)]:
        ta = rng.integers(-1, n_ad, size=T).astype(np.int32)
        if T > 100:
            ta[rng.integers(0, T, size=T // 2)] = rng.integers(0, min(3, n_ad))      # a few heavy adapters
        seg_adapter, seg_start, perm = oracle.segment(ta, n_ad)
        d_ta = to_dev(ta)
        d_nseg = torch.zeros(1, dtype=torch.int32, device="cuda")
        d_sa = torch.full((n_ad,), -7, dtype=torch.int32, device="cuda")
        d_ss = torch.full((n_ad + 1,), -7, dtype=torch.int32, device="cuda")
        d_perm = torch.full((T,), -7, dtype=torch.int32, device="cuda")
        pool.lora_segment(d_ta, T, n_ad, d_nseg, d_sa, d_ss, d_perm)
        torch.cuda.synchronize()
        n = int(d_nseg.item())
        assert n == len(seg_adapter)
        assert np.array_equal(d_sa.cpu().numpy()[:n], seg_adapter)
        assert np.array_equal(d_ss.cpu().numpy()[:n + 1], seg_start)
        assert np.array_equal(d_perm.cpu().numpy()[:seg_start[n]], perm)


def test_degenerate_batches():
    import torch
    cfg = small_cfg("f16", n_seqs=5, prefix_range=(64, 64), new_range=(16, 16), seed=90)
    step = wl.make_step(cfg)
    # sequences with zero new tokens, zero prefix, a single token, a prefix ending on a block boundary
    step.prefix_len[:] = [0, 16, 33, 0, 48]
    step.new_len[:] = [1, 0, 5, 17, 16]
    step.cu_new[1:] = np.cumsum(step.new_len)
    T = int(step.cu_new[-1])
    for k in ("q", "k_new", "v_new"):
        step.acts[k] = step.acts[k][:T].copy()
    dev0 = resident_pool(step)
    dev0[step.content_ids] = wl.quantize(np.random.default_rng(1).standard_normal(step.content.shape), "f16")
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    got = wl.dequantize(g.attention(append=True), "f16").reshape(T, cfg.n_q_heads, cfg.head_dim)
    ref_pool = dev0.copy()
    oracle.kv_append(ref_pool, "f16", 16, cfg.n_kv_heads, cfg.head_dim, step.cu_new, step.prefix_len, step.kv_tables,
                     step.acts["k_new"], step.acts["v_new"])
    want = oracle.paged_attention(ref_pool, "f16", 16, cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads, step.cu_new,
                                  step.prefix_len, step.kv_tables, step.acts["q"])
    ok, worst, nbad = close(got, want, *TOL["f16"])
    assert ok, (worst, nbad)
    # P = 0, N = 1: the output is exactly v0 (softmax over a single key)
    v0 = wl.dequantize(step.acts["v_new"][0], "f16").reshape(cfg.n_kv_heads, cfg.head_dim)
    assert np.array_equal(got[0], v0)
    # empty batch and all-empty sequences enqueue nothing and succeed
    g.pool.paged_prefix_attention(g.acts["q"], g.acts["q"], [0], [], g.kv_tables, cfg.n_q_heads)
    g.pool.paged_prefix_attention(g.acts["q"], g.acts["q"], [0, 0, 0], [3, 4], g.kv_tables, cfg.n_q_heads)
    g.pool.swap_in([], [])
    torch.cuda.synchronize()


def test_lora_no_adapter_tokens_and_zero_b():
    cfg = small_cfg("bf16", seed=91)
    step = wl.make_step(cfg)
    step.token_adapter[::3] = -1
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    got = g.lora(["q"])["q"]
    none = np.flatnonzero(step.token_adapter < 0)
    assert np.array_equal(got[none], step.acts["base_q"][none])           # untouched rows, bit for bit
    pr = step.proj["q"]
    want = oracle.lora_apply(dev0, "bf16", step.acts["x"], step.token_adapter, step.rank, step.scale, pr.a_tab_off,
                             pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables, pr.d_out,
                             y_in=step.acts["base_q"])
    ok, worst, nbad = close(wl.dequantize(got, "bf16"), want, *TOL["bf16"])
    assert ok, (worst, nbad)
    # B = 0 for every adapter: y is the base term exactly
    zero = dev0.copy()
    for a in np.flatnonzero(step.rank):
        for rho in range(step.rank[a]):
            oracle.lora_write_row(zero, "bf16", step.lora_tables[pr.b_tab_off[a]:], pr.b_row_base[a] + rho,
                                  np.zeros(pr.d_out, np.uint16))
    g2 = GpuStep(step, zero, np.zeros((1, cfg.block_elems), dev0.dtype))
    assert np.array_equal(g2.lora(["q"])["q"], step.acts["base_q"])


@pytest.mark.parametrize("with_base", [False, True])
@pytest.mark.parametrize("dtype,ranks", [("f16", (16,)), ("bf16", (32,)), ("f16", (64,)), ("bf16", (8, 16, 32, 64))])
def test_lora_adapters_drawn_per_token(dtype, ranks, with_base):
    """Every token draws its adapter on its own (12 adapters and "none"), so a 32-token tile of the sorted batch, a
    256-token tile group and the 128 tokens of a GEMM wave all mix adapters, segments end inside tiles, and rows
    without an adapter sit between the others: on the tiled path (2816 tokens and more), without a dense base
    (shrink and expand kernels) and with one (the LoRA branch inside the large-batch GEMM), at one, two and four
    rank tiles and with mixed ranks."""
    cfg = small_cfg(dtype, hidden=512, n_q_heads=18, n_kv_heads=18, n_seqs=24, prefix_range=(0, 0),
                    new_range=(118, 160), n_adapters=12, ranks=ranks, adapter_dist="distinct", n_dev_blocks=2400,
                    swap_in_frac=0.0, seed=120 + len(ranks) + ranks[0])
    step = wl.make_step(cfg)                    # "distinct" over 24 sequences: all 12 adapters get pages
    T = step.n_tokens
    assert T >= 2816 and int((step.rank > 0).sum()) == 12
    rng = np.random.default_rng(ranks[0])
    step.token_adapter = rng.integers(-1, 12, size=T).astype(np.int32)
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    rtol, atol = TOL[cfg.dtype]
    names = ["q", "k", "v"]
    W = None
    if with_base:
        W = {n: wl.quantize((rng.standard_normal((cfg.hidden, step.proj[n].d_out)) / np.sqrt(cfg.hidden))
                            .astype(np.float32), cfg.dtype) for n in names}
    got = g.lora(names, w_base={n: to_dev(W[n]) for n in names} if W else None)
    sel = np.arange(T, dtype=np.int32) if not with_base else np.unique(np.concatenate(
        [rng.choice(T, size=300, replace=False), np.arange(0, 140), np.arange(T - 140, T)])).astype(np.int32)
    none = step.token_adapter < 0
    assert none.sum() > 100
    ulp = 2.0 ** (-10 if cfg.dtype == "f16" else -7)
    for n in names:
        pr = step.proj[n]
        want = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                 pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                 pr.d_out, y_in=None if W else step.acts["base_" + n], w_base=W[n] if W else None,
                                 sel=sel)
        ok, worst, nbad = close(wl.dequantize(got[n][sel], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
        if not W:
            base = wl.dequantize(step.acts["base_" + n], cfg.dtype)
            assert np.array_equal(got[n][none], step.acts["base_" + n][none])     # rows without an adapter untouched
            err = np.abs((wl.dequantize(got[n], cfg.dtype) - base) - (want - base))
            assert err.max() <= ulp * (np.abs(want).max() + 1.0), (n, err.max())
            assert np.abs(want - base)[~none].max() > 10 * atol
        else:
            # the branch is there: rows with an adapter differ from the dense product alone by more than the bound
            dense = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], np.full(T, -1, np.int32), step.rank, step.scale,
                                      pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                      pr.d_out, w_base=W[n], sel=sel)
            with_ad = ~none[sel]
            assert np.abs(want - dense)[with_ad].max() > 10 * atol
            # compare the branch itself at one spacing of the element type at the output's magnitude plus the
            # rounding of the sum
            err = np.abs((wl.dequantize(got[n][sel], cfg.dtype) - dense) - (want - dense))
            assert err.max() <= 1.5 * ulp * (np.abs(want).max() + 1.0), (n, err.max())


@pytest.mark.parametrize("dtype,bt,gqa", [("f16", 16, False), ("bf16", 16, True), ("f16", 32, False)])
def test_attention_over_shared_prefix_blocks(dtype, bt, gqa):
    """Sequences of one adapter share the physical blocks of a common prefix (paper section 4.1; KV of different
    LoRAs is never shared, section 2.1): block ids repeat across tables.  Append writes only the sequences' own
    blocks; attention reads the shared ones from every table that names them.  Prefill rows (matrix-core kernel)
    and, in the grouped-query case, decode rows mixed in."""
    kw = dict(n_q_heads=8, n_kv_heads=2, hidden=1024, decode_frac=0.4) if gqa else {}
    cfg = small_cfg(dtype, block_tokens=bt, n_seqs=24, n_adapters=3, prefix_range=(40, 420), new_range=(1, 90),
                    share_frac=0.85, n_dev_blocks=1500, swap_in_frac=0.0, seed=131 + bt + gqa, **kw)
    step = wl.make_step(cfg)
    ids, counts = np.unique(step.kv_tables[step.kv_tables >= 0], return_counts=True)
    assert (counts > 1).sum() >= 20 and counts.max() >= 3, "the case shares too little"
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    n_kv, d, n_h = cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads
    out = g.attention(append=True)
    ref = dev0.copy()
    oracle.kv_append(ref, cfg.dtype, bt, n_kv, d, step.cu_new, step.prefix_len, step.kv_tables, step.acts["k_new"],
                     step.acts["v_new"])
    assert np.array_equal(g.dev_image().view(np.uint8), ref.view(np.uint8)), "append touched a shared block"
    shared = ids[counts > 1]
    assert np.array_equal(ref[shared], dev0[shared])                      # shared blocks are prefix blocks: unchanged
    want = oracle.paged_attention(ref, cfg.dtype, bt, n_kv, d, n_h, step.cu_new, step.prefix_len, step.kv_tables,
                                  step.acts["q"])
    ok, worst, nbad = close(wl.dequantize(out, cfg.dtype).reshape(want.shape), want, *TOL[cfg.dtype])
    assert ok, "max err %g (%d bad)" % (worst, nbad)


@pytest.mark.parametrize("dtype,heads,kv,d,seqs,prefix,new", [
    ("bf16", 32, 32, 128, 3, (3000, 9000), (1, 1)),       # a handful of decode sequences with long contexts
    ("f16", 8, 8, 64, 2, (2000, 5000), (1, 1)),
    ("f32", 4, 4, 128, 2, (1500, 2500), (1, 1)),
    ("bf16", 16, 2, 128, 4, (4000, 12000), (1, 1)),       # grouped-query decode: too few matrix-core items, rows + split
    ("f16", 8, 8, 128, 5, (100, 6000), (1, 3)),           # short and long contexts mixed, up to three new tokens
])
def test_split_kv_for_few_long_sequences(dtype, heads, kv, d, seqs, prefix, new):
    """Few rows over long contexts: the context of a row is cut into pieces, a wave each, and the pieces are merged in
    a fixed order (the split-KV form of the same softmax).  Against the oracle, and twice for identical bits."""
    cfg = small_cfg(dtype, hidden=heads * d, n_q_heads=heads, n_kv_heads=kv, head_dim=d, n_seqs=seqs,
                    prefix_range=prefix, new_range=new, decode_frac=1.0 if new == (1, 1) else 0.0, n_adapters=2,
                    ranks=(8,), projections=("q",), n_dev_blocks=seqs * (prefix[1] // 16 + 3) + 64, swap_in_frac=0.0,
                    seed=500 + heads + seqs)
    step = wl.make_step(cfg)
    assert step.n_tokens * heads < 2048                        # under the kernel's fill: the split path is taken
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((1, cfg.block_elems), dev0.dtype))
    out1 = g.attention(append=True)
    out2 = g.attention(append=False)                           # the fresh K/V are in place: same inputs, same bits
    assert np.array_equal(out1, out2)
    ref = dev0.copy()
    oracle.kv_append(ref, dtype, 16, kv, d, step.cu_new, step.prefix_len, step.kv_tables, step.acts["k_new"],
                     step.acts["v_new"])
    want = oracle.paged_attention(ref, dtype, 16, kv, d, heads, step.cu_new, step.prefix_len, step.kv_tables,
                                  step.acts["q"])
    ok, worst, nbad = close(wl.dequantize(out1, dtype).reshape(want.shape), want, *TOL[dtype])
    assert ok, "max err %g (%d bad)" % (worst, nbad)
