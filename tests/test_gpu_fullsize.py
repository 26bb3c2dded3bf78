"""GPU parity at the benchmark's full sizes: every integer / byte result compared in full, the
floating-point results on seeded samples of tokens that the oracle computes one by one.
The launch configuration is the one bench.py times (same entry points, same kernels)."""
import numpy as np
import pytest

import oracle
from helpers import TOL, GpuStep, SparseGpuPool, close, compact_step, to_dev
from paper_2505_03756_amd import workload as wl

pytestmark = pytest.mark.gpu


def _run_case(cfg, n_sample_tokens, seed=None):
    import torch
    step = wl.make_step(cfg, seed=seed)
    T = step.n_tokens
    rng = np.random.default_rng(12345)
    rtol, atol = TOL[cfg.dtype]
    gp = SparseGpuPool(step)
    g = GpuStep(step, gpool=gp)
    pool_c, kv_c, lt_c = compact_step(step)             # what the device tier must hold after the swap-in
    bt, n_kv, d, n_h = cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads

    # ---- swap: out first, then in; every touched block bit-exact afterwards
    out_before = gp.rows(step.swap_out_dev) if len(step.swap_out_dev) else None
    g.pool.swap_out(step.swap_out_dev, step.swap_out_host)
    g.pool.swap_in(step.swap_in_host, step.swap_in_dev)
    assert np.array_equal(gp.rows(step.content_ids).view(np.uint8), pool_c.view(np.uint8)), "swap-in"
    if out_before is not None:
        torch.cuda.synchronize()
        host_rows = gp.host.numpy()[step.swap_out_host].view(np.uint16 if cfg.dtype != "f32" else np.float32)
        assert np.array_equal(host_rows.view(np.uint8), out_before.view(np.uint8)), "swap-out"

    # ---- segmentation of the full batch, bit-exact
    n_ad = len(step.rank)
    d_nseg = torch.zeros(1, dtype=torch.int32, device="cuda")
    d_sa = torch.zeros(n_ad, dtype=torch.int32, device="cuda")
    d_ss = torch.zeros(n_ad + 1, dtype=torch.int32, device="cuda")
    d_perm = torch.zeros(T, dtype=torch.int32, device="cuda")
    g.pool.lora_segment(g.token_adapter, T, n_ad, d_nseg, d_sa, d_ss, d_perm)
    seg_adapter, seg_start, perm = oracle.segment(step.token_adapter, n_ad)
    n = int(d_nseg.item())
    assert n == len(seg_adapter)
    assert np.array_equal(d_sa.cpu().numpy()[:n], seg_adapter) and np.array_equal(d_ss.cpu().numpy()[:n + 1], seg_start)
    assert np.array_equal(d_perm.cpu().numpy()[:seg_start[n]], perm)

    # ---- LoRA: all projections at full size, sampled rows against the oracle
    sel = np.sort(rng.choice(T, size=min(T, n_sample_tokens), replace=False)).astype(np.int32)
    groups = {}
    for p in cfg.projections:
        groups.setdefault(step.proj[p].d_in, []).append(p)
    for d_in, names in groups.items():
        x_key = "x" if d_in == cfg.hidden else "x_%d" % d_in
        for lo in range(0, len(names), 3):
            chunk = names[lo:lo + 3]
            got = g.lora(chunk, x_key=x_key)
            for nme in chunk:
                pr = step.proj[nme]
                want = oracle.lora_apply(pool_c, cfg.dtype, step.acts[x_key], step.token_adapter, step.rank, step.scale,
                                         pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, lt_c, pr.d_out,
                                         y_in=step.acts["base_" + nme], sel=sel)
                ok, worst, nbad = close(wl.dequantize(got[nme][sel], cfg.dtype), want, rtol, atol)
                assert ok, "LoRA %s: max err %g (%d bad)" % (nme, worst, nbad)
                base = wl.dequantize(step.acts["base_" + nme][sel], cfg.dtype)
                assert np.abs(want - base).max() > 10 * atol, "sample carries no delta"

    # ---- KV append, bit-exact on every touched block
    g.pool.kv_append(g.acts["k_new"], g.acts["v_new"], step.cu_new, step.prefix_len, g.kv_tables)
    oracle.kv_append(pool_c, cfg.dtype, bt, n_kv, d, step.cu_new, step.prefix_len, kv_c, step.acts["k_new"],
                     step.acts["v_new"])
    assert np.array_equal(gp.rows(step.content_ids).view(np.uint8), pool_c.view(np.uint8)), "append"

    # ---- attention at full size, sampled tokens (all heads) against the oracle
    q = g.acts["q"]
    out = torch.zeros_like(q)
    g.pool.paged_prefix_attention(q, out, step.cu_new, step.prefix_len, g.kv_tables, n_h)
    torch.cuda.synchronize()
    # favour the ends of sequences (longest contexts, tile tails) and their starts (prefix seam)
    ends = step.cu_new[1:] - 1
    starts = step.cu_new[:-1]
    pick = np.unique(np.concatenate([rng.choice(ends, size=min(len(ends), n_sample_tokens // 3), replace=False),
                                     rng.choice(starts, size=min(len(starts), n_sample_tokens // 3), replace=False),
                                     sel[:n_sample_tokens // 3]])).astype(np.int32)
    got = wl.dequantize(out[torch.from_numpy(pick.astype(np.int64)).cuda()].cpu().numpy().view(
        np.uint16 if cfg.dtype != "f32" else np.float32), cfg.dtype).reshape(len(pick), n_h, d)
    want = oracle.paged_attention(pool_c, cfg.dtype, bt, n_kv, d, n_h, step.cu_new, step.prefix_len, kv_c,
                                  step.acts["q"], sel=pick)
    ok, worst, nbad = close(got, want, rtol, atol)
    assert ok, "attention: max err %g (%d bad)" % (worst, nbad)
    # property that holds at any size: every output row is finite (no poisoned slot leaked in)
    assert bool(torch.isfinite(out.view(torch.float16 if cfg.dtype == "f16" else torch.bfloat16)).all())
    gp.pool.close()


def test_7b_prefill_full_size():
    """Config 1 of the benchmark list (the one bench.py times): fp16, 64 prefill sequences, 40 % swap-in."""
    _run_case(wl.config("7b_prefill"), n_sample_tokens=48)


def test_7b_decode_full_size():
    """Config 2: bf16 decode, 256 sequences of 512-4096 context, 100 adapters of mixed rank."""
    _run_case(wl.config("7b_decode").scaled(n_dev_blocks=40000), n_sample_tokens=48)


def test_13b_shapes_in_full_size_pool():
    """Config 3 shapes (hidden 5120, 40 heads, MLP 13824, rank 32 on seven projections, Zipf 1.2) on a
    seeded subsample of 32 sequences, in a device tier of the full 600 000 x 320 KiB (197 GB), so that
    64-bit block offsets and page-rows that do not divide the block are exercised at real addresses."""
    _run_case(wl.config("13b").scaled(n_seqs=32, n_host_blocks=4096), n_sample_tokens=36)


def test_34b_gqa_shapes_in_full_size_pool():
    """Config 4 shapes (hidden 8192, 64 query / 8 kv heads, rank 64, prefixes up to 16384, 75 % decode) on a
    seeded subsample of 64 sequences, in a device tier of 3 000 000 x 64 KiB (197 GB)."""
    _run_case(wl.config("34b_gqa").scaled(n_seqs=64, n_dev_blocks=3000000, n_host_blocks=8192), n_sample_tokens=36)


def test_7b_prefill_dense_base_full_size():
    """The q, k, v call of the headline batch with the dense base computed by the library (w_base given): at this
    size the products take the large-batch GEMM and the LoRA branch is added inside it.  Sampled tokens (a random
    sample and both ends of every sequence) against the oracle."""
    import torch
    cfg = wl.config("7b_prefill")
    step = wl.make_step(cfg)
    T = step.n_tokens
    rng = np.random.default_rng(4321)
    rtol, atol = TOL[cfg.dtype]
    gp = SparseGpuPool(step)
    g = GpuStep(step, gpool=gp)
    pool_c, kv_c, lt_c = compact_step(step)
    g.pool.swap_in(step.swap_in_host, step.swap_in_dev)
    torch.cuda.synchronize()
    names = ["q", "k", "v"]
    W = {n: wl.quantize((rng.standard_normal((cfg.hidden, step.proj[n].d_out)) / np.sqrt(cfg.hidden)).astype(np.float32),
                        cfg.dtype) for n in names}
    got = g.lora(names, w_base={n: to_dev(W[n]) for n in names})
    sel = np.unique(np.concatenate([rng.choice(T, size=24, replace=False), step.cu_new[:-1][::4],
                                    step.cu_new[1:][::4] - 1, [T - 1]])).astype(np.int32)
    for n in names:
        pr = step.proj[n]
        want = oracle.lora_apply(pool_c, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                 pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, lt_c, pr.d_out,
                                 w_base=W[n], sel=sel)
        ok, worst, nbad = close(wl.dequantize(got[n][sel], cfg.dtype), want, rtol, atol)
        assert ok, "%s: max err %g (%d bad)" % (n, worst, nbad)
        assert np.abs(want).max() > 1.0
    gp.pool.close()
