"""flp_lora_apply_paged_static (the entry point that allocates nothing: its intermediates live in a fixed device
array) against flp_lora_apply_paged, through the C ABI: the two run the same kernels on the same inputs, so their
outputs must agree bit for bit (and both within tolerance of the oracle).  Two calls in a row on the shared array,
the second with a smaller input, then a third on another pool; a batch that does not fit is refused."""
import numpy as np
import pytest

import oracle
from helpers import TOL, GpuStep, close, resident_pool, to_dev
from paper_2505_03756_amd import flpool
from paper_2505_03756_amd import workload as wl

pytestmark = pytest.mark.gpu


def _cfg(dtype, **kw):
    base = dict(name="noalloc_" + dtype, dtype=dtype, hidden=512, n_q_heads=4, n_kv_heads=4, head_dim=128,
                n_dev_blocks=1500, n_host_blocks=4, n_adapters=6, ranks=(8, 16, 32), projections=("q", "k", "v", "o"),
                n_seqs=7, prefix_range=(0, 0), new_range=(1, 70), swap_in_frac=0.0, seed=501)
    base.update(kw)
    return wl.LayerConfig(**base)


def _both(step, names, w_base=None):
    cfg = step.cfg
    dev0 = resident_pool(step)
    g = GpuStep(step, dev0, np.zeros((4, cfg.block_elems), dev0.dtype))
    wb = {n: to_dev(w_base[n]) for n in names} if w_base else None
    want = g.lora(names, w_base=wb)
    got = g.lora(names, w_base=wb, static=True)
    rtol, atol = TOL[cfg.dtype]
    for n in names:
        assert np.array_equal(got[n], want[n]), "%s: static and allocating entry points differ" % n
        pr = step.proj[n]
        ref = oracle.lora_apply(dev0, cfg.dtype, step.acts["x"], step.token_adapter, step.rank, step.scale,
                                pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables, pr.d_out,
                                y_in=None if w_base else step.acts["base_" + n], w_base=w_base[n] if w_base else None)
        ok, worst, nbad = close(wl.dequantize(got[n], cfg.dtype), ref, rtol, atol)
        assert ok, "%s: max err %g (%d bad)" % (n, worst, nbad)
        if not w_base:
            base = wl.dequantize(step.acts["base_" + n], cfg.dtype)
            assert np.abs(ref - base).max() > 10 * atol, "the case carries no delta"
    g.pool.close()


def test_static_entry_point_matches_on_two_calls_in_a_row():
    assert flpool.static_scratch_bytes() == 64 << 20
    # 1) a prefill batch on the 32-token tiles with a dense base that is small enough to fit (large-batch GEMM with
    #    the LoRA branch inside: transposed base matrix, inverse permutation and segment lists in the array)
    big = wl.make_step(_cfg("f16", n_q_heads=18, n_kv_heads=18, n_seqs=24, new_range=(110, 160), ranks=(8, 16),
                            seed=502))
    assert big.n_tokens >= 2048
    rng = np.random.default_rng(5)
    W = {n: wl.quantize((rng.standard_normal((512, big.proj[n].d_out)) / np.sqrt(512)).astype(np.float32), "f16")
         for n in ("q", "k", "v")}
    _both(big, ["q", "k", "v"], w_base=W)
    # 2) right after it a smaller one without a base: the array still holds the first call's bits
    mid = wl.make_step(_cfg("f16", n_seqs=30, new_range=(40, 90), ranks=(16, 32), seed=503))
    assert 1024 <= mid.n_tokens < big.n_tokens
    _both(mid, ["q", "k", "v"])
    _both(mid, ["o"])
    # 3) and a decode batch (per-token kernels, mixed ranks, bf16) on yet another pool
    small = wl.make_step(_cfg("bf16", n_seqs=97, new_range=(1, 1), decode_frac=1.0, n_adapters=20,
                              ranks=(8, 16, 32, 64), seed=504))
    assert small.n_tokens == 97
    _both(small, ["q", "k", "v"])


def test_static_entry_point_refuses_what_does_not_fit():
    """A dense base at 20 000 tokens needs the unrounded product beside y (hundreds of MB): refused with FLP_ENOSPC
    before anything runs; y is untouched."""
    import torch
    cfg = _cfg("f16", hidden=1024, n_q_heads=8, n_kv_heads=8)
    pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, 64, 4)
    T = 1000                                         # small-batch GEMM: keeps 4 * T * d_out bytes per projection
    x = torch.zeros((T, 16384), dtype=torch.int16, device="cuda")
    y = torch.full((T, 16384), 7, dtype=torch.int16, device="cuda")
    w = torch.zeros((16384, 16384), dtype=torch.int16, device="cuda")
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    proj = dict(y=y, d_out=16384, w_base=w, a_tab_off=z, a_row_base=z, b_tab_off=z, b_row_base=z)
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(x, torch.full((T,), -1, dtype=torch.int32, device="cuda"), z,
                              torch.zeros(4, device="cuda"), z, [proj], n_tokens=T, d_in=16384, n_adapters=4,
                              max_rank=8, static=True)
    assert e.value.code == flpool.FLP_ENOSPC and "fixed buffer" in str(e.value)
    torch.cuda.synchronize()
    assert bool((y == 7).all())
    pool.close()
