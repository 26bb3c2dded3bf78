"""The step that bench.py times, against the oracle.  A scaled-down trace-driven workload (the benchmark's own class:
the same trace, metadata uploads, planner requests and library calls, fewer slots and blocks) runs a few steps; the
state before the last step is copied out, and what that step leaves behind (y of every projection, the appended K/V,
the attention output) is compared with the oracle run on the copy.  The adapter scale is raised for the test so that
a missing or misplaced branch is far outside the tolerance."""
import os
import sys

import numpy as np
import pytest

import oracle
from helpers import TOL, close
from paper_2505_03756_amd import workload as wl

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CASES = [
    # workload, overrides, steps before the checked one, sampled tokens
    ("7b_prefill", ["--seqs", "6", "--dev-blocks", "4096", "--host-blocks", "2048"], 3, 96),
    ("34b_gqa", ["--seqs", "24", "--dev-blocks", "49152", "--host-blocks", "65536"], 4, 64),
    ("7b_decode", ["--seqs", "24", "--dev-blocks", "8192", "--host-blocks", "64"], 2, 24),
    ("tiny", [], 3, 64),
]


@pytest.mark.parametrize("name,over,warm,n_sample", CASES, ids=[c[0] for c in CASES])
def test_benchmarked_step_matches_the_oracle(name, over, warm, n_sample, monkeypatch):
    import torch
    sys.path.insert(0, ROOT)
    import bench
    monkeypatch.setattr(sys, "argv", ["bench.py", "--workload", name, "--no-cpu-baseline", "--layers", "0"] + over)
    args = bench.parse()
    torch.cuda.set_device(0)
    b = bench.Bench(name, args)
    try:
        cfg, trc = b.cfg, b.trace
        s = 0.5 / float(np.sqrt(max(cfg.ranks) * cfg.hidden))         # a branch of half of y's spread
        b.d_scales = [torch.full((cfg.n_adapters,), v, dtype=torch.float32, device="cuda") for v in (s, -s)]
        # the o projection's input, the attention output, is an average of value rows and much smaller than x: its
        # call gets a larger scale of its own
        s_o = 16 * s
        scales_o = [torch.full((cfg.n_adapters,), v, dtype=torch.float32, device="cuda") for v in (s_o, -s_o)]
        lora_o = b.lora_o

        def lora_o_scaled(st_, stream):
            keep, b.d_scales = b.d_scales, scales_o
            try:
                lora_o(st_, stream)
            finally:
                b.d_scales = keep

        b.lora_o = lora_o_scaled
        b.reset_pipeline()
        b.run(warm, timed=False)
        torch.cuda.synchronize()

        def to_np(t, _sd=None):               # the benchmark's tensors are typed; the oracle takes the stored bits
            if t.dtype == torch.float32:
                return t.detach().cpu().numpy()
            return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)

        sd = wl.storage_dtype(cfg.dtype)
        before = {n: to_np(t, sd).copy() for n, t in b.ys.items()}
        pool0 = to_np(b.dev, sd).copy()
        x = to_np(b.x, sd)
        st = b.run(1, timed=False)[0]["st"]
        torch.cuda.synchronize()
        T = st.n_tokens
        assert T > 0
        sign = 1.0 if (b.n_lora_calls & 1) == 0 else -1.0
        after = {n: to_np(t, sd) for n, t in b.ys.items()}
        attn = to_np(b.attn_out, sd)
        pool1 = to_np(b.dev, sd)
        rng = np.random.default_rng(11)
        sel = np.sort(rng.choice(T, size=min(T, n_sample), replace=False)).astype(np.int32)
        rtol, atol = TOL[cfg.dtype]

        def check_lora(n, xin, s_call):
            pr = trc.proj[n]
            scale = np.full(cfg.n_adapters, sign * s_call, np.float32)
            want = oracle.lora_apply(pool0, cfg.dtype, np.ascontiguousarray(xin[:T]), st.token_adapter, st.rank, scale,
                                     pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, st.lora_tables,
                                     pr.d_out, y_in=np.ascontiguousarray(before[n][:T]), sel=sel)
            got = wl.dequantize(after[n][sel], cfg.dtype)
            ok, worst, nbad = close(got, want, rtol, atol)
            assert ok, "%s: max err %g, %d elements out of tolerance" % (n, worst, nbad)
            delta = np.abs(want - wl.dequantize(before[n][sel], cfg.dtype)).mean()
            assert delta > 10 * atol or cfg.dtype == "f32", "the branch of %s is too small to be seen: %g" % (n, delta)

        for n in b.names_qkv:
            check_lora(n, x, s)
        # K/V append: the step's own k and v rows into the blocks of its tables, bit for bit
        want_pool = pool0.copy()
        oracle.kv_append(want_pool, cfg.dtype, cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, st.cu_new, st.prefix_len,
                         st.kv_tables, np.ascontiguousarray(after["k"][:T]), np.ascontiguousarray(after["v"][:T]))
        used = np.unique(st.kv_tables[st.kv_tables >= 0])
        assert np.array_equal(pool1[used], want_pool[used]), "appended K/V differ"
        assert not np.array_equal(pool1[used], pool0[used]), "nothing was appended"
        # attention over the appended pool
        want = oracle.paged_attention(want_pool, cfg.dtype, cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim,
                                      cfg.n_q_heads, st.cu_new, st.prefix_len, st.kv_tables,
                                      np.ascontiguousarray(after["q"][:T]), sel=sel)
        got = wl.dequantize(attn[sel], cfg.dtype).reshape(want.shape)
        ok, worst, nbad = close(got, want, rtol, atol)
        assert ok, "attention: max err %g, %d elements out of tolerance" % (worst, nbad)
        if "o" in cfg.projections:
            check_lora("o", attn, s_o)
        # the moves of the run arrived: every block that a later step's tables name holds finite values
        assert np.isfinite(wl.dequantize(pool1[used], cfg.dtype)).all()
    finally:
        b.close()


PIPE_CASES = [
    ("7b_prefill", ["--seqs", "6", "--dev-blocks", "4096", "--host-blocks", "2048"], 8),
    ("13b", ["--seqs", "6", "--dev-blocks", "4096", "--host-blocks", "2048"], 8),
    ("34b_gqa", ["--seqs", "24", "--dev-blocks", "49152", "--host-blocks", "65536", "--early-moves-gb", "0.02"], 12),
]


@pytest.mark.parametrize("name,over,steps", PIPE_CASES, ids=[c[0] for c in PIPE_CASES])
def test_pipelined_steps_equal_the_same_steps_on_one_stream(name, over, steps, monkeypatch):
    """The benchmark's pipeline (moves issued by the planner on their own streams beside the compute, requests
    handed over before or after the first stages of a step, the host two steps ahead) against the same trace with
    every operation on ONE stream: after the same number of steps both tiers and every activation buffer hold the
    same bits.  An ordering mistake (a fetch into a block that a running step still reads, a write-back that starts
    before the append, a table upload that overtakes a kernel) shows up as a difference."""
    import torch
    sys.path.insert(0, ROOT)
    import bench

    def run(extra):
        monkeypatch.setattr(sys, "argv", ["bench.py", "--workload", name, "--no-cpu-baseline", "--layers", "0"] + over + extra)
        args = bench.parse()
        torch.cuda.set_device(0)
        torch.manual_seed(20250611)                       # the tiers and activations are drawn on the device
        b = bench.Bench(name, args)
        try:
            b.reset_pipeline()
            recs = b.run(steps, timed=False)
            torch.cuda.synchronize()
            bits = lambda t: t.detach().view(torch.int16).cpu().numpy().copy()
            out = {n: bits(t) for n, t in b.ys.items()}
            out["attn_out"] = bits(b.attn_out)
            out["dev"] = bits(b.dev)
            out["host"] = bits(b.host)
            moved = sum(len(r["st"].swap_in_dev) + len(r["st"].swap_out_dev) for r in recs)
            return out, moved
        finally:
            b.close()

    piped, moved = run([])
    serial, moved2 = run(["--one-stream"])
    assert moved == moved2 and moved > 0
    for key in piped:
        assert np.array_equal(piped[key], serial[key]), "%s differs between the pipelined and the one-stream run" % key
