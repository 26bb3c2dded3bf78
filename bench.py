#!/usr/bin/env python3
"""Benchmark of the paged multi-LoRA layer step on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
swap-in of the blocks that start on the host tier, batched LoRA on q/k/v (one
call, x read once), KV append, paged prefix attention, LoRA on o.  The base
projections x.W are taken as given (y arrives holding them); they are not part
of the path that is measured.

Prints ONE JSON line (see the keys at the bottom).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0    # dense fp16 / bf16 MFMA, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="7b_prefill")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--seed", type=int, default=None)
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "Run with --gpus 1; the value is that one GPU's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from helpers import GpuStep, build_pools
    from paper_2505_03756_amd import workload as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = wl.config(args.workload)
    if cfg.n_dev_blocks * cfg.block_bytes > 200 * 2 ** 30:
        raise SystemExit("workload %s does not fit this bench's host-side staging; use 7b_prefill or 7b_decode"
                         % args.workload)
    t0 = time.time()
    step = wl.make_step(cfg, seed=args.seed)
    T, S = step.n_tokens, cfg.n_seqs
    dev0, host0 = build_pools(step)
    g = GpuStep(step, dev0, host0)
    del dev0
    sys.stderr.write("[bench] workload %s: T=%d tokens, S=%d, %d KV+LoRA blocks, %d swapped in, setup %.1fs\n"
                     % (cfg.name, T, S, len(step.content_ids), len(step.swap_in_dev), time.time() - t0))

    names_qkv = [p for p in ("q", "k", "v") if p in cfg.projections]
    st = torch.cuda.current_stream()
    ys = {n: g.acts["base_" + n].clone() for n in cfg.projections}
    attn_out = torch.zeros_like(ys["q"])
    n_ad, max_rank = len(step.rank), int(max(1, step.rank.max()))
    pj = lambda n: dict(y=ys[n], d_out=step.proj[n].d_out, **g.proj[n])

    def stage_swap():
        g.pool.swap_out(step.swap_out_dev, step.swap_out_host, stream=st)
        g.pool.swap_in(step.swap_in_host, step.swap_in_dev, stream=st)

    def stage_lora_qkv():
        g.pool.lora_apply_paged(g.acts["x"], g.token_adapter, g.rank, g.scale, g.lora_tables,
                                [pj(n) for n in names_qkv], n_tokens=T, d_in=cfg.hidden, n_adapters=n_ad,
                                max_rank=max_rank, stream=st)

    def stage_append():
        g.pool.kv_append(ys["k"], ys["v"], step.cu_new, step.prefix_len, g.kv_tables, stream=st)

    def stage_attn():
        g.pool.paged_prefix_attention(ys["q"], attn_out, step.cu_new, step.prefix_len, g.kv_tables, cfg.n_q_heads,
                                      stream=st)

    def stage_lora_o():
        g.pool.lora_apply_paged(attn_out, g.token_adapter, g.rank, g.scale, g.lora_tables, [pj("o")], n_tokens=T,
                                d_in=cfg.n_q_heads * cfg.head_dim, n_adapters=n_ad, max_rank=max_rank, stream=st)

    stages = [("swap", stage_swap), ("lora_qkv", stage_lora_qkv), ("kv_append", stage_append),
              ("attention", stage_attn), ("lora_o", stage_lora_o)]

    def one_step():
        for _, f in stages:
            f()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps, per-stage HIP events on the launch stream
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    for k in range(args.steps):
        ev[k][0].record(st)
        for i, (_, f) in enumerate(stages):
            f()
            ev[k][i + 1].record(st)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {name: float(np.mean([ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(args.steps)]))
                for i, (name, _) in enumerate(stages)}

    # ---- algorithmic work of each stage
    e = wl.DTYPE_BYTES[cfg.dtype]
    L = step.prefix_len.astype(np.int64) + step.new_len
    N = step.new_len.astype(np.int64)
    P = step.prefix_len.astype(np.int64)
    n_h, n_kv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    attn_bytes = float(np.sum((L * 2 * n_kv + 2 * N * n_h) * d * e))
    attn_flops = float(np.sum(4.0 * n_h * d * N * (P + (N + 1) / 2.0)))
    swap_bytes = float((len(step.swap_in_dev) + len(step.swap_out_dev)) * cfg.block_bytes)
    append_bytes = float(2 * 2 * T * n_kv * d * e)
    active = np.flatnonzero(step.rank)
    def lora_bytes(names, d_in):
        b = T * d_in * e                                  # x, read once for all projections of the call
        for n in names:
            d_out = step.proj[n].d_out
            b += 2 * T * d_out * e                        # y read-modify-write
            b += float(np.sum(step.rank[active])) * (d_in + d_out) * e   # A and B pages of active adapters
            b += 2 * T * max_rank * 4                     # v written and read (fp32)
        return float(b)
    def lora_flops(names, d_in):
        r_tok = step.rank[step.token_adapter].astype(np.float64)
        return float(sum(2.0 * np.sum(r_tok) * (d_in + step.proj[n].d_out) for n in names))
    kernels = {
        "swap": {"bound": "pcie", "bytes": swap_bytes},
        "lora_qkv": {"bound": "hbm", "bytes": lora_bytes(names_qkv, cfg.hidden), "flops": lora_flops(names_qkv, cfg.hidden)},
        "kv_append": {"bound": "hbm", "bytes": append_bytes},
        "attention": {"bound": "hbm", "bytes": attn_bytes, "flops": attn_flops},
        "lora_o": {"bound": "hbm", "bytes": lora_bytes(["o"], n_h * d), "flops": lora_flops(["o"], n_h * d)},
    }
    for name, k in kernels.items():
        ms = stage_ms[name]
        k["ms"] = round(ms, 4)
        k["GBps"] = round(k["bytes"] / (ms * 1e6), 1) if ms > 0 else None
        if "flops" in k:
            k["TFLOPps"] = round(k["flops"] / (ms * 1e9), 2) if ms > 0 else None
        k["bytes"] = int(k["bytes"])
        if "flops" in k:
            k["flops"] = int(k["flops"])

    # dominant on-chip kernel = attention; which roofline binds it depends on the regime
    a = kernels["attention"]
    t_hbm = a["bytes"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = a["flops"] / (MFMA_PEAK_TFLOPS * 1e12)
    if cfg.dtype != "f32" and t_mfma > t_hbm:
        roof = {"bound": "mfma", "achieved": a["TFLOPps"], "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a["TFLOPps"] / MFMA_PEAK_TFLOPS, 4), "traffic": None, "kernel": "attention"}
    else:
        roof = {"bound": "hbm", "achieved": a["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(a["GBps"] / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "attention"}

    out = {
        "metric": "tokens/s of paged multi-LoRA layer step",
        "value": round(T / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "tokens_per_step": T, "n_seqs": S, "hidden": cfg.hidden,
                   "heads": "%dx%d (kv %d)" % (n_h, d, n_kv), "adapters": int(len(active)),
                   "ranks": sorted(set(int(r) for r in step.rank[active])),
                   "swap_in_blocks": int(len(step.swap_in_dev)), "block_bytes": cfg.block_bytes,
                   "base_gemm": "excluded (y arrives holding x.W)", "swap": "serialised with compute"},
        "roofline": roof,
        "kernels": kernels,
        "compute_only_tokens_per_s": round(T / (sum(v for k, v in stage_ms.items() if k != "swap") * 1e-3), 1),
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(step, args.cpu_seconds)
    print(json.dumps(out))


def cpu_baseline(step, target_s):
    """The oracle as it stands, timed on this machine's host cores over a bounded sample of the same
    step: for a random sample of tokens, every stage a token goes through (LoRA q/k/v/o rows and
    its attention row over the full context)."""
    import numpy as np
    import oracle
    from helpers import resident_pool
    from paper_2505_03756_amd import workload as wl
    cfg = step.cfg
    pool = resident_pool(step)
    bt, n_kv, d, n_h = cfg.block_tokens, cfg.n_kv_heads, cfg.head_dim, cfg.n_q_heads
    # the fresh K/V must be in the pool image before the attention rows are computed (not timed: a memcpy)
    oracle.kv_append(pool, cfg.dtype, bt, n_kv, d, step.cu_new, step.prefix_len, step.kv_tables,
                     step.acts["k_new"], step.acts["v_new"])
    rng = np.random.default_rng(7)
    T = step.n_tokens

    def run(sel):
        t0 = time.perf_counter()
        for n in cfg.projections:
            pr = step.proj[n]
            x = step.acts["x"] if pr.d_in == cfg.hidden else step.acts["x_%d" % pr.d_in]
            oracle.lora_apply(pool, cfg.dtype, x, step.token_adapter, step.rank, step.scale, pr.a_tab_off,
                              pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables, pr.d_out,
                              y_in=step.acts["base_" + n], sel=sel)
        oracle.paged_attention(pool, cfg.dtype, bt, n_kv, d, n_h, step.cu_new, step.prefix_len, step.kv_tables,
                               step.acts["q"], sel=sel)
        return time.perf_counter() - t0

    threads = oracle.num_threads()
    pilot = rng.choice(T, size=min(T, 2 * threads), replace=False).astype(np.int32)
    tp = run(pilot)
    n = int(min(T, max(len(pilot), len(pilot) * target_s / max(tp, 1e-3))))
    n -= n % threads if n > threads else 0
    sel = rng.choice(T, size=n, replace=False).astype(np.int32)
    dt = run(sel)
    return {"value": round(n / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d tokens of the same step (uniform, seeded): LoRA rows for %s and the attention row "
                      "over the full context, fp64, OpenMP over tokens; %.1f s" % (n, T, "/".join(cfg.projections), dt)}


if __name__ == "__main__":
    main()
