#!/usr/bin/env python3
"""Benchmark of the paged multi-LoRA layer step on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input:
swap-out / swap-in of the listed blocks between the pinned host tier and the
pool, batched LoRA on q/k/v (one call, x read once), KV append, paged prefix
attention, LoRA on o.  The base projections x.W are taken as given (y arrives
holding them); they are not part of the measured path.

The timed region runs K steps the way the method is meant to run (paper section
4.3, asynchronous swapping): the swap of a batch is enqueued on its own stream
and overlaps the compute of the previous batch; two batches with disjoint
blocks alternate.  `value` is tokens/s of that pipeline.  A second, serialised
pass (everything on one stream, HIP events between the stages) gives the
per-kernel durations that the roofline figures use.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# file (profiles/bench_7b_prefill_pmc.md), scaled by what the same counters read for a plain
# device-to-device copy of 1 GiB (FETCH_SIZE reads half the bytes, WRITE_SIZE all of them).  Only
# valid for the default workload and seed; null otherwise.
MEASURED_TRAFFIC = {("7b_prefill", 20250504): 1.682e9, ("7b_decode", 20250505): 1.0151e10}
MFMA_PEAK_TFLOPS = 2500.0    # dense fp16 / bf16 MFMA, published
PCIE_PEAK_GBS = 64.0         # PCIe Gen5 x16, one direction


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="7b_prefill")
    ap.add_argument("--swap-frac", type=float, default=None,
                    help="override the share of reusable blocks that arrive over the host link each step "
                         "(sweep for the break-even between swap and compute; the headline uses the workload's own)")
    ap.add_argument("--adapters", type=int, default=None, help="override the number of adapters (the paper's "
                    "1000 / 2000 LoRA experiment, section 6.9)")
    ap.add_argument("--adapter-dist", default=None, choices=["uniform", "zipf", "distinct", "skewed"],
                    help="override how sequences pick their adapter (section 6.9: uniform, distinct, skewed-x)")
    ap.add_argument("--skew-std", type=float, default=None, help="x of skewed-x, in adapter ids")
    ap.add_argument("--block-tokens", type=int, default=None, choices=[16, 32], help="token positions per pool block "
                    "(32: the block size of the paper's vLLM baseline, as a layout variant; the pool keeps its bytes)")
    ap.add_argument("--dev-blocks", type=int, default=None, help="override the pool's device block count (the 13b and "
                    "34b_gqa workloads name pools of 200-250 GB; a smaller pool that still holds the batch lets their "
                    "shapes be timed, several layers deep)")
    ap.add_argument("--host-blocks", type=int, default=None)
    ap.add_argument("--seqs", type=int, default=None, help="override the number of sequences; the new-token range "
                    "is scaled so that the step keeps its token count")
    ap.add_argument("--layers", type=int, default=2, help="decoder layers of the layer_stack section (0: skip); the "
                    "stack runs the batch through that many layers with per-layer pools and random weights")
    ap.add_argument("--mlp-dim", type=int, default=None, help="MLP width of the layer_stack section "
                    "(default: the workload's, else 11008 for hidden 4096)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--seed", type=int, default=None)
    return ap.parse_args()


class _Shared:
    pass


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "Run with --gpus 1; the value is that one GPU's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_03756_amd.harness import GpuStep, to_dev
    from paper_2505_03756_amd import flpool
    from paper_2505_03756_amd import workload as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = wl.config(args.workload)
    if args.swap_frac is not None:
        cfg = cfg.scaled(swap_in_frac=float(args.swap_frac))
    over = {}
    if args.adapters is not None:
        over["n_adapters"] = int(args.adapters)
    if args.adapter_dist is not None:
        over["adapter_dist"] = args.adapter_dist
    if args.skew_std is not None:
        over["skew_std"] = float(args.skew_std)
    if args.block_tokens is not None and args.block_tokens != cfg.block_tokens:
        f = args.block_tokens / float(cfg.block_tokens)
        over["block_tokens"] = int(args.block_tokens)
        over["n_dev_blocks"] = int(cfg.n_dev_blocks / f)
        over["n_host_blocks"] = int(cfg.n_host_blocks / f)
    if args.dev_blocks is not None:
        over["n_dev_blocks"] = int(args.dev_blocks)
    if args.host_blocks is not None:
        over["n_host_blocks"] = int(args.host_blocks)
    if args.seqs is not None and args.seqs != cfg.n_seqs:
        f = cfg.n_seqs / float(args.seqs)
        over["n_seqs"] = int(args.seqs)
        if cfg.decode_frac < 1.0:
            over["new_range"] = (max(1, int(round(cfg.new_range[0] * f))), max(1, int(round(cfg.new_range[1] * f))))
            over["prefix_range"] = (int(round(cfg.prefix_range[0] * f)), int(round(cfg.prefix_range[1] * f)))
    if over:
        cfg = cfg.scaled(**over)
    if cfg.n_dev_blocks * cfg.block_bytes > 200 * 2 ** 30:
        raise SystemExit("workload %s names a pool of %d GiB, a parity-test shape; time its kernels in a pool that "
                         "just holds the batch with --dev-blocks N (and --host-blocks)"
                         % (args.workload, cfg.n_dev_blocks * cfg.block_bytes >> 30))
    seed = cfg.seed if args.seed is None else args.seed
    t0 = time.time()

    # ---- the two tiers, the pool, and a shuffled free list (allocate all, free in a seeded order)
    tdt = torch.float32 if cfg.dtype == "f32" else torch.int16
    gp = _Shared()
    gp.cfg, gp.sd = cfg, wl.storage_dtype(cfg.dtype)
    gp.dev = torch.zeros((cfg.n_dev_blocks, cfg.block_elems), dtype=tdt, device="cuda")
    gp.host = torch.zeros((cfg.n_host_blocks, cfg.block_elems), dtype=tdt).pin_memory()
    gp.pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, cfg.n_dev_blocks, cfg.n_host_blocks,
                          block_tokens=cfg.block_tokens, dev=gp.dev, host=gp.host)
    rng = np.random.default_rng(seed)
    for tier, n in ((0, cfg.n_dev_blocks), (1, cfg.n_host_blocks)):
        ids = gp.pool.alloc(n, tier)
        gp.pool.free(rng.permutation(ids), tier)

    # ---- two batches with disjoint blocks (ids handed out by the library's allocator)
    n_sets = 2 if cfg.swap_in_frac > 0 or cfg.swap_out_frac > 0 else 1     # nothing to overlap without swaps
    sets = []
    host_np = gp.host.numpy()
    for i in range(n_sets):
        step = wl.make_step(cfg, seed=seed + 1000 * i, alloc_dev=lambda n: gp.pool.alloc(n, 0),
                            alloc_host=lambda n: gp.pool.alloc(n, 1))
        row_of = {int(b): r for r, b in enumerate(step.content_ids)}
        swapped = np.isin(step.content_ids, step.swap_in_dev)
        keep = np.flatnonzero(~swapped)
        for lo in range(0, len(keep), 512):
            sel = keep[lo:lo + 512]
            gp.dev[torch.from_numpy(step.content_ids[sel].astype(np.int64)).cuda()] = to_dev(step.content[sel])
        for h, d in zip(step.swap_in_host, step.swap_in_dev):
            host_np[h] = step.content[row_of[int(d)]].view(host_np.dtype)
        g = GpuStep(step, gpool=gp)
        step.content = None          # the images are on the tiers now
        sets.append(g)
    sys.stderr.write("[bench] workload %s: %s, setup %.1fs\n" % (
        cfg.name, "; ".join("batch %d: T=%d, %d blocks, %d swapped in" % (
            i, g.step.n_tokens, len(g.step.content_ids), len(g.step.swap_in_dev)) for i, g in enumerate(sets)),
        time.time() - t0))

    names_qkv = [p for p in ("q", "k", "v") if p in cfg.projections]
    qd = cfg.n_q_heads * cfg.head_dim

    class Runner:
        def __init__(self, g):
            self.g, self.step = g, g.step
            self.T = g.step.n_tokens
            self.ys = {n: g.acts["base_" + n].clone() for n in cfg.projections}
            # projections without a LoRA branch (the tiny config has q and v only): their base terms as they are
            for n, key in (("q", "q"), ("k", "k_new"), ("v", "v_new")):
                if n not in self.ys:
                    self.ys[n] = g.acts[key]
            self.attn_out = torch.zeros_like(self.ys["q"])
            self.n_ad, self.max_rank = len(g.step.rank), int(max(1, g.step.rank.max()))

        def pj(self, n):
            return dict(y=self.ys[n], d_out=self.step.proj[n].d_out, **self.g.proj[n])

        def swap(self, st):
            self.g.pool.swap_out(self.step.swap_out_dev, self.step.swap_out_host, stream=st)
            self.g.pool.swap_in(self.step.swap_in_host, self.step.swap_in_dev, stream=st)

        def lora_qkv(self, st):
            g = self.g
            g.pool.lora_apply_paged(g.acts["x"], g.token_adapter, g.rank, g.scale, g.lora_tables,
                                    [self.pj(n) for n in names_qkv], n_tokens=self.T, d_in=cfg.hidden,
                                    n_adapters=self.n_ad, max_rank=self.max_rank, stream=st)

        def kv_append(self, st):
            self.g.pool.kv_append(self.ys["k"], self.ys["v"], self.step.cu_new, self.step.prefix_len,
                                  self.g.kv_tables, stream=st)

        def attention(self, st):
            self.g.pool.paged_prefix_attention(self.ys["q"], self.attn_out, self.step.cu_new, self.step.prefix_len,
                                               self.g.kv_tables, cfg.n_q_heads, stream=st)

        def lora_o(self, st):
            g = self.g
            if "o" not in cfg.projections:
                return
            g.pool.lora_apply_paged(self.attn_out, g.token_adapter, g.rank, g.scale, g.lora_tables, [self.pj("o")],
                                    n_tokens=self.T, d_in=qd, n_adapters=self.n_ad, max_rank=self.max_rank, stream=st)

        def compute(self, st):
            self.lora_qkv(st)
            self.kv_append(st)
            self.attention(st)
            self.lora_o(st)

    runners = [Runner(g) for g in sets]
    s_comp, s_swap = torch.cuda.Stream(), torch.cuda.Stream()     # default priority, both

    def pipeline(n_steps):
        """swap(k) on the swap stream overlaps compute(k-1); batch k%2.  Returns tokens processed."""
        comp_done = [None] * n_steps
        tokens = 0
        for k in range(n_steps):
            r = runners[k % n_sets]
            if k >= n_sets:                       # the batch's blocks were last read by compute k - n_sets
                s_swap.wait_event(comp_done[k - n_sets])
            r.swap(s_swap)
            ev = torch.cuda.Event()
            ev.record(s_swap)
            s_comp.wait_event(ev)
            r.compute(s_comp)
            comp_done[k] = torch.cuda.Event()
            comp_done[k].record(s_comp)
            tokens += r.T
        return tokens

    pipeline(args.warmup)
    torch.cuda.synchronize()
    wall0 = time.perf_counter()
    tokens = pipeline(args.steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_per_step = wall * 1e3 / args.steps

    # ---- serialised pass on one stream: per-stage durations from HIP events on that stream
    r0 = runners[0]
    stages = [("swap", r0.swap), ("lora_qkv", r0.lora_qkv), ("kv_append", r0.kv_append), ("attention", r0.attention),
              ("lora_o", r0.lora_o)]
    n_rep = max(5, min(args.steps, 20))
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(n_rep)]
    torch.cuda.synchronize()
    ser0 = time.perf_counter()
    for k in range(n_rep):
        ev[k][0].record(s_comp)
        for i, (_, f) in enumerate(stages):
            f(s_comp)
            ev[k][i + 1].record(s_comp)
    torch.cuda.synchronize()
    serial_ms = (time.perf_counter() - ser0) * 1e3 / n_rep
    stage_ms = {name: float(np.median([ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(n_rep)]))
                for i, (name, _) in enumerate(stages)}

    # ---- algorithmic work of each stage (batch 0)
    step = r0.step
    T = r0.T
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
    max_rank = r0.max_rank

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
        "swap": {"bound": "pcie", "peak_GBps": PCIE_PEAK_GBS, "bytes": swap_bytes},
        "lora_qkv": {"bound": "hbm", "bytes": lora_bytes(names_qkv, cfg.hidden), "flops": lora_flops(names_qkv, cfg.hidden)},
        "kv_append": {"bound": "hbm", "bytes": append_bytes},
        "attention": {"bound": "hbm", "bytes": attn_bytes, "flops": attn_flops},
        "lora_o": {"bound": "hbm", "bytes": lora_bytes(["o"], qd), "flops": lora_flops(["o"], qd)}
        if "o" in cfg.projections else {"bound": "hbm", "bytes": 0.0, "flops": 0.0},
    }
    for name, k in kernels.items():
        ms = stage_ms[name]
        k["ms"] = round(ms, 4)
        k["GBps"] = round(k["bytes"] / (ms * 1e6), 1) if ms > 0 else None
        peak = k.pop("peak_GBps", HBM_PEAK_GBS)
        k["frac_of_peak"] = round(k["GBps"] / peak, 4) if ms > 0 else None
        if "flops" in k:
            k["TFLOPps"] = round(k["flops"] / (ms * 1e9), 2) if ms > 0 else None
            k["flops"] = int(k["flops"])
        k["bytes"] = int(k["bytes"])

    # ---- what this machine reaches with no arithmetic at all: a device-to-device copy and a pinned host-to-device
    #      copy (the runtime's own copy routines), the second denominator of every stage
    ach = achievable_rates(s_comp)
    for name, k in kernels.items():
        den = ach["pcie_h2d_GBps"] if k["bound"] == "pcie" else ach["hbm_copy_GBps"]
        k["frac_of_achievable"] = round(k["GBps"] / den, 4) if k["GBps"] else None

    # dominant on-chip kernel = attention; report it against the roofline that binds it
    a = kernels["attention"]
    t_hbm = a["bytes"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = a["flops"] / (MFMA_PEAK_TFLOPS * 1e12)
    traffic = MEASURED_TRAFFIC.get((cfg.name, seed)) if not over and args.swap_frac is None else None
    kname = "attn_mfma_kernel" if (cfg.dtype != "f32" and cfg.head_dim == 128 and
                                   int(N.max()) * (n_h // n_kv) >= 8) else "attn_rows_kernel"
    if cfg.dtype != "f32" and t_mfma > t_hbm:
        roof = {"bound": "mfma", "achieved": a["TFLOPps"], "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(a["TFLOPps"] / MFMA_PEAK_TFLOPS, 4), "traffic": traffic, "kernel": kname,
                "hbm_frac_of_same_launch": a["frac_of_peak"]}
    else:
        roof = {"bound": "hbm", "achieved": a["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(a["GBps"] / HBM_PEAK_GBS, 4), "traffic": traffic, "kernel": kname,
                "algorithmic_bytes": a["bytes"], "mfma_TFLOPps_of_same_launch": a["TFLOPps"],
                "mfma_frac_of_same_launch": round(a["TFLOPps"] / MFMA_PEAK_TFLOPS, 4)}

    # ---- the same LoRA calls with the dense base projection computed by the library (w_base given);
    #      reported on the side: the base model is not part of the pool's hot path
    base_info = None
    if cfg.dtype != "f32":
        wq = {n: torch.randn(step.proj[n].d_in, step.proj[n].d_out, device="cuda", dtype=torch.float16)
              .mul_(step.proj[n].d_in ** -0.5).to(torch.float16 if cfg.dtype == "f16" else torch.bfloat16)
              .view(torch.int16) for n in cfg.projections}
        g0 = r0.g

        def qkv_b(st):
            g0.pool.lora_apply_paged(g0.acts["x"], g0.token_adapter, g0.rank, g0.scale, g0.lora_tables,
                                     [dict(r0.pj(n), w_base=wq[n]) for n in names_qkv], n_tokens=T, d_in=cfg.hidden,
                                     n_adapters=r0.n_ad, max_rank=r0.max_rank, stream=st)

        def o_b(st):
            g0.pool.lora_apply_paged(r0.attn_out, g0.token_adapter, g0.rank, g0.scale, g0.lora_tables,
                                     [dict(r0.pj("o"), w_base=wq["o"])], n_tokens=T, d_in=qd, n_adapters=r0.n_ad,
                                     max_rank=r0.max_rank, stream=st)
        tms = {}
        for nm, f in (("lora_qkv", qkv_b), ("lora_o", o_b)):
            f(s_comp)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(s_comp)
            for _ in range(3):
                f(s_comp)
            e1.record(s_comp)
            torch.cuda.synchronize()
            tms[nm] = e0.elapsed_time(e1) / 3
        # the two calls now hold the dense products AND the LoRA branches (on large batches the expand step is the
        # GEMM's epilogue), so the rate is taken over the whole calls: dense flops / time of both calls
        gemm_flops = 2.0 * T * sum(step.proj[n].d_in * step.proj[n].d_out for n in list(names_qkv) + ["o"])
        gemm_ms = tms["lora_qkv"] + tms["lora_o"]
        base_info = {"lora_qkv_ms": round(tms["lora_qkv"], 4), "lora_o_ms": round(tms["lora_o"], 4),
                     "gemm_flops": int(gemm_flops), "gemm_ms": round(gemm_ms, 4),
                     "gemm_TFLOPps": round(gemm_flops / (gemm_ms * 1e9), 1),
                     "gemm_frac_of_mfma_peak": round(gemm_flops / (gemm_ms * 1e9) / MFMA_PEAK_TFLOPS, 4),
                     "note": "dense flops over the time of both calls, LoRA branches included",
                     "compute_only_tokens_per_s": round(T / ((sum(v for k, v in stage_ms.items()
                                                                  if k not in ("swap", "lora_qkv", "lora_o"))
                                                              + gemm_ms) * 1e-3), 1)}

    compute_ms = sum(v for k, v in stage_ms.items() if k != "swap")
    out = {
        "metric": "tokens/s of paged multi-LoRA layer step",
        "value": round(tokens / wall, 1),
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
        "config": {"workload": cfg.name, "tokens_per_step": [r.T for r in runners], "n_seqs": cfg.n_seqs,
                   "hidden": cfg.hidden, "heads": "%dx%d (kv %d)" % (n_h, d, n_kv), "adapters": int(len(active)),
                   "ranks": sorted(set(int(r) for r in step.rank[active])),
                   "swap_in_blocks": [int(len(r.step.swap_in_dev)) for r in runners], "block_bytes": cfg.block_bytes,
                   "base_gemm": "excluded (y arrives holding x.W)", "overrides": over or None,
                   "adapter_pool": cfg.n_adapters, "adapter_dist": cfg.adapter_dist,
                   "swap": ("own stream, overlapped with the previous batch's compute (two alternating batches)"
                            if n_sets == 2 else "none in this workload")},
        "roofline": roof,
        "kernels": kernels,
        "achievable": ach,
        "serialised": {"ms_per_step": round(serial_ms, 4), "tokens_per_s": round(T / (serial_ms * 1e-3), 1),
                       "compute_only_ms": round(compute_ms, 4),
                       "compute_only_tokens_per_s": round(T / (compute_ms * 1e-3), 1)},
        "with_base_gemm": base_info,
    }

    if args.layers > 0 and cfg.dtype != "f32":
        out["layer_stack"] = layer_stack(args, cfg, runners[0], s_comp)
    if not args.no_cpu_baseline:
        out["host_logic"] = host_logic()
        out["cpu_baseline"] = cpu_baseline(wl.make_step(cfg, seed=seed), args.cpu_seconds)
    print(json.dumps(out))


def achievable_rates(stream):
    """Rates of plain copies on this machine, measured with HIP events on `stream`: 1 GiB device to device (read +
    write counted, the way the HBM-bound stages count their bytes) and 512 MiB from pinned host memory to the
    device.  Median of 5 after one warm-up each."""
    import numpy as np
    import torch
    n_dev, n_host = 1 << 30, 1 << 29
    src = torch.empty(n_dev, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    host = torch.empty(n_host, dtype=torch.uint8, pin_memory=True).fill_(1)

    def med(f):
        ts = []
        with torch.cuda.stream(stream):
            f()
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                f()
                e1.record(stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1))
        return float(np.median(ts))
    torch.cuda.synchronize()
    t_copy = med(lambda: dst.copy_(src, non_blocking=True))
    t_h2d = med(lambda: dst[:n_host].copy_(host, non_blocking=True))
    torch.cuda.synchronize()
    del src, dst, host
    return {"hbm_copy_GBps": round(2 * n_dev / (t_copy * 1e6), 1), "pcie_h2d_GBps": round(n_host / (t_h2d * 1e6), 1),
            "note": "1 GiB device-to-device copy (read + write bytes) and 512 MiB pinned host-to-device copy by the "
                    "runtime's copy routines, median of 5"}


def layer_stack(args, cfg, r0, stream):
    """The batch through `--layers` whole decoder layers (include/fllayer.h): RMSNorm, dense base projections
    with the paged LoRA branch, RoPE, KV append, paged prefix attention, gated-SiLU MLP, residuals; one pool
    per layer (each a copy of the batch's pool: same block ids and tables in every layer), random weights of
    the model's shapes.  All blocks are resident (the swap belongs to the headline figure, not to this one)."""
    import numpy as np
    import torch
    from paper_2505_03756_amd import fllayer, flpool
    g, step, T = r0.g, r0.step, r0.T
    L = int(args.layers)
    mlp = int(args.mlp_dim or cfg.mlp_dim or {4096: 11008, 5120: 13824, 8192: 22016}.get(cfg.hidden, 4 * cfg.hidden))
    tdt = torch.float16 if cfg.dtype == "f16" else torch.bfloat16
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20250611)
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    shapes = {"q": (qd, cfg.hidden), "k": (kd, cfg.hidden), "v": (kd, cfg.hidden), "o": (cfg.hidden, qd),
              "gate": (mlp, cfg.hidden), "up": (mlp, cfg.hidden), "down": (cfg.hidden, mlp)}
    layers, keep = [], []
    host_stub = torch.zeros(cfg.block_elems, dtype=torch.int16).pin_memory()
    for l in range(L):
        if l == 0:
            pool = g.pool
        else:                                   # this layer's pool: the same blocks at the same ids
            dev = g.dev.clone()
            pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, dev.shape[0], 1, block_tokens=cfg.block_tokens,
                               dev=dev, host=host_stub)
            keep.append(dev)
        W = {n: (torch.randn(sh, generator=gen, device="cuda", dtype=torch.float32) * sh[1] ** -0.5).to(tdt)
             for n, sh in shapes.items()}
        W["in_norm"] = (1 + 0.1 * torch.randn(cfg.hidden, generator=gen, device="cuda")).to(tdt)
        W["post_norm"] = (1 + 0.1 * torch.randn(cfg.hidden, generator=gen, device="cuda")).to(tdt)
        layers.append(fllayer.Layer(pool, cfg.hidden, cfg.n_q_heads, mlp, W))
    pos = np.concatenate([step.prefix_len[i] + np.arange(step.cu_new[i + 1] - step.cu_new[i])
                          for i in range(len(step.prefix_len))]).astype(np.int32)
    places = {n: g.proj[n] for n in g.proj}
    batch = fllayer.Batch(step.cu_new, step.prefix_len, torch.from_numpy(pos).cuda(), g.kv_tables, g.token_adapter,
                          g.rank, g.scale, g.lora_tables, places, n_adapters=len(step.rank),
                          max_rank=int(max(1, step.rank.max())), max_blocks_per_seq=step.kv_tables.shape[1])
    nbytes = layers[0].scratch_bytes(T)
    scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    sp = (scratch.data_ptr() + 255) & ~255
    h0 = torch.randn((T, cfg.hidden), generator=gen, device="cuda", dtype=torch.float32).to(tdt)
    h = h0.clone()

    def run():
        h.copy_(h0)
        for ly in layers:
            ly.forward(batch, h, sp, nbytes, stream=stream)

    torch.cuda.synchronize()            # pools and weights were filled on torch's default stream
    with torch.cuda.stream(stream):
        run()
        torch.cuda.synchronize()
        assert bool(torch.isfinite(h.float()).all()), "layer stack produced non-finite values"
        reps = 3
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            run()
        e1.record(stream)
        torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    gemm_flops = 2.0 * T * sum(a * b for a, b in shapes.values())
    return {"layers": L, "mlp_dim": mlp, "tokens": T, "ms_stack": round(ms, 3), "ms_per_layer": round(ms / L, 3),
            "tokens_per_s_per_layer": round(T / (ms / L * 1e-3), 1),
            "dense_flops_per_layer": int(gemm_flops),
            "dense_TFLOPps_if_all_time_were_gemm": round(gemm_flops * L / (ms * 1e9), 1),
            "lora_on": sorted(places), "note": "blocks resident; random weights; one pool per layer"}


def host_logic():
    """The cache manager / cache swapper that produces the block lists (host only, a few seconds): a
    seeded 300 s chat trace through the library, the paper's three ablations beside it, and the
    manager's own overheads against the paper's budget (< 0.5 ms per match and update, <= 5 ms per
    swapping decision)."""
    from paper_2505_03756_amd import cache_sim
    keep = ("queries", "kv_hit_ratio", "kv_hit_ratio_hbm", "lora_cold_starts", "cold_start_ms_per_query",
            "invalid_kv_share_mean", "swapper_out_GB", "nodes_at_end", "match_update_us_mean", "match_update_us_p99",
            "tick_ms_mean", "tick_ms_max")
    res = {}
    for name in cache_sim.VARIANTS:
        r = cache_sim.simulate(name, duration_s=300.0, n_dev_blocks=8192)
        res[name] = {k: r[k] for k in keep}
    res["trace"] = ("synthetic chat trace, 300 s at 2 conversations/s, 50 LoRAs (Zipf), 8192 HBM blocks of 256 KiB, "
                    "thresholds 0.95 / 0.70, 100 ms monitor interval")
    return res


def cpu_baseline(step, target_s):
    """The oracle as it stands, timed on this machine's host cores over a bounded sample of the same
    workload: for a random sample of tokens, every stage a token goes through (LoRA q/k/v/o rows and
    its attention row over the full context)."""
    import numpy as np
    import oracle
    from paper_2505_03756_amd.harness import resident_pool
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
    host = {"nproc": os.cpu_count()}
    try:
        with open("/proc/cpuinfo") as f:
            host["cpu"] = next(l.split(":", 1)[1].strip() for l in f if l.startswith("model name"))
        with open("/proc/meminfo") as f:
            host["mem_GiB"] = round(int(next(l for l in f if l.startswith("MemTotal")).split()[1]) / 2 ** 20, 1)
    except (OSError, StopIteration, ValueError):
        pass
    return {"value": round(n / dt, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle", "host": host,
            "sample": "%d of %d tokens of one batch of the same workload (uniform, seeded): LoRA rows for %s and the "
                      "attention row over the full context, fp64, OpenMP over tokens; %.1f s"
                      % (n, T, "/".join(cfg.projections), dt)}


if __name__ == "__main__":
    main()
