#!/usr/bin/env python3
"""Benchmark of the paged multi-LoRA layer step on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input: block alloc / free for
the queries that come and go, swap-out / swap-in of the listed blocks between the pinned host tier
and the pool, batched LoRA on q/k/v (one call, x read once), KV append, paged prefix attention, LoRA
on o.  The base projections x.W are taken as given (y arrives holding them); they are not part of
the measured path.

The steps follow a seeded serving trace (paper_2505_03756_amd/trace.py): a fixed number of sequence
slots, queries that finish and are replaced, their block moves.  The timed region runs the steps the
way the method is meant to run (paper section 4.3, asynchronous swapping): the moves of step k (for
queries that join at step k + 1) run on their own stream while step k computes; a step's compute
waits for the moves of the step before.  `value` is tokens/s over the K timed steps.

The headline workload is the largest of the five that the benchmark description names (34b_gqa: the
pool fills the card, bursty arrivals); the other four follow as `sub_records` with the same fields.
A serialised pass (everything on one stream, HIP events between the stages) gives the per-kernel
durations of one batch; the roofline figure of the dominant on-chip kernel comes from HIP events
around that kernel inside the timed region.

Prints ONE JSON line.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = 2500.0    # dense fp16 / bf16 MFMA, published
FP32_PEAK_TFLOPS = 157.3     # fp32 vector, published
PCIE_PEAK_GBS = 64.0         # PCIe Gen5 x16, one direction
_COMPUTE_STREAM = None
WORKLOADS = ("34b_gqa", "13b", "7b_prefill", "7b_decode", "tiny")
# HBM bytes per launch of a workload's dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# file, scaled by what the same counters read for a plain copy of known size: profiles/measured_traffic.json.
# Every entry carries the hash of the kernel's source file at the time of the profile; an entry whose hash no
# longer matches is not reported (traffic: null).
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "measured_traffic.json")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None, choices=WORKLOADS,
                    help="time only this workload (default: 34b_gqa as the headline, the other four as sub-records)")
    ap.add_argument("--swap-frac", type=float, default=None,
                    help="override the share of needed blocks brought in over the host link each step "
                         "(sweep for the break-even between swap and compute)")
    ap.add_argument("--shift-period", type=int, default=None, help="steps between redraws of the adapter popularity "
                    "(13b: 1000; scale it down together with --steps)")
    ap.add_argument("--adapters", type=int, default=None, help="override the number of adapters (the paper's "
                    "1000 / 2000 LoRA experiment, section 6.9)")
    ap.add_argument("--adapter-dist", default=None, choices=["uniform", "zipf"],
                    help="override how queries pick their adapter")
    ap.add_argument("--block-tokens", type=int, default=None, choices=[16, 32], help="token positions per pool block "
                    "(32: the block size of the paper's vLLM baseline, as a layout variant; the pool keeps its bytes)")
    ap.add_argument("--dev-blocks", type=int, default=None, help="override the pool's device block count")
    ap.add_argument("--host-blocks", type=int, default=None)
    ap.add_argument("--seqs", type=int, default=None, help="override the number of sequence slots")
    ap.add_argument("--prefix-range", type=int, nargs=2, default=None, metavar=("LO", "HI"),
                    help="override the range the prefix lengths are drawn from (few long sequences: --seqs 4 "
                         "--prefix-range 16383 16383)")
    ap.add_argument("--early-moves-gb", type=float, default=0.75, help="a step whose moves reach this many GB (about "
                    "10 ms of the host link in both directions) hands them to the planner before its first compute "
                    "stage instead of after the KV append (0: always early; a large value: never)")
    ap.add_argument("--no-narrow-moves", action="store_true", help="never flag a request as unhurried (by default a "
                    "request handed over after the KV append whose moves need less than half a step at the narrow "
                    "rate is: the planner then launches its moves narrow)")
    ap.add_argument("--one-stream", action="store_true", help="moves and compute on ONE stream (no overlap): the "
                    "baseline the asynchronous pipeline is compared with")
    ap.add_argument("--one-swap-stream", action="store_true", help="write-backs and fetches share one stream beside "
                    "the compute stream (the two directions of the host link one after the other)")
    ap.add_argument("--layers", type=int, default=None, help="decoder layers of the layer_stack section (0: skip; "
                    "default: 2 for 7b_prefill); the stack runs a batch through that many layers with per-layer "
                    "pools and random weights")
    ap.add_argument("--mlp-dim", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=None, help="target CPU time of the oracle sample "
                    "(default 14 s for the headline, 4 s for a sub-record)")
    ap.add_argument("--calibrate-copy", action="store_true", help="run only a plain block copy of 1 GiB through "
                    "flp_pool_swap_in between two device tiers (the kernel of known traffic that scales the "
                    "rocprofv3 FETCH_SIZE / WRITE_SIZE readings) and exit")
    ap.add_argument("--attention-clock", type=float, default=None, metavar="SECONDS", help="run only the attention "
                    "stage of one batch of the workload in a loop for SECONDS while rocm-smi samples the shader "
                    "clock, on the pool as drawn and then on a zeroed pool, and print the two rates and clocks")
    ap.add_argument("--seed", type=int, default=None)
    return ap.parse_args()


def log(msg):
    sys.stderr.write("[bench] %s\n" % msg)
    sys.stderr.flush()


# ----------------------------------------------------------------------------------------------- set-up
def pool_size_for(cfg, args):
    """Device and host block counts: the workload's own, the largest the card holds for the 34B pool."""
    import torch
    nd, nh = cfg.n_dev_blocks, cfg.n_host_blocks
    if cfg.name == "34b_gqa":
        nh = 262144                                           # 16 GiB: a burst's moves of three steps in flight
    elif cfg.name == "13b":
        nh = 49152                                            # 15 GiB
    elif cfg.name == "7b_prefill":
        nh = 8192
    if args.dev_blocks is not None:
        nd = int(args.dev_blocks)
    else:
        free, _ = torch.cuda.mem_get_info()
        headroom = 20 * 2 ** 30                               # activations, outputs, LoRA intermediates, copies
        while nd * cfg.block_bytes + headroom > free:
            nd = int(nd * 0.9)
    if args.host_blocks is not None:
        nh = int(args.host_blocks)
    return nd, nh


def fill_random(t, std=1.0, chunk_elems=1 << 28):
    """Fill a device tensor of 16-bit or fp32 storage with N(0, std^2) values (synthetic block contents and
    activations), a chunk at a time."""
    import torch
    flat = t.view(-1)
    n = flat.numel()
    for lo in range(0, n, chunk_elems):
        hi = min(n, lo + chunk_elems)
        r = torch.randn(hi - lo, device=t.device, dtype=torch.float32)
        if std != 1.0:
            r.mul_(std)
        flat[lo:hi].copy_(r)
        del r


class Bench:
    """One workload on the card: pool, trace, device copies of the batch metadata, activations."""

    def __init__(self, name, args):
        import numpy as np
        import torch
        from paper_2505_03756_amd import flpool, trace as tr, workload as wl
        self.np, self.torch, self.wl = np, torch, wl
        cfg = wl.config(name)
        over = {}
        if args.adapters is not None:
            over["n_adapters"] = int(args.adapters)
        if args.adapter_dist is not None:
            over["adapter_dist"] = args.adapter_dist
        if args.block_tokens is not None and args.block_tokens != cfg.block_tokens:
            f = args.block_tokens / float(cfg.block_tokens)
            over.update(block_tokens=int(args.block_tokens), n_dev_blocks=int(cfg.n_dev_blocks / f),
                        n_host_blocks=int(cfg.n_host_blocks / f))
        if args.seqs is not None:
            over["n_seqs"] = int(args.seqs)
        if args.prefix_range is not None:
            over["prefix_range"] = (int(args.prefix_range[0]), int(args.prefix_range[1]))
        if over:
            cfg = cfg.scaled(**over)
        self.over = over
        tc = tr.trace_config(name)
        if args.swap_frac is not None:
            tc.mode, tc.churn_frac = ("churn", float(args.swap_frac)) if args.swap_frac > 0 else ("static", 0.0)
        if args.shift_period is not None:
            tc.shift_period = int(args.shift_period)
        nd, nh = pool_size_for(cfg, args)
        cfg = cfg.scaled(n_dev_blocks=nd, n_host_blocks=nh)
        self.cfg, self.tc, self.args = cfg, tc, args
        self.seed = args.seed if args.seed is not None else (tc.seed if tc.seed is not None else cfg.seed)
        t0 = time.time()
        # ---- the two tiers.  Block contents are N(0,1) values in the pool's element type: every block may become
        #      KV or adapter pages as the trace recycles it.
        self.fdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[cfg.dtype]
        self.dev = torch.empty((nd, cfg.block_elems), dtype=self.fdt, device="cuda")
        fill_random(self.dev)
        self.host = torch.empty((nh, cfg.block_elems), dtype=self.fdt, pin_memory=True)
        for lo in range(0, nh, 8192):                          # host tier: copies of device blocks (random data too)
            n = min(8192, nh - lo)
            self.host[lo:lo + n].copy_(self.dev[(lo % max(1, nd - n)):(lo % max(1, nd - n)) + n])
        torch.cuda.synchronize()
        self.pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, nd, nh, block_tokens=cfg.block_tokens,
                                dev=self.dev, host=self.host)
        rng = np.random.default_rng(self.seed)
        for tier, n in ((0, nd), (1, nh)):                     # a shuffled free list: allocate all, free in a seeded order
            ids = self.pool.alloc(n, tier)
            self.pool.free(rng.permutation(ids), tier)
        # ---- the trace, on the library's allocator
        self.trace = tr.ServingTrace(cfg, tc, self.seed, lambda n: self.pool.alloc(n, 0), lambda ids: self.pool.free(ids, 0),
                                     lambda n: self.pool.alloc(n, 1), lambda ids: self.pool.free(ids, 1))
        trc = self.trace
        S = cfg.n_seqs
        # ---- device copies of the batch metadata (three rotating pinned staging sets; see run())
        n_max = cfg.new_range[1] if cfg.decode_frac < 1.0 else 1
        n_mean = (1.0 - cfg.decode_frac) * 0.5 * (cfg.new_range[0] + cfg.new_range[1]) + cfg.decode_frac
        self.t_cap = int(min(S * n_max, 1.5 * S * n_mean + 4096))   # far above any batch the trace draws; checked per step
        i32 = torch.int32
        self.d_tables = torch.full((S, trc.max_blocks), -1, dtype=i32, device="cuda")
        # Everything else a step uploads travels as ONE blob in one copy: the adapters' ranks and block tables, the
        # ids of the sequence slots whose table rows changed (int64, for the scatter), the tokens' adapters, and the
        # changed rows themselves, which a device-side scatter then puts into d_tables.
        ev2 = lambda n: (n + 1) & ~1                           # int32 offsets kept even: the id section is read as int64
        A, Lt, mb = cfg.n_adapters, max(1, len(trc.lora_tables)), trc.max_blocks
        self.off_idx = ev2(A)
        self.off_tok = self.off_idx + 2 * S
        blob_cap = self.off_tok + ev2(self.t_cap) + S * mb + Lt
        self.d_blob = torch.zeros(blob_cap, dtype=i32, device="cuda")
        self.d_rank = self.d_blob[:A]
        self.d_changed = self.d_blob[self.off_idx:self.off_idx + 2 * S].view(torch.int64)
        self.d_token_adapter = self.d_blob[self.off_tok:self.off_tok + self.t_cap]
        self.d_lora_tables = torch.zeros(Lt, dtype=i32, device="cuda")    # replaced from the blob when the tables change
        # y is updated in place (y += scale * B A x), the same buffers serve every step, and blocks that held the
        # appended k and v rows come back as adapter pages when the trace recycles them: a branch of noticeable size
        # would feed on itself over a long run (and overflow the 16-bit types).  The bench keeps the activations
        # stationary: the branch is 0.3 % of y's spread and its sign alternates from step to step, so after n steps
        # y has drifted by less than 0.003 * sqrt(n) of its spread.  The kernels' work does not depend on the scale.
        s = 0.003 / float(np.sqrt(max(cfg.ranks) * cfg.hidden))
        self.d_scales = [torch.full((cfg.n_adapters,), v, dtype=torch.float32, device="cuda") for v in (s, -s)]
        self.n_lora_calls = 0
        self.early_move_bytes = args.early_moves_gb * 1e9
        self.d_proj = {n: {k: torch.from_numpy(getattr(pr, k)).cuda() for k in
                           ("a_tab_off", "a_row_base", "b_tab_off", "b_row_base")} for n, pr in trc.proj.items()}
        self.stage = [torch.zeros(blob_cap, dtype=i32, pin_memory=True) for _ in range(3)]
        # ---- activations of the largest batch the trace can produce (the first T rows are used)
        qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
        mk = lambda w: torch.empty((self.t_cap, w), dtype=self.fdt, device="cuda")
        self.x = mk(cfg.hidden)
        fill_random(self.x)
        self.ys = {"q": mk(qd), "k": mk(kd), "v": mk(kd)}
        if "o" in cfg.projections:
            self.ys["o"] = mk(cfg.hidden)
        for t in self.ys.values():
            fill_random(t)
        self.attn_out = torch.zeros((self.t_cap, qd), dtype=self.fdt, device="cuda")
        self.names_qkv = [p for p in ("q", "k", "v") if p in cfg.projections]
        self.max_rank = int(max(cfg.ranks))
        # default priority, all three.  The two directions of the host link are independent: write-backs and
        # fetches get a stream each.
        # One compute stream for the life of the process (a workload after the first would otherwise get a stream
        # that the runtime may bind to the hardware queue of a move stream, where the two take turns).
        global _COMPUTE_STREAM
        if _COMPUTE_STREAM is None:
            _COMPUTE_STREAM = torch.cuda.Stream()
        self.s_comp = _COMPUTE_STREAM
        self.planner = None
        if args.one_stream:
            self.s_in = self.s_out = self.s_comp
        elif args.one_swap_stream:
            self.s_in = self.s_out = torch.cuda.Stream()
        else:
            # the library's planner (include/flsched.h) owns the two move streams and their ordering
            from paper_2505_03756_amd import flsched
            self.planner = flsched.Planner(self.pool)
            self.s_in = self.s_out = None
        torch.cuda.synchronize()
        log("%s: pool %d x %d KiB (%.1f GiB), host tier %d blocks, %d slots, set-up %.1f s" % (
            cfg.name, nd, cfg.block_bytes >> 10, nd * cfg.block_bytes / 2 ** 30, nh, S, time.time() - t0))

    # ---- one step's pieces -------------------------------------------------------------------------
    def upload(self, st, k):
        """Batch metadata of trace step `st` to the device, on the compute stream, through staging blob k % 3: one
        copy of a few hundred KB, one scatter of the changed table rows and, when adapters were exchanged, one copy
        of their block tables."""
        torch, np = self.torch, self.np
        sg = self.stage[k % 3]
        h = sg.numpy()
        T, S, mb = st.n_tokens, self.cfg.n_seqs, self.trace.max_blocks
        ch = st.changed_slots
        n = len(ch)
        h[:len(st.rank)] = st.rank
        h[self.off_idx:self.off_idx + 2 * S].view(np.int64)[:n] = ch
        h[self.off_tok:self.off_tok + T] = st.token_adapter
        off_rows = self.off_tok + ((T + 1) & ~1)
        if n:
            h[off_rows:off_rows + n * mb].reshape(n, mb)[:] = st.kv_tables[ch]
        off_lt = off_rows + n * mb
        n_lt = len(st.lora_tables) if st.tables_changed else 0
        h[off_lt:off_lt + n_lt] = st.lora_tables[:n_lt]
        end = off_lt + n_lt
        with torch.cuda.stream(self.s_comp):
            self.d_blob[:end].copy_(sg[:end], non_blocking=True)
            if n:
                self.d_tables.index_copy_(0, self.d_changed[:n], self.d_blob[off_rows:off_lt].view(n, mb))
            if n_lt:
                self.d_lora_tables[:n_lt].copy_(self.d_blob[off_lt:end])

    def pj(self, n):
        return dict(y=self.ys[n], d_out=self.trace.proj[n].d_out, **self.d_proj[n])

    def swap(self, st, stream, stream_out=None):
        self.pool.swap_out(st.swap_out_dev, st.swap_out_host, stream=stream_out or stream)
        self.pool.swap_in(st.swap_in_host, st.swap_in_dev, stream=stream)

    def lora_qkv(self, st, stream):
        if not self.names_qkv:
            return
        self.n_lora_calls += 1
        self.pool.lora_apply_paged(self.x, self.d_token_adapter, self.d_rank, self.d_scales[self.n_lora_calls & 1],
                                   self.d_lora_tables,
                                   [self.pj(n) for n in self.names_qkv], n_tokens=st.n_tokens, d_in=self.cfg.hidden,
                                   n_adapters=self.cfg.n_adapters, max_rank=self.max_rank, stream=stream)

    def kv_append(self, st, stream):
        self.pool.kv_append(self.ys["k"], self.ys["v"], st.cu_new, st.prefix_len, self.d_tables, stream=stream)

    def attention(self, st, stream):
        self.pool.paged_prefix_attention(self.ys["q"], self.attn_out, st.cu_new, st.prefix_len, self.d_tables,
                                         self.cfg.n_q_heads, stream=stream)

    def lora_o(self, st, stream):
        if "o" not in self.cfg.projections:
            return
        qd = self.cfg.n_q_heads * self.cfg.head_dim
        self.pool.lora_apply_paged(self.attn_out, self.d_token_adapter, self.d_rank,
                                   self.d_scales[self.n_lora_calls & 1], self.d_lora_tables,
                                   [self.pj("o")], n_tokens=st.n_tokens, d_in=qd, n_adapters=self.cfg.n_adapters,
                                   max_rank=self.max_rank, stream=stream)

    # ---- algorithmic work of one batch ----------------------------------------------------------------
    def work(self, st):
        np, cfg = self.np, self.cfg
        e = self.wl.DTYPE_BYTES[cfg.dtype]
        N = st.new_len.astype(np.int64)
        P = st.prefix_len.astype(np.int64)
        L = P + N
        n_h, n_kv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
        T = int(N.sum())
        w = {"attn_bytes": float(np.sum((L * 2 * n_kv + 2 * N * n_h) * d * e)),
             "attn_flops": float(np.sum(4.0 * n_h * d * N * (P + (N + 1) / 2.0))),
             "append_bytes": float(2 * 2 * T * n_kv * d * e),
             "swap_bytes": float((len(st.swap_in_dev) + len(st.swap_out_dev)) * cfg.block_bytes)}
        active = np.flatnonzero(st.rank)
        r_tok = st.rank[st.token_adapter].astype(np.float64)

        def lora(names, d_in):
            b = T * d_in * e                                   # x, read once for all projections of the call
            f = 0.0
            for n in names:
                d_out = self.trace.proj[n].d_out
                b += 2 * T * d_out * e                         # y read-modify-write
                b += float(np.sum(st.rank[active])) * (d_in + d_out) * e     # A and B pages of the adapters in the batch
                b += 2 * T * self.max_rank * 4                 # v written and read (fp32)
                f += 2.0 * float(np.sum(r_tok)) * (d_in + d_out)
            return float(b), f
        w["lora_qkv_bytes"], w["lora_qkv_flops"] = lora(self.names_qkv, cfg.hidden)
        w["lora_o_bytes"], w["lora_o_flops"] = lora(["o"], n_h * d) if "o" in cfg.projections else (0.0, 0.0)
        return w

    # ---- the timed pipeline -----------------------------------------------------------------------
    def run(self, n_steps, timed):
        """n_steps of the trace.  Step k: the host draws the step, uploads the batch and enqueues
          - the write-back of what left at step k - 1 on the out stream, after the compute of step k - 1 (which
            still appended to those blocks),
          - the fetches for what joins at step k + 1 on the in stream, after the write-back of step k - 1 (the
            free list hands out the blocks that it released),
          - the compute of step k on the compute stream, after the fetches of step k - 1.
        Write-back, fetch and compute of one step thus run side by side.  The host runs at most two steps ahead
        of the GPU (it waits for the compute of step k - 2, which also makes the blocks it frees now safe to hand
        out).  Returns per-step records."""
        torch = self.torch
        recs = []
        one = self.args.one_stream
        self.t_prev = None                                   # a pause between two calls is no step
        for k in range(n_steps):
            g = self.step_no
            if g >= 2:
                self.comp_done[(g - 2) % 3].synchronize()     # staging set g % 3 and the blocks freed now are free
            st = self.trace.step()
            if st.n_tokens > self.t_cap:
                raise SystemExit("bench.py: a step of %d tokens exceeds the activation buffers (%d)" % (st.n_tokens, self.t_cap))
            self.upload(st, g)
            # Request g = the queries that join at step g + 1, with their fetches and the write-backs of what left.
            # Moves that fit beside the attention kernel are handed to the planner after the two streaming stages
            # (LoRA q,k,v and the KV append), with the compute announced up to there: beside the moves the streaming
            # stages run many times slower (memory latency under the host-link traffic), the attention kernel, bound
            # by the matrix cores, a few per cent.  Moves that outlast the compute bound the step by themselves and
            # start as early as they may.  Measured on 34b_gqa (35 burst steps in 200): 18.15 ms per step always
            # early, 17.47 with this rule, 17.21 never early (which stretches the attention launches of the burst
            # steps to 26 ms).
            move_bytes = (len(st.swap_in_dev) + len(st.swap_out_dev)) * self.cfg.block_bytes
            early = self.planner is not None and move_bytes >= self.early_move_bytes
            if early:
                self.planner.submit(g, st.swap_in_host, st.swap_in_dev, st.swap_out_dev, st.swap_out_host)
            if self.planner is not None:
                if g >= 1:
                    self.planner.stream_wait(g - 1, self.s_comp)     # this step's joiners were fetched by request g - 1
            else:
                if not one:
                    if self.prev_comp is not None:
                        self.s_out.wait_event(self.prev_comp)
                    if self.prev_out is not None and self.s_in is not self.s_out:
                        self.s_in.wait_event(self.prev_out)
                self.swap(st, self.s_in, self.s_out)
                ev_out, ev_in = torch.cuda.Event(), torch.cuda.Event()
                ev_out.record(self.s_out)
                ev_in.record(self.s_in)
                if self.prev_in is not None and not one:
                    self.s_comp.wait_event(self.prev_in)
                self.prev_in, self.prev_out = ev_in, ev_out
            ev = None
            self.lora_qkv(st, self.s_comp)
            self.kv_append(st, self.s_comp)
            if self.planner is not None and not early:
                self.planner.compute_enqueued(self.s_comp)
                # moves that need less than half of a step's time at the narrow rate (about 60 GB/s) are flagged as
                # unhurried: the planner launches them narrow and the attention kernel beside them keeps its pace
                unhurried = (not self.args.no_narrow_moves and self.step_est is not None
                             and move_bytes / 60e9 < 0.5 * self.step_est)
                self.planner.submit(g, st.swap_in_host, st.swap_in_dev, st.swap_out_dev, st.swap_out_host,
                                    unhurried=unhurried)
            if timed:
                ev = (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                ev[0].record(self.s_comp)
            self.attention(st, self.s_comp)
            if timed:
                ev[1].record(self.s_comp)
            self.lora_o(st, self.s_comp)
            done = torch.cuda.Event()
            done.record(self.s_comp)
            self.comp_done[g % 3] = done
            self.prev_comp = done
            if self.planner is not None:
                self.planner.compute_enqueued(self.s_comp)
            self.step_no += 1
            now = time.perf_counter()
            if self.t_prev is not None and g >= 3:           # the host runs two steps ahead, then at the GPU's pace
                dt = now - self.t_prev
                self.step_est = dt if self.step_est is None else 0.8 * self.step_est + 0.2 * dt
            self.t_prev = now
            recs.append(dict(st=st, ev=ev, t_host=now))
        return recs

    def reset_pipeline(self):
        self.step_no, self.prev_comp, self.prev_in, self.prev_out, self.comp_done = 0, None, None, None, [None] * 3
        self.t_prev, self.step_est = None, None             # host-side estimate of the time a step takes (seconds)

    def close(self):
        """Give the card back: the next workload sizes its pool by what is free."""
        import gc
        torch = self.torch
        torch.cuda.synchronize()
        if self.planner is not None:
            self.planner.close()
        self.pool.close()
        for k in list(self.__dict__):
            if k not in ("cfg", "tc", "args", "over"):
                delattr(self, k)
        gc.collect()
        torch.cuda.empty_cache()


def per_step(values):
    """A per-step series as it is for short runs, as quantiles and phase means for long ones."""
    import numpy as np
    if len(values) <= 64:
        return list(values)
    v = np.asarray(values, dtype=np.float64)
    n = len(v)
    return {"steps": n, "mean": round(float(v.mean()), 2), "min": float(v.min()), "max": float(v.max()),
            "quantiles_5_25_50_75_95": [round(float(q), 2) for q in np.percentile(v, [5, 25, 50, 75, 95])],
            "means_of_tenths_of_the_run": [round(float(x.mean()), 2) for x in np.array_split(v, 10)]}


def kernel_hash(fname):
    with open(os.path.join(ROOT, "paper_2505_03756_amd", "csrc", fname), "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def measured_traffic(workload, kernel, src):
    try:
        with open(TRAFFIC_FILE) as f:
            tab = json.load(f)
    except (OSError, ValueError):
        return None
    ent = tab.get("%s/%s" % (workload, kernel))
    if not ent or ent.get("source_sha256_16") != kernel_hash(src):
        return None
    return ent.get("hbm_bytes_per_launch")


def run_workload(name, args, headline):
    import numpy as np
    import torch
    b = Bench(name, args)
    cfg, tc = b.cfg, b.tc
    import gc
    b.reset_pipeline()
    b.run(args.warmup, timed=False)
    torch.cuda.synchronize()
    gc.collect()
    clock = ClockSampler(pause=0.05) if headline else None     # what the chip clocks at under the timed steps
    gc.disable()                    # the interpreter's cycle collector costs tens of ms when it strikes inside a step
    try:
        t_wall0 = time.time()
        wall0 = time.perf_counter()
        recs = b.run(args.steps, timed=True)
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
        t_wall1 = time.time()
    finally:
        gc.enable()
    sclk = [c for t, c in clock.stop() if t_wall0 + 0.1 <= t <= t_wall1] if clock else []
    tokens = sum(r["st"].n_tokens for r in recs)
    ms_per_step = wall * 1e3 / args.steps
    T_last = recs[-1]["st"].n_tokens
    for nm, t in list(b.ys.items()) + [("attn_out", b.attn_out)]:     # the buffers the steps updated in place
        v = t[:T_last].float()
        assert bool(torch.isfinite(v).all()) and float(v.abs().max()) < 32.0, "%s left the range of the inputs" % nm

    # ---- the dominant on-chip kernel inside the timed region: attention, HIP events on its own stream
    attn_ms = [r["ev"][0].elapsed_time(r["ev"][1]) for r in recs]
    works = [b.work(r["st"]) for r in recs]
    a_bytes = float(np.mean([w["attn_bytes"] for w in works]))
    a_flops = float(np.mean([w["attn_flops"] for w in works]))
    a_ms = float(np.mean(attn_ms))
    n_h, n_kv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    st_last = recs[-1]["st"]
    mfma_path = cfg.dtype != "f32" and d == 128 and int(st_last.new_len.max()) * (n_h // n_kv) >= 8
    kname, ksrc = ("attn_mfma_kernel", "attention_mfma.hip") if mfma_path else ("attn_rows_kernel", "attention.hip")
    gbps, tflops = a_bytes / (a_ms * 1e6), a_flops / (a_ms * 1e9)
    t_hbm, t_mfma = a_bytes / (HBM_PEAK_GBS * 1e9), a_flops / (MFMA_PEAK_TFLOPS * 1e12)
    traffic = measured_traffic(cfg.name, kname, ksrc) if not b.over and args.swap_frac is None else None
    common = {"traffic": traffic, "kernel": kname, "launches_timed": len(attn_ms), "avg_launch_ms": round(a_ms, 4),
              "median_launch_ms": round(float(np.median(attn_ms)), 4),
              "algorithmic_bytes_per_launch": int(a_bytes), "algorithmic_flops_per_launch": int(a_flops),
              "measured": "HIP events around the kernel's launches on the compute stream inside the timed region "
                          "(moves running beside it)"}
    if mfma_path and t_mfma > t_hbm:
        roof = dict(bound="mfma", achieved=round(tflops, 2), peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=round(tflops / MFMA_PEAK_TFLOPS, 4), hbm_frac_of_same_launch=round(gbps / HBM_PEAK_GBS, 4), **common)
    else:
        roof = dict(bound="hbm", achieved=round(gbps, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(gbps / HBM_PEAK_GBS, 4), mfma_frac_of_same_launch=round(tflops / MFMA_PEAK_TFLOPS, 4)
                    if mfma_path else None, **common)

    # ---- serialised pass over one batch (the last one of the timed region): per-stage durations
    torch.cuda.synchronize()
    st = st_last
    stages = [("swap", b.swap), ("lora_qkv", b.lora_qkv), ("kv_append", b.kv_append), ("attention", b.attention),
              ("lora_o", b.lora_o)]
    n_rep = 7
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(n_rep)]
    ser0 = time.perf_counter()
    for k in range(n_rep):
        ev[k][0].record(b.s_comp)
        for i, (_, f) in enumerate(stages):
            f(st, b.s_comp)
            ev[k][i + 1].record(b.s_comp)
    torch.cuda.synchronize()
    serial_ms = (time.perf_counter() - ser0) * 1e3 / n_rep
    stage_ms = {nm: float(np.median([ev[k][i].elapsed_time(ev[k][i + 1]) for k in range(n_rep)]))
                for i, (nm, _) in enumerate(stages)}
    w = b.work(st)
    kernels = {
        "swap": {"bound": "pcie", "peak_GBps": PCIE_PEAK_GBS, "bytes": w["swap_bytes"],
                 "blocks_in": int(len(st.swap_in_dev)), "blocks_out": int(len(st.swap_out_dev))},
        "lora_qkv": {"bound": "hbm", "bytes": w["lora_qkv_bytes"], "flops": w["lora_qkv_flops"]},
        "kv_append": {"bound": "hbm", "bytes": w["append_bytes"]},
        "attention": {"bound": roof["bound"], "bytes": w["attn_bytes"], "flops": w["attn_flops"]},
        "lora_o": {"bound": "hbm", "bytes": w["lora_o_bytes"], "flops": w["lora_o_flops"]},
    }
    ach = achievable_rates(b.s_comp) if headline else None
    for nm, kk in kernels.items():
        ms = stage_ms[nm]
        kk["ms"] = round(ms, 4)
        kk["GBps"] = round(kk["bytes"] / (ms * 1e6), 1) if ms > 0 and kk["bytes"] else None
        peak = kk.pop("peak_GBps", HBM_PEAK_GBS)
        kk["frac_of_peak"] = round(kk["GBps"] / peak, 4) if kk["GBps"] else None
        if "flops" in kk:
            kk["TFLOPps"] = round(kk["flops"] / (ms * 1e9), 2) if ms > 0 else None
            if nm.startswith("lora") and kk["TFLOPps"] is not None:
                kk["mfma_frac"] = round(kk["TFLOPps"] / MFMA_PEAK_TFLOPS, 5)
            kk["flops"] = int(kk["flops"])
        kk["bytes"] = int(kk["bytes"])
        if ach and kk["GBps"]:
            den = ach["pcie_h2d_GBps"] if kk["bound"] == "pcie" else ach["hbm_copy_GBps"]
            kk["frac_of_achievable"] = round(kk["GBps"] / den, 4)
    compute_ms = sum(v for k2, v in stage_ms.items() if k2 != "swap")
    # the same kernel with nothing beside it (serialised pass, last batch), for the reader of `frac`: in a step that the
    # host link bounds the launches of the timed region run beside both move kernels and are stretched by them
    ka = kernels["attention"]
    if sclk:
        roof["sclk_MHz_during_timed_steps"] = {"median": float(np.median(sclk)), "min": int(min(sclk)),
                                               "max": int(max(sclk)), "samples": len(sclk), "source": "rocm-smi"}
    roof["alone_ms_last_batch"] = ka["ms"]
    roof["frac_alone_last_batch"] = round((ka["TFLOPps"] / MFMA_PEAK_TFLOPS) if roof["bound"] == "mfma"
                                          else (ka["GBps"] / HBM_PEAK_GBS), 4)
    trc = b.trace
    n_in = [len(r["st"].swap_in_dev) for r in recs]
    n_out = [len(r["st"].swap_out_dev) for r in recs]
    swap_GB = [(i + o) * cfg.block_bytes / 1e9 for i, o in zip(n_in, n_out)]
    t_steps = np.diff(np.asarray([wall0] + [r["t_host"] for r in recs])) * 1e3      # host-side pace of the pipeline
    rec = {
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
        "config": {"workload": cfg.name, "tokens_per_step_mean": round(tokens / args.steps, 1), "n_seqs": cfg.n_seqs,
                   "hidden": cfg.hidden, "heads": "%dx%d (kv %d)" % (n_h, d, n_kv),
                   "pool_blocks": cfg.n_dev_blocks, "pool_GiB": round(cfg.n_dev_blocks * cfg.block_bytes / 2 ** 30, 1),
                   "host_blocks": cfg.n_host_blocks, "block_bytes": cfg.block_bytes,
                   "adapter_pool": cfg.n_adapters, "adapter_dist": cfg.adapter_dist,
                   "adapters_in_last_batch": int((st.rank > 0).sum()), "ranks": sorted(set(int(r) for r in cfg.ranks)),
                   "lora_on": list(cfg.projections), "base_gemm": "excluded (y arrives holding x.W)",
                   "trace": {"mode": tc.mode, "seed": int(b.seed), "churn_frac": tc.churn_frac if tc.mode == "churn" else None,
                             "swap_out": tc.swap_out, "shift_period": tc.shift_period or None,
                             "lam_calm": tc.lam_calm if tc.mode == "bursty" else None,
                             "lam_burst": tc.lam_burst if tc.mode == "bursty" else None,
                             "burst_steps_in_timed_region": int(sum(r["st"].burst for r in recs)),
                             "replaced_slots_per_step": per_step([int(r["st"].n_replaced) for r in recs]),
                             "distinct_adapters_per_step": per_step([int((r["st"].rank > 0).sum()) for r in recs])},
                   "overrides": b.over or None,
                   "swap": ("one stream, no overlap" if args.one_stream else
                            ("write-backs and fetches of step k on %s beside the compute of step k; the compute of "
                             "step k + 1 waits for the fetches" % ("one stream of their own" if args.one_swap_stream
                                                                   else "a stream each, issued and ordered by the "
                                                                        "library's planner (flsched.h)")))
                   if tc.mode != "static" else "none in this workload"},
        "roofline": roof,
        "step_pace_ms": per_step([round(float(x), 3) for x in t_steps]),
        "swap_traffic": {"GB_per_step_mean": round(float(np.mean(swap_GB)), 4), "GB_per_step_max": round(max(swap_GB), 4),
                         "GB_per_step_quartiles": [round(float(q), 4) for q in np.percentile(swap_GB, [25, 50, 75])],
                         "host_link_GBps_over_run": round(sum(swap_GB) / wall, 2),
                         "blocks_in_per_step": per_step(n_in), "blocks_out_per_step": per_step(n_out)},
        "kernels": kernels,
        "serialised": {"batch": "last batch of the timed region", "tokens": st.n_tokens, "ms_per_step": round(serial_ms, 4),
                       "tokens_per_s": round(st.n_tokens / (serial_ms * 1e-3), 1), "compute_only_ms": round(compute_ms, 4),
                       "compute_only_tokens_per_s": round(st.n_tokens / (compute_ms * 1e-3), 1)},
    }
    if ach:
        rec["achievable"] = ach
    layers = args.layers if args.layers is not None else (2 if cfg.name == "7b_prefill" else 0)
    if layers > 0 and cfg.dtype != "f32":
        rec["layer_stack"] = layer_stack(b, st, layers, args)
    b.close()
    if not args.no_cpu_baseline:
        secs = args.cpu_seconds if args.cpu_seconds is not None else (14.0 if headline else 4.0)
        rec["cpu_baseline"] = cpu_baseline(cfg, secs)
    return rec


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported. "
              "Run with --gpus 1; the value is that one GPU's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        return calibrate_copy()
    if args.attention_clock is not None:
        return attention_clock(args)
    names = [args.workload] if args.workload else list(WORKLOADS)
    out = None
    for i, name in enumerate(names):
        t0 = time.time()
        rec = run_workload(name, args, headline=(i == 0))
        log("%s: %.0f tokens/s, %.3f ms/step (%.0f s)" % (name, rec["value"], rec["ms_per_step"], time.time() - t0))
        if out is None:
            out = rec
            out["sub_records"] = {}
        else:
            out["sub_records"][name] = rec
    if not args.no_cpu_baseline:
        out["host_logic"] = host_logic()
    print(json.dumps(out))


# ----------------------------------------------------------------------------------------------- side figures
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


class ClockSampler:
    """Shader clock as `rocm-smi --showclocks --csv` reports it, sampled by a thread until stop(); samples are
    (time.time(), MHz).  Any failure of the tool just leaves the list short."""

    def __init__(self, pause=0.25):
        import threading
        self.samples, self._stop, self._pause = [], threading.Event(), pause
        self._th = threading.Thread(target=self._run, daemon=True)
        self._th.start()

    def _run(self):
        import re
        import subprocess
        while not self._stop.is_set():
            try:
                r = subprocess.run(["/opt/rocm/bin/rocm-smi", "--showclocks", "--csv"], capture_output=True, text=True,
                                   timeout=10)
                m = re.findall(r"\((\d+)Mhz\)", r.stdout.strip().splitlines()[-1])
                if m:
                    self.samples.append((time.time(), int(m[-1])))     # the last clock of the row is sclk
            except (OSError, subprocess.SubprocessError, IndexError):
                pass
            self._stop.wait(self._pause)

    def stop(self):
        self._stop.set()
        self._th.join(timeout=15)
        return self.samples


def attention_clock(args):
    """The attention stage alone, back to back for some seconds, with the shader clock sampled from rocm-smi beside
    it: on the pool as drawn (N(0,1) keys and values) and on a zeroed pool.  The instruction stream is the same in
    both phases; what differs is the power the matrix cores draw, and with it the clock the chip holds."""
    import numpy as np
    import torch
    name = args.workload or WORKLOADS[0]
    b = Bench(name, args)
    b.reset_pipeline()
    recs = b.run(3, timed=False)
    torch.cuda.synchronize()
    st = recs[-1]["st"]
    flops = b.work(st)["attn_flops"]
    clock = ClockSampler()
    samples = clock.samples
    out = {"workload": name, "tokens": st.n_tokens, "flops_per_launch": flops, "phases": []}
    try:
        for phase in ("pool as drawn", "pool zeroed"):
            if phase == "pool zeroed":
                b.dev.zero_()
            for _ in range(3):
                b.attention(st, b.s_comp)
            torch.cuda.synchronize()
            t0, ms = time.time(), []
            while time.time() - t0 < args.attention_clock:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(b.s_comp)
                for _ in range(5):
                    b.attention(st, b.s_comp)
                e1.record(b.s_comp)
                torch.cuda.synchronize()
                ms.append(e0.elapsed_time(e1) / 5)
            t1 = time.time()
            clk = [c for t, c in samples if t0 + 1.0 <= t <= t1]
            out["phases"].append({"data": phase, "launches": 5 * len(ms), "ms_per_launch": round(float(np.mean(ms)), 4),
                                  "TFLOPps": round(flops / float(np.mean(ms)) / 1e9, 1),
                                  "sclk_MHz_median": float(np.median(clk)) if clk else None,
                                  "sclk_MHz_min_max": [min(clk), max(clk)] if clk else None, "sclk_samples": len(clk)})
            time.sleep(1.5)
    finally:
        clock.stop()
    idle = [c for t, c in samples[-4:]]
    out["sclk_MHz_idle_after"] = idle
    print(json.dumps(out))
    b.close()


def calibrate_copy():
    """A plain copy of known HBM traffic through the library: 1 GiB of blocks from one device tier to another."""
    import numpy as np
    import torch
    from paper_2505_03756_amd import flpool
    bb = 262144
    n = (1 << 30) // bb
    dst = torch.zeros(n * bb, dtype=torch.uint8, device="cuda")
    src = torch.ones(n * bb, dtype=torch.uint8, device="cuda")
    pool = flpool.Pool("f16", 32, 128, n, n, dev=dst, host=src)
    ids = np.arange(n, dtype=np.int32)
    st = torch.cuda.Stream()
    pool.swap_in(ids, ids, stream=st)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(3):
        pool.swap_in(ids, ids, stream=st)
    e1.record(st)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 3
    assert bool((dst == 1).all())
    print(json.dumps({"calibrate_copy": {"bytes_read": n * bb, "bytes_written": n * bb, "launches": 4, "ms": round(ms, 4),
                                         "GBps_read_plus_write": round(2 * n * bb / ms / 1e6, 1)}}))


def layer_stack(b, st, L, args):
    """The batch `st` through L whole decoder layers (include/fllayer.h): RMSNorm, dense base projections with the
    paged LoRA branch, RoPE, KV append, paged prefix attention, gated-SiLU MLP, residuals; one pool per layer (layer
    0 uses the benchmark's pool, the others a small pool of their own that holds the batch's blocks at renumbered
    ids), random weights of the model's shapes.  All blocks are resident."""
    import numpy as np
    import torch
    from paper_2505_03756_amd import fllayer, flpool
    cfg, T = b.cfg, st.n_tokens
    mlp = int(args.mlp_dim or cfg.mlp_dim or {4096: 11008, 5120: 13824, 8192: 22016}.get(cfg.hidden, 4 * cfg.hidden))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20250611)
    qd, kd = cfg.n_q_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    shapes = {"q": (qd, cfg.hidden), "k": (kd, cfg.hidden), "v": (kd, cfg.hidden), "o": (cfg.hidden, qd),
              "gate": (mlp, cfg.hidden), "up": (mlp, cfg.hidden), "down": (cfg.hidden, mlp)}
    # the blocks the batch touches, renumbered densely for the per-layer pools
    used = np.unique(np.concatenate([st.kv_tables[st.kv_tables >= 0], st.lora_tables]))
    remap = np.zeros(int(used.max()) + 1, np.int32)
    remap[used] = np.arange(len(used), dtype=np.int32)
    kv_small = torch.from_numpy(np.where(st.kv_tables >= 0, remap[np.maximum(st.kv_tables, 0)], -1).astype(np.int32)).cuda()
    lt_small = torch.from_numpy(remap[st.lora_tables]).cuda()
    idx = torch.from_numpy(used.astype(np.int64)).cuda()
    host_stub = torch.zeros(cfg.block_elems, dtype=b.fdt).pin_memory()
    layers, keep = [], []
    for l in range(L):
        dev = b.dev[idx].clone()
        pool = flpool.Pool(cfg.dtype, cfg.n_kv_heads, cfg.head_dim, dev.shape[0], 1, block_tokens=cfg.block_tokens,
                           dev=dev, host=host_stub)
        keep.append((dev, pool))
        W = {n: (torch.randn(sh, generator=gen, device="cuda", dtype=torch.float32) * sh[1] ** -0.5).to(b.fdt)
             for n, sh in shapes.items()}
        W["in_norm"] = (1 + 0.1 * torch.randn(cfg.hidden, generator=gen, device="cuda")).to(b.fdt)
        W["post_norm"] = (1 + 0.1 * torch.randn(cfg.hidden, generator=gen, device="cuda")).to(b.fdt)
        layers.append(fllayer.Layer(pool, cfg.hidden, cfg.n_q_heads, mlp, W))
    # adapter pages as drawn: N(0,1) block contents would make the branches dominate; scale the adapters instead
    scale = torch.full((cfg.n_adapters,), 0.02 * 0.02, dtype=torch.float32, device="cuda")
    pos = np.concatenate([st.prefix_len[i] + np.arange(st.new_len[i]) for i in range(cfg.n_seqs)]).astype(np.int32)
    places = {n: b.d_proj[n] for n in b.d_proj}
    batch = fllayer.Batch(st.cu_new, st.prefix_len, torch.from_numpy(pos).cuda(), kv_small, b.d_token_adapter,
                          b.d_rank, scale, lt_small, places, n_adapters=cfg.n_adapters, max_rank=b.max_rank,
                          max_blocks_per_seq=st.kv_tables.shape[1])
    nbytes = layers[0].scratch_bytes(T)
    scratch = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    sp = (scratch.data_ptr() + 255) & ~255
    h0 = torch.randn((T, cfg.hidden), generator=gen, device="cuda", dtype=torch.float32).to(b.fdt)
    h = h0.clone()
    stream = b.s_comp

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
    gemm_flops = 2.0 * T * sum(x * y for x, y in shapes.values())
    for _, pool in keep:
        pool.close()
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


def cpu_baseline(cfg, target_s):
    """The oracle as it stands, timed on this machine's host cores over a bounded sample of the same workload: a
    seeded subsample of the workload's sequences (same shapes, lengths and adapter mix) and, of their tokens, a
    random sample sized to the time budget; every stage a token goes through (LoRA rows of every projection and
    its attention row over the full context).  Three timings: all cores with double running sums (the parity
    build: `value`), one thread, and all cores with fp32 running sums (a second build of the same source)."""
    import numpy as np
    import oracle
    from paper_2505_03756_amd import workload as wl
    from paper_2505_03756_amd.harness import resident_pool
    n_seqs = min(cfg.n_seqs, 16 if cfg.block_bytes * cfg.prefix_range[1] > (1 << 29) else 32)
    per_seq = -(-(cfg.prefix_range[1] + cfg.new_range[1]) // cfg.block_tokens) + 2
    sub = cfg.scaled(n_seqs=n_seqs, n_dev_blocks=int(n_seqs * per_seq * 1.3) + 4096, n_host_blocks=8,
                     swap_in_frac=0.0, swap_out_frac=0.0, n_adapters=min(cfg.n_adapters, 64))
    step = wl.make_step(sub, seed=cfg.seed)
    pool = resident_pool(step)
    bt, n_kv, d, n_h = sub.block_tokens, sub.n_kv_heads, sub.head_dim, sub.n_q_heads
    oracle.kv_append(pool, sub.dtype, bt, n_kv, d, step.cu_new, step.prefix_len, step.kv_tables,
                     step.acts["k_new"], step.acts["v_new"])          # not timed: a copy
    rng = np.random.default_rng(7)
    T = step.n_tokens

    def run(sel):
        t0 = time.perf_counter()
        for n in sub.projections:
            pr = step.proj[n]
            x = step.acts["x"] if pr.d_in == sub.hidden else step.acts["x_%d" % pr.d_in]
            oracle.lora_apply(pool, sub.dtype, x, step.token_adapter, step.rank, step.scale, pr.a_tab_off,
                              pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables, pr.d_out,
                              y_in=step.acts["base_" + n], sel=sel)
        oracle.paged_attention(pool, sub.dtype, bt, n_kv, d, n_h, step.cu_new, step.prefix_len, step.kv_tables,
                               step.acts["q"], sel=sel)
        return time.perf_counter() - t0

    threads = oracle.num_threads()
    pilot = rng.choice(T, size=min(T, 2 * threads), replace=False).astype(np.int32)
    tp = run(pilot)
    budget = 0.6 * target_s                                            # the other two timings share the rest
    n = int(min(T, max(len(pilot), len(pilot) * budget / max(tp, 1e-3))))
    n -= n % threads if n > threads else 0
    sel = rng.choice(T, size=n, replace=False).astype(np.int32)
    dt = run(sel)
    rate = n / dt
    # one thread, the same build
    n1 = int(max(1, min(n, rate / threads * 0.2 * target_s)))
    oracle.set_threads(1)
    try:
        dt1 = run(sel[:n1])
    finally:
        oracle.set_threads(0)
    # fp32 running sums, all cores (a second build of the same source; timing only)
    n32 = int(max(1, min(n, rate * 0.2 * target_s)))
    n32 -= n32 % threads if n32 > threads else 0
    oracle.set_variant("f32acc")
    try:
        dt32 = run(sel[:n32])
    finally:
        oracle.set_variant("parity")
    host = {"nproc": os.cpu_count()}
    try:
        with open("/proc/cpuinfo") as f:
            host["cpu"] = next(l.split(":", 1)[1].strip() for l in f if l.startswith("model name"))
        with open("/proc/meminfo") as f:
            host["mem_GiB"] = round(int(next(l for l in f if l.startswith("MemTotal")).split()[1]) / 2 ** 20, 1)
    except (OSError, StopIteration, ValueError):
        pass
    return {"value": round(rate, 2), "unit": "tokens/s", "cores": threads, "kind": "oracle", "host": host,
            "single_thread_tokens_per_s": round(n1 / dt1, 3), "single_thread_sample_tokens": n1,
            "fp32_accumulation_tokens_per_s": round(n32 / dt32, 2), "fp32_accumulation_sample_tokens": n32,
            "sample": "%d of the %d tokens of %d sequences drawn like the workload's (seeded): LoRA rows for %s and the "
                      "attention row over the full context, fp64 running sums, OpenMP over tokens; %.1f s"
                      % (n, T, n_seqs, "/".join(sub.projections), dt)}


if __name__ == "__main__":
    main()
