import argparse
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))


def run_hip_probe(name="issue_power_probe"):
    exe = os.path.join(HERE, "_" + name)
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), "--offload-arch=gfx950", "-O3", "-std=c++17",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", exe,
           os.path.join(HERE, name + ".hip")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.exit("hipcc failed:\n" + r.stderr)
    return subprocess.run([exe]).returncode


def per_tile():
    """Time of one 64-key tile step of the matrix-core attention kernel: the same 256-row tiles with two
    prefix lengths (10 tiles apart), on 32 workgroups (32 CUs busy) and on 256 (all CUs busy), the latter
    with distinct and with shared K/V blocks (HBM reads against L2 hits)."""
    import numpy as np
    import torch
    from .. import workload as wl
    from ..harness import GpuStep, build_pools
    cfg = wl.config("7b_prefill")
    step = wl.make_step(cfg, with_acts=True)
    dev0, host0 = build_pools(step)
    g = GpuStep(step, dev0, host0)
    st = torch.cuda.Stream()
    g.pool.swap_in(step.swap_in_host, step.swap_in_dev, stream=st)
    q = g.acts["q"]
    g.pool.kv_append(g.acts["k_new"], g.acts["v_new"], step.cu_new, step.prefix_len, g.kv_tables, stream=st)
    torch.cuda.synchronize()
    N = step.new_len.astype(int)
    P = step.prefix_len.astype(int)
    cu = step.cu_new.astype(int)
    cand = [i for i in range(len(N)) if 225 <= N[i] <= 256 and P[i] >= 1000]
    cand.sort(key=lambda i: -(P[i] + N[i]))

    def run(sel, prefix):
        qs = torch.cat([q[cu[i]:cu[i + 1]] for i in sel]).contiguous()
        out = torch.zeros_like(qs)
        cu_s = np.concatenate([[0], np.cumsum([N[i] for i in sel])]).astype(np.int32)
        tabs = g.kv_tables[torch.tensor(sel, device=g.kv_tables.device)].contiguous()
        pl = np.full(len(sel), prefix, dtype=np.int32)
        f = lambda: g.pool.paged_prefix_attention(qs, out, cu_s, pl, tabs, cfg.n_q_heads, stream=st)
        for _ in range(3):
            f()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(4):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(10):
                f()
            e1.record(st)
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) / 10)
        return best * 1e3

    for nseq, same in ((1, False), (8, False), (8, True)):
        sel = [cand[0]] * nseq if same else (cand * 8)[:nseq]
        t_long, t_short = run(sel, 960), run(sel, 320)
        print("%3d workgroups, %s K/V: %.1f us (prefix 960), %.1f us (prefix 320) -> %.3f us per tile step" %
              (nseq * cfg.n_kv_heads, "shared  " if same else "distinct", t_long, t_short, (t_long - t_short) / 10.0),
              flush=True)
    return 0


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--per-tile", action="store_true")
    ap.add_argument("--hbm", action="store_true", help="rates of plain read / copy / update-in-place kernels")
    a = ap.parse_args()
    sys.exit(per_tile() if a.per_tile else run_hip_probe("hbm_stream_probe") if a.hbm else run_hip_probe())
