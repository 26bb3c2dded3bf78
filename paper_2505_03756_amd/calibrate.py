"""Plain block copy of a known size through the library (device tier to device tier).

`python -m paper_2505_03756_amd.calibrate [--gib N]` moves N GiB with flp_pool_swap_in over a
pool whose "host" tier is placed in device memory, and prints the achieved copy rate.  Run it
under `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` to read what those counters report for
a kernel whose HBM traffic is known exactly (N GiB fetched, N GiB written): the ratio scales
the same counters of the other kernels.
"""
import argparse
import time

import numpy as np


def main():
    import torch
    from . import flpool
    ap = argparse.ArgumentParser()
    ap.add_argument("--gib", type=int, default=1)
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    bb = 262144
    n = args.gib * (1 << 30) // bb
    dst = torch.zeros(n * bb, dtype=torch.uint8, device="cuda")
    src = torch.ones(n * bb, dtype=torch.uint8, device="cuda")
    pool = flpool.Pool("f16", 32, 128, n, n, dev=dst, host=src)
    ids = np.arange(n, dtype=np.int32)
    st = torch.cuda.Stream()
    pool.swap_in(ids, ids, stream=st)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(st)
    for _ in range(args.reps):
        pool.swap_in(ids, ids, stream=st)
    e1.record(st)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.reps
    assert bool((dst == 1).all())
    print("copied %d GiB per launch: %.3f ms, %.1f GB/s copied (%.1f GB/s read+write)"
          % (args.gib, ms, n * bb / ms / 1e6, 2 * n * bb / ms / 1e6))


if __name__ == "__main__":
    main()
