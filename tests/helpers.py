"""Test-side helpers: the harness plumbing lives in the package; only the comparison rule and the
tolerances are defined here."""
import numpy as np

from paper_2505_03756_amd.harness import (GpuPool, GpuStep, SparseGpuPool, build_pools, compact_step,  # noqa: F401
                                          poison_value, resident_pool, to_dev, to_np)


def close(got, ref, rtol, atol):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    tol = atol + rtol * np.abs(ref)
    bad = ~(err <= tol)
    return not bad.any(), float(err.max() if err.size else 0.0), int(bad.sum())


TOL = {"f32": (1e-4, 1e-5), "f16": (2e-3, 1e-2), "bf16": (2e-3, 1e-2)}


# ------------------------------------------------------------------ stratified samples of a large batch
def attention_rows_sample(step, rng, per_cell=1, cells_per_seq=None, seqs=None):
    """Token indices for the attention check, chosen over the structure the matrix-core kernel works in: a
    workgroup owns 256 query rows of one (sequence, kv head), row = token * G + head % G, its eight waves 32 rows
    each; the context is walked in tiles of 64 keys.  Every sequence contributes its first and last new token, a
    token from every wave of every row tile (all of them for the ragged last tile; `cells_per_seq` caps the
    others at random), and the tokens whose context ends right before, at and after a 64-key boundary.
    `seqs` restricts the sample to those sequences."""
    cfg = step.cfg
    G = cfg.n_q_heads // cfg.n_kv_heads
    picks = []
    for i in (range(len(step.prefix_len)) if seqs is None else seqs):
        t0, N, P = int(step.cu_new[i]), int(step.new_len[i]), int(step.prefix_len[i])
        if N <= 0:
            continue
        own = {0, N - 1}
        rows = N * G
        n_tiles = -(-rows // 256)
        cells = []
        for t in range(n_tiles):
            for w in range(8):
                lo = (256 * t + 32 * w + G - 1) // G
                hi = min(N, (256 * t + 32 * w + 31) // G + 1)
                if lo < hi:
                    cells.append((t == n_tiles - 1, lo, hi))
        last = [c for c in cells if c[0]]
        rest = [c for c in cells if not c[0]]
        if cells_per_seq is not None and len(rest) > cells_per_seq:
            rest = [rest[k] for k in rng.choice(len(rest), size=cells_per_seq, replace=False)]
        for _, lo, hi in last + rest:
            own.update(int(j) for j in rng.integers(lo, hi, size=per_cell))
        for j in range(N):                       # context length P + j + 1 around a multiple of 64
            if (P + j + 1) % 64 in (63, 0, 1):
                own.add(j)
                if len(own) > 64:
                    break
        picks.extend(t0 + j for j in sorted(own))
    return np.unique(np.asarray(picks, dtype=np.int32))


def lora_rows_sample(step, rng, n_min):
    """Token indices for the LoRA check, chosen over the structure the tiled kernels work in: tokens are grouped by
    adapter, a segment is cut into tiles of 32 tokens and groups of 256.  Every adapter contributes its first and
    last token, the tokens around its tile boundaries and some of its ragged last tile; tokens without an adapter
    and a random remainder fill the sample up to n_min."""
    ta = step.token_adapter
    picks = set()
    for a in np.unique(ta):
        idx = np.flatnonzero(ta == a)
        if a < 0:
            picks.update(int(t) for t in idx[:4])
            continue
        n = len(idx)
        pos = {0, n - 1, min(n - 1, 31), min(n - 1, 32), min(n - 1, 255), min(n - 1, 256)}
        tail0 = (n - 1) // 32 * 32
        pos.update(int(p) for p in rng.integers(tail0, n, size=4))
        picks.update(int(idx[p]) for p in pos)
    T = len(ta)
    if len(picks) < n_min:
        rest = np.setdiff1d(np.arange(T), np.fromiter(picks, dtype=np.int64, count=len(picks)))
        picks.update(int(t) for t in rng.choice(rest, size=min(len(rest), n_min - len(picks)), replace=False))
    return np.asarray(sorted(picks), dtype=np.int32)
