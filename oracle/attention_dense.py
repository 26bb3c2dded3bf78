"""Whole-sequence form of the attention oracle (TEST INFRASTRUCTURE ONLY), numpy fp64.

The definition of paged prefix attention (paper sections 2.1 and 4.2: a query attends over the stored
KV of its matched prefix together with the KV of its own new tokens) evaluated for ALL new tokens of one
sequence at once, with library matrix products as the steps: gather K and V of positions 0..P+N-1 through
the sequence's block table (the C oracle's gather), scores = sm_scale * Q K^T, causal mask (new token j sees
positions 0..P+j), softmax with the maximum subtracted, out = W V.  No blocking, no running maximum.

It exists because the per-row C oracle needs minutes for all rows of a 16 k-token context; it is pinned
against that oracle and against closed forms in tests/test_oracle_attention.py.
"""
from __future__ import annotations

import numpy as np

from . import kv_gather


def _values(bits, dtype):
    if dtype == "f32":
        return np.asarray(bits, dtype=np.float32).astype(np.float64)
    b = np.asarray(bits).view(np.uint16)
    if dtype == "f16":
        return b.view(np.float16).astype(np.float64)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def paged_attention_sequence(pool, dtype, bt, n_kv, d, n_h, cu_new, prefix_len, tables, q, seq, sm_scale=0.0):
    """Output rows [N, n_h, d] (float64) of all N new tokens of sequence `seq`.
    q: storage array [T, n_h * d] or [T, n_h, d] of the whole batch."""
    t0, t1 = int(cu_new[seq]), int(cu_new[seq + 1])
    N, P = t1 - t0, int(prefix_len[seq])
    out = np.zeros((N, n_h, d), dtype=np.float64)
    if N == 0:
        return out
    L = P + N
    K, V = kv_gather(pool, dtype, bt, n_kv, d, np.ascontiguousarray(tables[seq]), L)      # [L, n_kv, d]
    Q = _values(np.asarray(q).reshape(-1, n_h, d)[t0:t1], dtype)                          # [N, n_h, d]
    scale = sm_scale if sm_scale > 0 else 1.0 / np.sqrt(float(d))
    group = n_h // n_kv
    visible = np.arange(L)[None, :] <= (P + np.arange(N))[:, None]                        # [N, L]
    for h in range(n_h):
        g = h // group
        s = scale * (Q[:, h, :] @ K[:, g, :].T)                                           # [N, L]
        s = np.where(visible, s, -np.inf)
        s -= s.max(axis=1, keepdims=True)
        w = np.exp(s)
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ V[:, g, :]
    return out
