"""CPU oracle of the layer glue around the pool's hot path (TEST INFRASTRUCTURE ONLY: imported by
tests/, the smoke check and the benchmark's cpu_baseline leg, never by the product path).

The paper serves Llama-7B/13B/34B (section 6.1) and delegates the model itself to the serving
engine; what a layer of these models computes is the published Llama architecture.  Each function is
the definition written out in float64 with numpy:

  rmsnorm     y = x / sqrt(mean(x^2) + eps) * w                      (root-mean-square layer norm)
  rope        rotary position embedding, "rotate-half" pairing: channel i < d/2 is paired with channel
              i + d/2 and the pair is rotated by the angle pos * theta^(-2 i / d)
  silu_mul    out = gate * sigmoid(gate) * up                         (the gated SiLU of the MLP)
  layer       pre-norm decoder layer: h += O(attn(rope(Q(n1)), rope(K(n1)), V(n1))), n1 = rmsnorm(h);
              h += Down(silu_mul(Gate(n2), Up(n2))), n2 = rmsnorm(h); every projection is the dense base
              plus the token's LoRA branch (Eq. 1 / Eq. 2 of the paper), K and V go through the paged pool.

Interfaces between the steps are tensors in the pool's element type, so the composed layer rounds to
that type exactly where the boundary (include/fllayer.h) says a tensor is produced, and nowhere else:
a projection rounds base + delta once.

Readings (the paper is silent on all of them): eps = 1e-5 and theta = 10000 unless given; no bias
terms; the residual stream is kept in the pool's element type.
"""
import numpy as np

from . import kv_append as _kv_append
from . import lora_apply as _lora_apply
from . import paged_attention as _paged_attention


# ----------------------------------------------------------------------------- element types
def round_store(values, dtype):
    """Round float64 values to the element type (nearest even, one rounding from float64).
    Returns (storage array: float32 or uint16 bit patterns, the values those bits represent as float64)."""
    v = np.asarray(values, dtype=np.float64)
    if dtype == "f32":
        s = v.astype(np.float32)
        return s, s.astype(np.float64)
    if dtype == "f16":
        with np.errstate(over="ignore"):                # beyond 65504 rounds to infinity, silently
            s = v.astype(np.float16)
        return s.view(np.uint16), s.astype(np.float64)
    assert dtype == "bf16"
    # 8 significant bits, exponent range of float32: quantum 2^(e - 7) with e = max(exponent, -126)
    _, e = np.frexp(np.abs(v))
    ex = np.maximum(e - 1, -126)
    q = np.ldexp(1.0, ex - 7)
    r = np.rint(np.abs(v) / q) * q                      # rint rounds halves to even
    r = np.where(r > 3.3895313892515355e38, np.inf, r)
    r = np.where(np.isfinite(v) & (v != 0), np.copysign(r, v), v)
    bits = (r.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)   # exact: r has 8 significant bits
    return bits, r


def load(storage, dtype):
    """Storage array -> float64 values."""
    s = np.asarray(storage)
    if dtype == "f32":
        return s.astype(np.float64)
    if dtype == "f16":
        return s.view(np.float16).astype(np.float64)
    return (s.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------- the glue steps
def rmsnorm(x, w, eps=1e-5):
    """x [T, H], w [H] (float64 values) -> x / sqrt(mean_over_H(x^2) + eps) * w."""
    x = np.asarray(x, np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(w, np.float64)


def rope(x, positions, theta=10000.0):
    """x [T, n_heads, d], positions [T] -> rotated copy.  Pair (i, i + d/2) of every head turns by
    positions[t] * theta^(-2 i / d): (a, b) -> (a cos - b sin, b cos + a sin)."""
    x = np.asarray(x, np.float64)
    T, _, d = x.shape
    half = d // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.asarray(positions, np.float64)[:, None] * theta ** (-2.0 * i / d)[None, :]     # [T, d/2]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu_mul(gate, up):
    g = np.asarray(gate, np.float64)
    return g / (1.0 + np.exp(-g)) * np.asarray(up, np.float64)


# ----------------------------------------------------------------------------- the layer
def layer_forward(cfg, step, pool, weights, h_storage, positions, eps=1e-5, theta=10000.0):
    """One decoder layer over the batch `step` (a workload.Step) on the pool image `pool`
    ([n_blocks, block_elems] storage, modified: the new K/V are appended).

    weights: dict of storage arrays: "in_norm", "post_norm" [H]; "q","k","v","o","gate","up","down"
    as [d_out, d_in] (the layout of a linear layer's weight).  h_storage [T, H] storage.
    Returns the new residual stream as storage [T, H] plus a dict of the intermediate tensors (storage)."""
    dt = cfg.dtype
    T = step.n_tokens
    W = {k: load(v, dt) for k, v in weights.items()}
    inter = {}

    def project(x_st, names):
        """base + LoRA for the projections `names` of input x (storage [T, d_in]) -> storage [T, d_out] each."""
        out = {}
        xv = load(x_st, dt)
        for n in names:
            base = xv @ W[n].T                                            # dense base, float64
            pr = step.proj.get(n)
            if pr is None:                                                # no LoRA on this projection
                delta = 0.0
            else:
                zeros = np.zeros((T, pr.d_out), dtype=np.asarray(x_st).dtype)     # the oracle adds the branch to y_in
                delta = _lora_apply(pool, dt, np.ascontiguousarray(x_st), step.token_adapter, step.rank, step.scale,
                                    pr.a_tab_off, pr.a_row_base, pr.b_tab_off, pr.b_row_base, step.lora_tables,
                                    pr.d_out, y_in=zeros)
            out[n], _ = round_store(base + delta, dt)
        return out

    h = load(h_storage, dt)
    n1, _ = round_store(rmsnorm(h, W["in_norm"], eps), dt)
    inter["n1"] = n1
    qkv = project(n1, ["q", "k", "v"])
    nh, nkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    q, _ = round_store(rope(load(qkv["q"], dt).reshape(T, nh, d), positions, theta).reshape(T, nh * d), dt)
    k, _ = round_store(rope(load(qkv["k"], dt).reshape(T, nkv, d), positions, theta).reshape(T, nkv * d), dt)
    v = qkv["v"]
    inter.update(q=q, k=k, v=v)
    _kv_append(pool, dt, cfg.block_tokens, nkv, d, step.cu_new, step.prefix_len, step.kv_tables,
               np.ascontiguousarray(k).reshape(T, nkv, d), np.ascontiguousarray(v).reshape(T, nkv, d))
    att = _paged_attention(pool, dt, cfg.block_tokens, nkv, d, nh, step.cu_new, step.prefix_len, step.kv_tables,
                           np.ascontiguousarray(q).reshape(T, nh, d))
    att_st, _ = round_store(np.asarray(att).reshape(T, nh * d), dt)
    inter["attn"] = att_st
    o = project(att_st, ["o"])["o"]
    inter["o"] = o
    h1, h1v = round_store(h + load(o, dt), dt)
    n2, _ = round_store(rmsnorm(h1v, W["post_norm"], eps), dt)
    inter.update(h1=h1, n2=n2)
    gu = project(n2, ["gate", "up"])
    act, _ = round_store(silu_mul(load(gu["gate"], dt), load(gu["up"], dt)), dt)
    inter.update(gate=gu["gate"], up=gu["up"], act=act)
    dn = project(act, ["down"])["down"]
    inter["down"] = dn
    h2, _ = round_store(h1v + load(dn, dt), dt)
    return h2, inter
