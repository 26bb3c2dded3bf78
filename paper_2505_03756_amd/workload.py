"""Seeded synthetic workloads for the paged multi-LoRA layer step.

This module only *draws inputs*: shapes, lengths, adapter choices, block ids,
random block contents and swap lists.  It holds none of the method's
arithmetic and no address rule of the pool: blocks are filled element-wise
with random values and both the CPU oracle and the HIP library interpret them
through the block tables with their own, separately written, layout code.
The only sizing fact it uses is how many page-rows of a given length fit in a
block (needed to know how many blocks to ask the allocator for).

The paper evaluates on chat / translation / agent traces with 20-100 adapters
of rank 32 or 64 whose weights are drawn from a normal distribution (paper
section 6.1); none of those traces is used or reproduced here.  The five
workloads below take their shapes from the benchmark description of this
repository and stand in for them.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

import numpy as np

DTYPE_CODE = {"f32": 0, "f16": 1, "bf16": 2}
DTYPE_BYTES = {"f32": 4, "f16": 2, "bf16": 2}


# ----------------------------------------------------------------------------
# number-format helpers (format conversion only)
# ----------------------------------------------------------------------------
def quantize(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values once (nearest-even) to the storage dtype.

    f32 -> float32 array; f16 / bf16 -> uint16 array of raw bits.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    if dtype == "f16":
        return a.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = a.view(np.uint32).astype(np.uint64)
        r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
        return r.astype(np.uint16)
    raise ValueError(dtype)


def dequantize(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Storage array -> float64 values (exact)."""
    if dtype == "f32":
        return np.asarray(bits, dtype=np.float32).astype(np.float64)
    b = np.asarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return b.view(np.float16).astype(np.float64)
    if dtype == "bf16":
        return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(dtype)


def storage_dtype(dtype: str):
    return np.float32 if dtype == "f32" else np.uint16


# ----------------------------------------------------------------------------
# configuration
# ----------------------------------------------------------------------------
@dataclass
class LayerConfig:
    name: str
    dtype: str                      # "f32" | "f16" | "bf16"
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_dev_blocks: int
    n_host_blocks: int
    n_adapters: int
    ranks: Tuple[int, ...]          # each adapter draws its rank uniformly from these
    projections: Tuple[str, ...]    # subset of q,k,v,o,gate,up,down
    n_seqs: int
    prefix_range: Tuple[int, int]   # inclusive
    new_range: Tuple[int, int]      # inclusive (used by prefill sequences)
    decode_frac: float = 0.0        # fraction of sequences with exactly 1 new token
    lora_scale: float = 1.0
    adapter_dist: str = "uniform"   # "uniform" | "zipf" | "distinct" | "skewed" (see _seq_adapters)
    zipf_alpha: float = 1.0
    swap_in_frac: float = 0.0       # share of reusable blocks that start on the host tier
    swap_out_frac: float = 0.0      # share (of reusable count) of idle blocks swapped out first
    block_tokens: int = 16
    mlp_dim: int = 0
    lora_std: float = 0.02
    seed: int = 20250503
    skew_std: float = 32.0          # standard deviation, in adapter ids, of the "skewed" distribution
    share_frac: float = 0.0         # probability that a sequence shares leading prefix blocks with an earlier
                                    # sequence of the same adapter (paper section 4.1: queries of one LoRA that
                                    # start alike hang below the same nodes; KV of different LoRAs is never shared)

    @property
    def block_elems(self) -> int:
        return 2 * self.block_tokens * self.n_kv_heads * self.head_dim

    @property
    def block_bytes(self) -> int:
        return self.block_elems * DTYPE_BYTES[self.dtype]

    def proj_dims(self, p: str) -> Tuple[int, int]:
        qd = self.n_q_heads * self.head_dim
        kd = self.n_kv_heads * self.head_dim
        return {
            "q": (self.hidden, qd), "k": (self.hidden, kd), "v": (self.hidden, kd),
            "o": (qd, self.hidden), "gate": (self.hidden, self.mlp_dim),
            "up": (self.hidden, self.mlp_dim), "down": (self.mlp_dim, self.hidden),
        }[p]

    def scaled(self, **kw) -> "LayerConfig":
        return dataclasses.replace(self, **kw)


def config(name: str) -> LayerConfig:
    """The five benchmark workloads (index 0..4 or by name)."""
    table = {
        "tiny": LayerConfig(
            "tiny", "f32", 256, 4, 4, 64, 128, 64, 4, (8,), ("q", "v"), 8,
            (0, 64), (1, 32), lora_scale=2.0, seed=20250503),
        "7b_prefill": LayerConfig(
            "7b_prefill", "f16", 4096, 32, 32, 128, 16384, 4096, 32, (16,),
            ("q", "k", "v", "o"), 64, (0, 2048), (128, 512),
            adapter_dist="zipf", zipf_alpha=1.0, swap_in_frac=0.4, seed=20250504),
        "7b_decode": LayerConfig(
            "7b_decode", "bf16", 4096, 32, 32, 128, 65536, 1024, 100, (8, 16, 32, 64),
            ("q", "k", "v", "o"), 256, (512, 4096), (1, 1), decode_frac=1.0,
            seed=20250505),
        "13b": LayerConfig(
            "13b", "f16", 5120, 40, 40, 128, 600000, 16384, 200, (32,),
            ("q", "k", "v", "o", "gate", "up", "down"), 128, (0, 4096), (128, 512),
            adapter_dist="zipf", zipf_alpha=1.2, swap_in_frac=0.25, swap_out_frac=0.25,
            mlp_dim=13824, seed=20250506),
        "34b_gqa": LayerConfig(
            "34b_gqa", "bf16", 8192, 64, 8, 128, 3750000, 65536, 500, (64,),
            ("q", "k", "v", "o"), 512, (0, 16384), (128, 512), decode_frac=0.75,
            adapter_dist="zipf", zipf_alpha=1.0, swap_in_frac=0.1, swap_out_frac=0.1,
            seed=20250507),
    }
    if isinstance(name, int):
        name = list(table)[name]
    return table[name]


CONFIG_NAMES = ("tiny", "7b_prefill", "7b_decode", "13b", "34b_gqa")


# ----------------------------------------------------------------------------
# one step of synthetic input
# ----------------------------------------------------------------------------
@dataclass
class LoraProj:
    name: str
    d_in: int
    d_out: int
    a_tab_off: np.ndarray   # int32[n_adapters]  start of the table holding this A's rows
    a_row_base: np.ndarray  # int32[n_adapters]  first page-row of A inside that table
    b_tab_off: np.ndarray
    b_row_base: np.ndarray


@dataclass
class Step:
    cfg: LayerConfig
    # sequences
    prefix_len: np.ndarray          # int32[S]
    new_len: np.ndarray             # int32[S]
    cu_new: np.ndarray              # int32[S+1]
    seq_adapter: np.ndarray         # int32[S]
    kv_tables: np.ndarray           # int32[S, max_blocks]  (-1 padded)
    token_adapter: np.ndarray       # int32[T]
    # adapters
    rank: np.ndarray                # int32[n_adapters] (0 = not resident)
    scale: np.ndarray               # float32[n_adapters]
    lora_tables: np.ndarray         # int32[...] concatenated per-adapter tables
    proj: Dict[str, LoraProj]
    # block contents: rows of `content` belong to device block ids `content_ids`
    content_ids: np.ndarray         # int32[n_touched]
    content: np.ndarray             # storage[n_touched, block_elems]
    lora_block_ids: np.ndarray
    prefix_block_ids: np.ndarray
    fresh_block_ids: np.ndarray
    # swap lists (host tier id <-> device id); contents of swapped-in blocks start on the host
    swap_in_host: np.ndarray
    swap_in_dev: np.ndarray
    swap_out_dev: np.ndarray
    swap_out_host: np.ndarray
    # activations (storage dtype)
    acts: Dict[str, np.ndarray] = field(default_factory=dict)

    @property
    def n_tokens(self) -> int:
        return int(self.cu_new[-1])


def rows_per_block(block_elems: int, row_len: int) -> int:
    return block_elems // row_len


def _popularity(cfg: LayerConfig, rng) -> np.ndarray:
    n = cfg.n_adapters
    if cfg.adapter_dist == "uniform":
        return np.full(n, 1.0 / n)
    w = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** cfg.zipf_alpha
    w /= w.sum()
    p = np.empty(n)
    p[rng.permutation(n)] = w          # popularity rank -> adapter id, seeded
    return p


def _seq_adapters(cfg: LayerConfig, rng, S: int) -> np.ndarray:
    """One adapter id per sequence.  "uniform" and "zipf" draw from a popularity vector; the other two
    are the paper's remaining LoRA distributions (section 6.9, the 1000 / 2000 LoRA experiment):
    "distinct" hands the adapters out in turn (sequence i gets adapter (first + i) mod n, first seeded),
    "skewed" rounds a normal deviate around the middle id with standard deviation skew_std."""
    n = cfg.n_adapters
    if cfg.adapter_dist == "distinct":
        first = int(rng.integers(0, n))
        return ((first + np.arange(S)) % n).astype(np.int32)
    if cfg.adapter_dist == "skewed":
        ids = np.rint(rng.normal(n / 2.0, cfg.skew_std, size=S)).astype(np.int64)
        return np.clip(ids, 0, n - 1).astype(np.int32)
    pop = _popularity(cfg, rng)
    return rng.choice(n, size=S, p=pop).astype(np.int32)


def make_step(cfg: LayerConfig, seed: Optional[int] = None,
              alloc_dev: Optional[Callable[[int], np.ndarray]] = None,
              alloc_host: Optional[Callable[[int], np.ndarray]] = None,
              poison_fresh: bool = True, with_acts: bool = True,
              fill_content: bool = True) -> Step:
    """Draw one step.  `alloc_dev(n)` / `alloc_host(n)` hand out block ids (for
    example the library's or the oracle's allocator); by default ids come from a
    seeded permutation of the id range, which is what a shuffled free list
    would return."""
    seed = cfg.seed if seed is None else seed
    rng = np.random.default_rng(seed)
    be = cfg.block_elems
    bt = cfg.block_tokens

    # (the id permutations are always drawn, so that a step has the same lengths and adapters
    # whoever hands out the block ids)
    perm_d = rng.permutation(cfg.n_dev_blocks).astype(np.int32)
    perm_h = rng.permutation(cfg.n_host_blocks).astype(np.int32)
    if alloc_dev is None:
        cur_d = [0]

        def alloc_dev(n):
            if cur_d[0] + n > len(perm_d):
                raise RuntimeError("synthetic workload needs more device blocks than the pool has")
            out = perm_d[cur_d[0]:cur_d[0] + n]
            cur_d[0] += n
            return out
    if alloc_host is None:
        cur_h = [0]

        def alloc_host(n):
            if cur_h[0] + n > len(perm_h):
                raise RuntimeError("synthetic workload needs more host blocks than the pool has")
            out = perm_h[cur_h[0]:cur_h[0] + n]
            cur_h[0] += n
            return out

    # ---- sequences -------------------------------------------------------
    S = cfg.n_seqs
    prefix_len = rng.integers(cfg.prefix_range[0], cfg.prefix_range[1] + 1, size=S).astype(np.int32)
    new_len = rng.integers(cfg.new_range[0], cfg.new_range[1] + 1, size=S).astype(np.int32)
    if cfg.decode_frac > 0:
        is_dec = rng.random(S) < cfg.decode_frac
        if cfg.decode_frac >= 1.0:
            is_dec[:] = True
        new_len[is_dec] = 1
    cu_new = np.zeros(S + 1, dtype=np.int32)
    cu_new[1:] = np.cumsum(new_len)
    T = int(cu_new[-1])
    seq_adapter = _seq_adapters(cfg, rng, S)
    token_adapter = np.repeat(seq_adapter, new_len).astype(np.int32)

    # ---- adapters present in the batch get pages --------------------------
    all_rank = rng.choice(np.asarray(cfg.ranks), size=cfg.n_adapters).astype(np.int32)
    present = np.unique(seq_adapter)
    rank = np.zeros(cfg.n_adapters, dtype=np.int32)
    rank[present] = all_rank[present]
    scale = np.full(cfg.n_adapters, cfg.lora_scale, dtype=np.float32)

    projs: Dict[str, LoraProj] = {}
    for p in cfg.projections:
        d_in, d_out = cfg.proj_dims(p)
        z = lambda: np.zeros(cfg.n_adapters, dtype=np.int32)
        projs[p] = LoraProj(p, d_in, d_out, z(), z(), z(), z())
    tables: List[np.ndarray] = []
    tab_cursor = 0
    lora_blocks: List[np.ndarray] = []
    for a in present:
        r = int(rank[a])
        # one table per distinct row length; matrices packed in projection order, A then B
        by_len: Dict[int, int] = {}
        place: List[Tuple[str, str, int, int]] = []
        for p in cfg.projections:
            d_in, d_out = cfg.proj_dims(p)
            for which, ln in (("a", d_in), ("b", d_out)):
                base = by_len.get(ln, 0)
                place.append((p, which, ln, base))
                by_len[ln] = base + r
        tab_off_of: Dict[int, int] = {}
        for ln, nrows in by_len.items():
            nblk = -(-nrows // rows_per_block(be, ln))
            ids = np.asarray(alloc_dev(nblk), dtype=np.int32)
            tab_off_of[ln] = tab_cursor
            tables.append(ids)
            lora_blocks.append(ids)
            tab_cursor += nblk
        for p, which, ln, base in place:
            if which == "a":
                projs[p].a_tab_off[a] = tab_off_of[ln]
                projs[p].a_row_base[a] = base
            else:
                projs[p].b_tab_off[a] = tab_off_of[ln]
                projs[p].b_row_base[a] = base
    lora_tables = np.concatenate(tables).astype(np.int32) if tables else np.zeros(0, np.int32)
    lora_block_ids = np.concatenate(lora_blocks).astype(np.int32) if lora_blocks else np.zeros(0, np.int32)

    # ---- KV block tables ---------------------------------------------------
    tot = prefix_len.astype(np.int64) + new_len
    nblk = (tot + bt - 1) // bt
    npre = (prefix_len.astype(np.int64) + bt - 1) // bt        # blocks that hold reusable prefix KV
    max_blocks = int(max(1, nblk.max()))
    kv_tables = np.full((S, max_blocks), -1, dtype=np.int32)
    pre_ids: List[np.ndarray] = []
    fresh_ids: List[np.ndarray] = []
    # shared prefixes: a sequence may reuse the physical blocks of the leading FULL prefix blocks of an earlier
    # sequence with the same adapter (a random number of them, at least one); the block that its own new tokens
    # continue in is never shared.  Drawn only when the knob is on, so other workloads keep their streams.
    n_shared = np.zeros(S, dtype=np.int64)
    donor = np.full(S, -1, dtype=np.int64)
    if cfg.share_frac > 0:
        last_of: Dict[int, int] = {}
        for i in range(S):
            a = int(seq_adapter[i])
            j = last_of.get(a, -1)
            if j >= 0 and rng.random() < cfg.share_frac:
                room = min(int(prefix_len[i]) // bt, int(prefix_len[j]) // bt)
                if room > 0:
                    n_shared[i] = int(rng.integers(1, room + 1))
                    donor[i] = j
            last_of[a] = i
    for i in range(S):
        ns = int(n_shared[i])
        own = np.asarray(alloc_dev(int(nblk[i]) - ns), dtype=np.int32)
        ids = np.concatenate([kv_tables[donor[i], :ns], own]).astype(np.int32) if ns else own
        kv_tables[i, :len(ids)] = ids
        pre_ids.append(ids[ns:int(npre[i])])
        fresh_ids.append(ids[int(npre[i]):])
    prefix_block_ids = np.concatenate(pre_ids).astype(np.int32)
    fresh_block_ids = np.concatenate(fresh_ids).astype(np.int32)

    # ---- swap lists ---------------------------------------------------------
    reusable = np.concatenate([lora_block_ids, prefix_block_ids])
    n_in = int(round(cfg.swap_in_frac * len(reusable)))
    pick = rng.permutation(len(reusable))[:n_in]
    swap_in_dev = reusable[np.sort(pick)].astype(np.int32)
    swap_in_host = np.asarray(alloc_host(n_in), dtype=np.int32)
    n_out = int(round(cfg.swap_out_frac * len(reusable)))
    swap_out_dev = np.asarray(alloc_dev(n_out), dtype=np.int32)     # idle resident blocks
    swap_out_host = np.asarray(alloc_host(n_out), dtype=np.int32)

    # ---- block contents -----------------------------------------------------
    content_ids = np.concatenate([lora_block_ids, prefix_block_ids, fresh_block_ids, swap_out_dev]).astype(np.int32)
    sd = storage_dtype(cfg.dtype)
    if fill_content:
        content = np.empty((len(content_ids), be), dtype=sd)
        n_l, n_p, n_f = len(lora_block_ids), len(prefix_block_ids), len(fresh_block_ids)
        _fill_normal(content[:n_l], cfg.lora_std, cfg.dtype, rng)
        _fill_normal(content[n_l:n_l + n_p], 1.0, cfg.dtype, rng)
        if poison_fresh:
            # recycled blocks hold arbitrary old bits: use NaN patterns so that any
            # slot read beyond a sequence's length shows up in the result
            content[n_l + n_p:n_l + n_p + n_f] = (np.float32(np.nan) if cfg.dtype == "f32"
                                                  else (0x7E00 if cfg.dtype == "f16" else 0x7FC0))
        else:
            _fill_normal(content[n_l + n_p:n_l + n_p + n_f], 1.0, cfg.dtype, rng)
        _fill_normal(content[n_l + n_p + n_f:], 1.0, cfg.dtype, rng)
    else:
        content = np.empty((0, be), dtype=sd)

    st = Step(cfg, prefix_len, new_len, cu_new, seq_adapter, kv_tables, token_adapter,
              rank, scale, lora_tables, projs, content_ids, content,
              lora_block_ids, prefix_block_ids, fresh_block_ids,
              swap_in_host, swap_in_dev, swap_out_dev, swap_out_host)

    if with_acts:
        qd = cfg.n_q_heads * cfg.head_dim
        kd = cfg.n_kv_heads * cfg.head_dim
        acts = st.acts
        acts["x"] = _normal((T, cfg.hidden), 1.0, cfg.dtype, rng)
        acts["q"] = _normal((T, qd), 1.0, cfg.dtype, rng)
        acts["k_new"] = _normal((T, kd), 1.0, cfg.dtype, rng)
        acts["v_new"] = _normal((T, kd), 1.0, cfg.dtype, rng)
        for p in cfg.projections:
            d_in, d_out = cfg.proj_dims(p)
            acts["base_" + p] = _normal((T, d_out), 1.0, cfg.dtype, rng)
            if d_in != cfg.hidden and ("x_" + str(d_in)) not in acts:
                acts["x_" + str(d_in)] = _normal((T, d_in), 1.0, cfg.dtype, rng)
    return st


def _normal(shape, std, dtype, rng) -> np.ndarray:
    out = np.empty(shape, dtype=storage_dtype(dtype))
    _fill_normal(out.reshape(-1), std, dtype, rng)
    return out


def _fill_normal(dst: np.ndarray, std: float, dtype: str, rng, chunk: int = 1 << 22) -> None:
    """Fill with N(0, std^2) rounded to `dtype`.  Each chunk draws from its own child
    stream (keyed by the parent stream and the chunk index), so the result does not
    depend on how many threads do the work."""
    flat = dst.reshape(-1)
    n = flat.shape[0]
    if n == 0:
        return
    n_chunks = -(-n // chunk)
    base = int(rng.integers(0, 2 ** 63 - 1))

    def work(ci):
        lo, hi = ci * chunk, min(n, (ci + 1) * chunk)
        g = np.random.Generator(np.random.Philox(key=[base, ci]))
        v = g.standard_normal(hi - lo, dtype=np.float32)
        if std != 1.0:
            v *= np.float32(std)
        flat[lo:hi] = quantize(v, dtype)

    if n_chunks == 1:
        work(0)
    else:
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(work, range(n_chunks)))


def expected_distinct_adapters(pop: Sequence[float], batch: int) -> float:
    """Expected number of distinct adapters among `batch` independent draws,
    sum_i 1 - (1 - p_i)^batch  (paper Eq. 3 uses the same expression to size the
    adapter set a batch needs)."""
    p = np.asarray(pop, dtype=np.float64)
    return float(np.sum(1.0 - (1.0 - p) ** batch))
