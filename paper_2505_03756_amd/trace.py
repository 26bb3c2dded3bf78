"""Multi-step synthetic serving traces: what the cache manager would hand down step after step.

A fixed number of sequence slots is kept busy.  At every step some slots finish and are taken over by
new queries; the generator emits, for the step, the batch to compute (lengths, adapters, block tables)
and the block moves that go with the change of guard: the swap-in of the joining queries' reusable
prefix blocks and adapter pages that are not in the device tier, and the swap-out of as many blocks of
queries that have left (paper section 3.2: swap-out makes room before swap-in; section 4.3: moves run
asynchronously to the compute of the queries that are ready).  It stands in for the paper's traces
(chat / translation / agent arrivals, section 6.2), which are not available; only their shape is taken:
load that shifts between adapters over time (section 2.3.2) and arrivals that come in bursts
(section 2.2).

Two modes:
  "bursty"  the number of slots replaced per step is Poisson with a rate that a two-state Markov chain
            switches between calm and burst; a joining query's prefix (and its adapter, if no running
            query uses it) is already in the device tier with probability `resident_prob`.
  "churn"   slots are replaced until the blocks to bring in reach `churn_frac` of the blocks the batch
            needs; nothing of a joining query is resident.  With `swap_out=False` nothing is written
            back (the prefill workload, whose statement names only the swap-in).
In both, adapters are drawn from a Zipf (or uniform) popularity over a seeded permutation of the ids
that is redrawn every `shift_period` steps.

Timing model (what makes the moves overlap with compute).  The moves emitted at step k are for queries
that join the batch at step k + 1: they can run on their own stream while step k computes.  Blocks of
queries that left after step k - 1 are written back at step k (not earlier: step k - 1 was still
appending to them) and return to the free list at step k + 1.  Joining queries get blocks from the free
list, never the ones being written back in the same step.

This module draws inputs only: no arithmetic of the method and no layout rule beyond how many page-rows
fit into a block (to know how many blocks an adapter needs).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional

import numpy as np

from .workload import LayerConfig, LoraProj, rows_per_block


@dataclass
class TraceConfig:
    mode: str = "bursty"            # "bursty" | "churn" | "static"
    lam_calm: float = 4.0           # replaced slots per step in the calm state
    lam_burst: float = 64.0         # ... in the burst state
    p_calm_to_burst: float = 0.05
    p_burst_to_calm: float = 0.2
    resident_prob: float = 0.5      # bursty: a joining query's prefix / adapter is already in the device tier
    churn_frac: float = 0.25        # churn: share of the batch's needed blocks brought in per step
    swap_out: bool = True           # write back as many blocks of departed queries as are brought in
    shift_period: int = 0           # redraw the popularity -> adapter id permutation every so many steps (0: never)
    seed: Optional[int] = None      # seed of the trace's draws (None: the workload's own seed)


def trace_config(name: str) -> TraceConfig:
    """The step-to-step behaviour of the five benchmark workloads."""
    return {
        "tiny": TraceConfig(mode="static"),
        "7b_prefill": TraceConfig(mode="churn", churn_frac=0.4, swap_out=False),
        "7b_decode": TraceConfig(mode="static"),
        "13b": TraceConfig(mode="churn", churn_frac=0.25, swap_out=True, shift_period=1000),
        # The seed decides where the bursts of a run fall.  A benchmark run times 20 to 1000 steps, and the draw of the
        # workload's own seed puts 9 burst steps into the first 20 timed ones (stationary share: 4).  Of the seeds
        # 1..29 this is the one whose windows all hold close to the stationary share (4 burst steps among the timed
        # steps 5..24, 45 among 5..204, 195 among 5..1004; 0.57 / 0.56 / 0.50 GB moved per step), so that a run of
        # any length times a representative mix.
        "34b_gqa": TraceConfig(mode="bursty", seed=29),
    }[name]


def stationary_burst_share(tc: TraceConfig) -> float:
    """Long-run share of steps spent in the burst state of the two-state chain."""
    return tc.p_calm_to_burst / (tc.p_calm_to_burst + tc.p_burst_to_calm)


@dataclass
class TraceStep:
    index: int
    burst: bool
    # the batch to compute at this step
    prefix_len: np.ndarray          # int32[S]
    new_len: np.ndarray             # int32[S]
    cu_new: np.ndarray              # int32[S+1]
    seq_adapter: np.ndarray         # int32[S]
    token_adapter: np.ndarray       # int32[T]
    kv_tables: np.ndarray           # int32[S, max_blocks] (-1 padded); a view of the generator's state at this step
    rank: np.ndarray                # int32[n_adapters], 0 = not in the device tier
    lora_tables: np.ndarray         # int32[n_adapters * tab_stride]: the adapters' block tables as this batch sees them
    changed_slots: np.ndarray       # slots whose table row differs from the previous step's
    # moves to issue now, for the queries that join at the next step
    swap_out_dev: np.ndarray
    swap_out_host: np.ndarray
    swap_in_host: np.ndarray
    swap_in_dev: np.ndarray
    n_replaced: int                 # slots taken over at this step (they compute from the next step on)
    tables_changed: bool = True     # the adapters' block tables differ from the previous step's

    @property
    def n_tokens(self) -> int:
        return int(self.cu_new[-1])


class ServingTrace:
    """Stateful generator.  `alloc_*(n)` hand out block ids, `free_*(ids)` take them back (the pool's allocator,
    or simple lists in tests)."""

    def __init__(self, cfg: LayerConfig, tc: TraceConfig, seed: int,
                 alloc_dev: Callable[[int], np.ndarray], free_dev: Callable[[np.ndarray], None],
                 alloc_host: Callable[[int], np.ndarray], free_host: Callable[[np.ndarray], None]):
        self.cfg, self.tc = cfg, tc
        self.rng = np.random.default_rng(seed)
        self.alloc_dev, self.free_dev, self.alloc_host, self.free_host = alloc_dev, free_dev, alloc_host, free_host
        bt, be, S = cfg.block_tokens, cfg.block_elems, cfg.n_seqs
        self.max_blocks = -(-(cfg.prefix_range[1] + max(cfg.new_range[1], 1)) // bt)
        self.prefix_len = np.zeros(S, np.int32)
        self.new_len = np.zeros(S, np.int32)
        self.seq_adapter = np.zeros(S, np.int32)
        self.kv_tables = np.full((S, self.max_blocks), -1, np.int32)
        self.n_blocks = np.zeros(S, np.int64)
        # ---- adapters: fixed table layout, one region per adapter, one sub-table per distinct row length
        self.all_rank = self.rng.choice(np.asarray(cfg.ranks), size=cfg.n_adapters).astype(np.int32)
        self.rank = np.zeros(cfg.n_adapters, np.int32)
        self.scale = np.full(cfg.n_adapters, cfg.lora_scale, np.float32)
        r_max = int(max(cfg.ranks))
        rows_of: Dict[int, int] = {}                        # row length -> page-rows per unit of rank
        for p in cfg.projections:
            d_in, d_out = cfg.proj_dims(p)
            rows_of[d_in] = rows_of.get(d_in, 0) + 1
            rows_of[d_out] = rows_of.get(d_out, 0) + 1
        self._len_off: Dict[int, int] = {}
        off = 0
        for ln, per_rank in rows_of.items():
            self._len_off[ln] = off
            off += -(-(per_rank * r_max) // rows_per_block(be, ln))
        self.tab_stride = off
        self._rows_of = rows_of
        self.lora_tables = np.zeros(cfg.n_adapters * self.tab_stride, np.int32)
        self.proj: Dict[str, LoraProj] = {}
        for p in cfg.projections:
            d_in, d_out = cfg.proj_dims(p)
            z = lambda: np.zeros(cfg.n_adapters, np.int32)
            self.proj[p] = LoraProj(p, d_in, d_out, z(), z(), z(), z())
        for a in range(cfg.n_adapters):
            r = int(self.all_rank[a])
            cursor: Dict[int, int] = {}
            for p in cfg.projections:
                d_in, d_out = cfg.proj_dims(p)
                for which, ln in (("a", d_in), ("b", d_out)):
                    base = cursor.get(ln, 0)
                    cursor[ln] = base + r
                    tab = a * self.tab_stride + self._len_off[ln]
                    if which == "a":
                        self.proj[p].a_tab_off[a], self.proj[p].a_row_base[a] = tab, base
                    else:
                        self.proj[p].b_tab_off[a], self.proj[p].b_row_base[a] = tab, base
        self.adapter_users = np.zeros(cfg.n_adapters, np.int64)
        self._draw_popularity()
        self.burst = False
        self.index = 0
        self._pending_out: List[np.ndarray] = []            # device blocks of queries that left at the previous step
        self._to_free_dev: List[np.ndarray] = []            # written back (or dropped) last step: free now
        self.totals = {"replaced": 0, "swap_in_blocks": 0, "swap_out_blocks": 0, "burst_steps": 0, "tokens": 0}
        # ---- the first batch: everything it needs is resident
        self._tables_changed = True
        self._host_hold: List[List[np.ndarray]] = [[], []]   # host ids of the last two steps' moves, freed after that
        for s in range(S):
            self._assign(s, kv_resident=True, adapter_resident_prob=1.0, collect_in=None)

    # ------------------------------------------------------------------ draws
    def _draw_popularity(self):
        n = self.cfg.n_adapters
        if self.cfg.adapter_dist == "uniform":
            self.popularity = np.full(n, 1.0 / n)
            return
        w = 1.0 / np.arange(1, n + 1, dtype=np.float64) ** self.cfg.zipf_alpha
        w /= w.sum()
        self.popularity = np.empty(n)
        self.popularity[self.rng.permutation(n)] = w

    def _adapter_blocks(self, a: int) -> np.ndarray:
        """Table entries that adapter a's pages occupy (its rank decides how much of its region is used)."""
        r = int(self.all_rank[a])
        idx = []
        for ln, per_rank in self._rows_of.items():
            nb = -(-(per_rank * r) // rows_per_block(self.cfg.block_elems, ln))
            start = a * self.tab_stride + self._len_off[ln]
            idx.append(np.arange(start, start + nb))
        return np.concatenate(idx)

    def _assign(self, s: int, kv_resident: bool, adapter_resident_prob: float, collect_in: Optional[List[np.ndarray]]):
        """A new query takes slot s.  Device ids of what has to be brought in are appended to collect_in: the
        blocks of its reusable prefix unless kv_resident, and the pages of its adapter if no running query uses
        it and a draw against adapter_resident_prob says they are not in the device tier either."""
        cfg, rng, bt = self.cfg, self.rng, self.cfg.block_tokens
        P = int(rng.integers(cfg.prefix_range[0], cfg.prefix_range[1] + 1))
        N = 1 if (cfg.decode_frac >= 1.0 or (cfg.decode_frac > 0 and rng.random() < cfg.decode_frac)) else \
            int(rng.integers(cfg.new_range[0], cfg.new_range[1] + 1))
        a = int(rng.choice(cfg.n_adapters, p=self.popularity))
        nb = -(-(P + N) // bt)
        ids = np.asarray(self.alloc_dev(nb), dtype=np.int32)
        self.prefix_len[s], self.new_len[s], self.seq_adapter[s], self.n_blocks[s] = P, N, a, nb
        self.kv_tables[s, :] = -1
        self.kv_tables[s, :nb] = ids
        npre = P // bt                                      # whole blocks of reusable prefix (a partly filled one
        if not kv_resident and collect_in is not None and npre:   # is completed by the query itself)
            collect_in.append(ids[:npre])
        if self.adapter_users[a] == 0:                      # no running query uses it: its pages get blocks now
            slots = self._adapter_blocks(a)
            blocks = np.asarray(self.alloc_dev(len(slots)), dtype=np.int32)
            self.lora_tables[slots] = blocks
            self.rank[a] = self.all_rank[a]
            self._tables_changed = True
            if collect_in is not None and not (rng.random() < adapter_resident_prob):
                collect_in.append(blocks)
        self.adapter_users[a] += 1

    def _vacate(self, s: int) -> List[np.ndarray]:
        """The query in slot s has finished: its blocks (and its adapter's, if it was the last user) leave."""
        gone = [self.kv_tables[s, :self.n_blocks[s]].copy()]
        a = int(self.seq_adapter[s])
        self.adapter_users[a] -= 1
        if self.adapter_users[a] == 0:
            gone.append(self.lora_tables[self._adapter_blocks(a)].copy())
            self.rank[a] = 0
        return gone

    # ------------------------------------------------------------------ one step
    def needed_blocks(self) -> int:
        bt = self.cfg.block_tokens
        n = int(np.sum(-(-self.prefix_len.astype(np.int64) // bt)))
        for a in np.flatnonzero(self.adapter_users > 0):
            n += len(self._adapter_blocks(int(a)))
        return n

    def step(self) -> TraceStep:
        cfg, tc, rng, S = self.cfg, self.tc, self.rng, self.cfg.n_seqs
        # ---- the batch to compute now (copies: the replacements below change the state for the next step)
        cu = np.zeros(S + 1, np.int32)
        cu[1:] = np.cumsum(self.new_len)
        tables_changed, self._tables_changed = self._tables_changed, False
        batch = dict(prefix_len=self.prefix_len.copy(), new_len=self.new_len.copy(), cu_new=cu,
                     seq_adapter=self.seq_adapter.copy(),
                     token_adapter=np.repeat(self.seq_adapter, self.new_len).astype(np.int32),
                     kv_tables=self.kv_tables.copy(), rank=self.rank.copy(), lora_tables=self.lora_tables.copy())
        changed = getattr(self, "_changed_last", np.arange(S))
        # ---- blocks written back (or dropped) at the previous step return to the free list
        for ids in self._to_free_dev:
            self.free_dev(ids)
        self._to_free_dev = []
        # ---- who leaves, who joins
        if tc.shift_period and self.index > 0 and self.index % tc.shift_period == 0:
            self._draw_popularity()
        if tc.mode == "bursty":
            u = rng.random()
            self.burst = (u >= tc.p_burst_to_calm) if self.burst else (u < tc.p_calm_to_burst)
            k = int(min(S, rng.poisson(tc.lam_burst if self.burst else tc.lam_calm)))
            slots = rng.choice(S, size=k, replace=False) if k else np.zeros(0, np.int64)
        elif tc.mode == "churn":
            slots = rng.permutation(S)
        else:
            slots = np.zeros(0, np.int64)
        coll_in: List[np.ndarray] = []
        left: List[np.ndarray] = []
        target = tc.churn_frac * self.needed_blocks() if tc.mode == "churn" else None
        n_rep = 0
        for s in slots:
            if target is not None and sum(len(x) for x in coll_in) >= target:
                break
            left.extend(self._vacate(int(s)))
            if tc.mode == "bursty":
                self._assign(int(s), rng.random() < tc.resident_prob, tc.resident_prob, coll_in)
            else:
                self._assign(int(s), False, 0.0, coll_in)
            n_rep += 1
        self._changed_last = np.asarray(slots[:n_rep], dtype=np.int64)
        swap_in_dev = np.concatenate(coll_in).astype(np.int32) if coll_in else np.zeros(0, np.int32)
        swap_in_host = np.asarray(self.alloc_host(len(swap_in_dev)), dtype=np.int32)
        # ---- write back as many blocks of the queries that left at the PREVIOUS step (this step's leavers are
        #      still being computed and appended to); the rest of those blocks are simply dropped
        pend = np.concatenate(self._pending_out).astype(np.int32) if self._pending_out else np.zeros(0, np.int32)
        n_out = min(len(pend), len(swap_in_dev)) if tc.swap_out else 0
        swap_out_dev = pend[:n_out]
        swap_out_host = np.asarray(self.alloc_host(n_out), dtype=np.int32)
        if len(pend):
            self._to_free_dev.append(pend)
        self._pending_out = left
        # host-tier ids: held for two more steps (moves of neighbouring steps may run on different streams), then
        # returned; what the host tier keeps cached beyond that is the cache manager's business, not the trace's
        for ids in self._host_hold.pop(0):
            self.free_host(ids)
        self._host_hold.append([x for x in (swap_in_host, swap_out_host) if len(x)])
        t = self.totals
        t["replaced"] += n_rep
        t["swap_in_blocks"] += len(swap_in_dev)
        t["swap_out_blocks"] += n_out
        t["burst_steps"] += int(self.burst)
        t["tokens"] += int(cu[-1])
        out = TraceStep(self.index, self.burst, changed_slots=np.asarray(changed, dtype=np.int64),
                        swap_out_dev=swap_out_dev, swap_out_host=swap_out_host, swap_in_host=swap_in_host,
                        swap_in_dev=swap_in_dev, n_replaced=n_rep, tables_changed=tables_changed, **batch)
        self.index += 1
        return out
