"""The multi-step trace generator (paper_2505_03756_amd/trace.py): the bursty arrival chain, the popularity
that shifts between adapters, and the invariants of the block moves it emits.  Inputs only: no arithmetic of
the method is involved."""
import numpy as np
import pytest

from paper_2505_03756_amd import trace as tr
from paper_2505_03756_amd import workload as wl


class ListAllocator:
    """LIFO free list (what the pool's allocator does), with double-free and leak checks."""

    def __init__(self, n):
        self.free, self.out = list(range(n - 1, -1, -1)), set()

    def alloc(self, n):
        assert n <= len(self.free), "out of blocks"
        ids = [self.free.pop() for _ in range(n)]
        self.out.update(ids)
        return np.asarray(ids, np.int32)

    def release(self, ids):
        for i in ids:
            assert int(i) in self.out, "freed a block that was not allocated"
            self.out.discard(int(i))
            self.free.append(int(i))


def small(**kw):
    base = dict(name="trace", dtype="f16", hidden=256, n_q_heads=2, n_kv_heads=2, head_dim=64, n_dev_blocks=60000,
                n_host_blocks=60000, n_adapters=40, ranks=(8, 16), projections=("q", "k", "v", "o"), n_seqs=96,
                prefix_range=(0, 300), new_range=(4, 40), decode_frac=0.5, adapter_dist="zipf", zipf_alpha=1.0, seed=3)
    base.update(kw)
    return wl.LayerConfig(**base)


def make(cfg, tc, seed=11):
    d, h = ListAllocator(cfg.n_dev_blocks), ListAllocator(cfg.n_host_blocks)
    return tr.ServingTrace(cfg, tc, seed, d.alloc, d.release, h.alloc, h.release), d, h


def test_bursty_chain_matches_its_closed_forms():
    """Two-state Markov-modulated Poisson arrivals: the long-run share of burst steps is p_cb / (p_cb + p_bc) = 0.2,
    the mean number of replaced slots 0.8 * 4 + 0.2 * 64 = 16, the mean length of a burst 1 / p_bc = 5 steps."""
    tc = tr.TraceConfig(mode="bursty")
    assert tr.stationary_burst_share(tc) == pytest.approx(0.2)
    cfg = small(n_seqs=128, prefix_range=(0, 40), new_range=(1, 4))
    t, _, _ = make(cfg, tc)
    n = 6000
    burst, rep = np.zeros(n, bool), np.zeros(n)
    for k in range(n):
        st = t.step()
        burst[k], rep[k] = st.burst, st.n_replaced
    assert abs(burst.mean() - 0.2) < 0.03
    assert abs(rep[~burst].mean() - 4.0) < 0.25 and abs(rep[burst].mean() - 64.0) < 1.5
    assert abs(rep.mean() - (0.8 * 4 + 0.2 * 64)) < 2.0
    runs = np.diff(np.flatnonzero(np.diff(np.concatenate([[0], burst.astype(int), [0]]))))[::2]
    assert abs(runs.mean() - 5.0) < 0.8


def test_popularity_shift_and_distinct_adapters_per_phase():
    """Churn mode with a popularity that is redrawn every `shift_period` steps (paper section 2.3.2: the load moves
    between adapters).  Inside a phase the number of distinct adapters in the batch follows Eq. 3's expression
    sum_i 1 - (1 - p_i)^BS; across a shift the hot adapters change."""
    cfg = small(n_adapters=60, zipf_alpha=1.2, decode_frac=0.0, n_seqs=64)
    tc = tr.TraceConfig(mode="churn", churn_frac=0.5, shift_period=40)
    t, _, _ = make(cfg, tc)
    expect = wl.expected_distinct_adapters(t.popularity, cfg.n_seqs)
    pops, distinct, hot = [], [], []
    for k in range(120):
        st = t.step()
        pops.append(t.popularity.copy())
        if k % 40 >= 15:                                  # the batch has turned over since the last shift
            distinct.append(len(np.unique(st.seq_adapter)))
        if k % 40 == 39:
            hot.append(np.bincount(st.seq_adapter, minlength=60).argmax())
    assert abs(np.mean(distinct) - expect) < 2.5, (np.mean(distinct), expect)
    assert np.array_equal(pops[5], pops[38]) and not np.array_equal(pops[38], pops[41])
    assert np.allclose(np.sort(pops[0]), np.sort(pops[100]))       # the same Zipf weights, dealt to other ids
    assert [int(np.argmax(pops[39])), int(np.argmax(pops[79])), int(np.argmax(pops[119]))] == [int(h) for h in hot]
    assert len(set(int(h) for h in hot)) >= 2


@pytest.mark.parametrize("mode", ["bursty", "churn", "churn_in_only", "static"])
def test_moves_and_tables_stay_consistent(mode):
    tc = {"bursty": tr.TraceConfig(mode="bursty", lam_calm=3, lam_burst=30),
          "churn": tr.TraceConfig(mode="churn", churn_frac=0.25, shift_period=7),
          "churn_in_only": tr.TraceConfig(mode="churn", churn_frac=0.4, swap_out=False),
          "static": tr.TraceConfig(mode="static")}[mode]
    cfg = small()
    t, dev, host = make(cfg, tc)
    bt = cfg.block_tokens
    prev_tables = None
    written_back = set()
    for k in range(60):
        st = t.step()
        S = cfg.n_seqs
        # the batch: lengths, tokens, adapters
        assert st.cu_new[0] == 0 and np.array_equal(np.diff(st.cu_new), st.new_len)
        assert np.array_equal(st.token_adapter, np.repeat(st.seq_adapter, st.new_len))
        assert np.array_equal(np.flatnonzero(st.rank > 0), np.unique(st.seq_adapter))
        nb = -(-(st.prefix_len.astype(np.int64) + st.new_len) // bt)
        used = [st.kv_tables[i, :nb[i]] for i in range(S)]
        assert all((u >= 0).all() for u in used) and all((st.kv_tables[i, nb[i]:] == -1).all() for i in range(S))
        flat = np.concatenate(used)
        assert len(np.unique(flat)) == len(flat)                     # no block in two tables (no sharing here)
        # rows that the step says did not change did not
        if prev_tables is not None:
            same = np.setdiff1d(np.arange(S), st.changed_slots)
            assert np.array_equal(st.kv_tables[same], prev_tables[same])
        prev_tables = st.kv_tables.copy()
        # moves: destinations distinct, nothing both written back and filled in one step, sizes as stated
        assert len(st.swap_in_dev) == len(st.swap_in_host) and len(st.swap_out_dev) == len(st.swap_out_host)
        assert len(np.unique(st.swap_in_dev)) == len(st.swap_in_dev)
        assert len(np.unique(st.swap_out_host)) == len(st.swap_out_host)
        assert not np.intersect1d(st.swap_in_dev, st.swap_out_dev).size
        assert not np.intersect1d(st.swap_in_host, st.swap_out_host).size
        if tc.mode == "static":
            assert st.n_replaced == 0 and not len(st.swap_in_dev)
        if not tc.swap_out:
            assert not len(st.swap_out_dev)
        else:
            assert len(st.swap_out_dev) <= len(st.swap_in_dev)       # "an equal-size swap-out", as far as leavers go
        # what is brought in belongs to the NEXT batch (current generator state), never to blocks of this batch's
        # unchanged sequences; what is written back is in no current table
        nxt = t.kv_tables[t.kv_tables >= 0]
        lora_now = np.concatenate([t.lora_tables[t._adapter_blocks(int(a))] for a in np.flatnonzero(t.adapter_users)])
        assert np.isin(st.swap_in_dev, np.concatenate([nxt, lora_now])).all()
        assert not np.isin(st.swap_out_dev, np.concatenate([nxt, lora_now, flat])).any()
        written_back.update(int(b) for b in st.swap_out_dev)
    # block conservation: everything handed out is in a table, an adapter's pages, or waiting to be written back / freed
    held = set(int(b) for b in t.kv_tables[t.kv_tables >= 0])
    held |= set(int(b) for a in np.flatnonzero(t.adapter_users) for b in t.lora_tables[t._adapter_blocks(int(a))])
    held |= set(int(b) for ids in t._pending_out for b in ids) | set(int(b) for ids in t._to_free_dev for b in ids)
    assert held == dev.out
    if tc.mode != "static" and tc.swap_out:
        assert len(written_back) > 0


def test_trace_is_a_function_of_its_seed():
    cfg = small()
    a, _, _ = make(cfg, tr.TraceConfig(mode="bursty"), seed=5)
    b, _, _ = make(cfg, tr.TraceConfig(mode="bursty"), seed=5)
    c, _, _ = make(cfg, tr.TraceConfig(mode="bursty"), seed=6)
    sa, sb, sc = [x.step() for x in (a, b, c)]
    for _ in range(10):
        sa, sb, sc = a.step(), b.step(), c.step()
    assert np.array_equal(sa.kv_tables, sb.kv_tables) and np.array_equal(sa.swap_in_dev, sb.swap_in_dev)
    assert not np.array_equal(sa.prefix_len, sc.prefix_len)


def test_benchmark_workloads_have_their_trace_shapes():
    assert tr.trace_config("34b_gqa").mode == "bursty" and tr.trace_config("13b").shift_period == 1000
    assert tr.trace_config("13b").churn_frac == 0.25 and tr.trace_config("13b").swap_out
    assert tr.trace_config("7b_prefill").churn_frac == 0.4 and not tr.trace_config("7b_prefill").swap_out
    assert tr.trace_config("7b_decode").mode == "static" and tr.trace_config("tiny").mode == "static"
    # the prefill workload brings in 40 % of what the batch needs, step after step
    cfg = wl.config("7b_prefill").scaled(n_dev_blocks=40000, n_host_blocks=40000)
    t, _, _ = make(cfg, tr.trace_config("7b_prefill"))
    shares = []
    for k in range(12):
        need = t.needed_blocks()
        st = t.step()
        shares.append(len(st.swap_in_dev) / need)
    assert 0.38 < np.mean(shares) < 0.47, shares
