"""The seeded input generator: the adapter distributions of the paper's 1000 / 2000 LoRA experiment
(section 6.9) and the invariants every drawn step has.  No arithmetic of the method is involved."""
import numpy as np
import pytest

from paper_2505_03756_amd import workload as wl


def cfg(**kw):
    base = dict(name="gen", dtype="f16", hidden=256, n_q_heads=2, n_kv_heads=2, head_dim=64, n_dev_blocks=30000,
                n_host_blocks=64, n_adapters=1000, ranks=(8,), projections=("q", "v"), n_seqs=400,
                prefix_range=(0, 0), new_range=(1, 3), seed=5)
    base.update(kw)
    return wl.LayerConfig(**base)


def seq_adapters(step):
    return step.token_adapter[step.cu_new[:-1]]


def test_distinct_hands_adapters_out_in_turn():
    step = wl.make_step(cfg(adapter_dist="distinct"), with_acts=False, fill_content=False)
    a = seq_adapters(step).astype(np.int64)
    assert len(np.unique(a)) == 400                         # fewer sequences than adapters: all different
    assert np.all((a[1:] - a[:-1]) % 1000 == 1)             # consecutive ids, wrapping at n
    step = wl.make_step(cfg(adapter_dist="distinct", n_adapters=64), with_acts=False, fill_content=False)
    counts = np.bincount(seq_adapters(step), minlength=64)
    assert counts.max() - counts.min() <= 1                 # polling: loads differ by at most one query


def test_uniform_over_many_adapters_matches_eq3_expectation():
    # expected number of distinct adapters among BS queries = n (1 - (1 - 1/n)^BS): Eq. 3 with equal probabilities
    n, S = 1000, 400
    expect = n * (1.0 - (1.0 - 1.0 / n) ** S)
    got = [len(np.unique(seq_adapters(wl.make_step(cfg(adapter_dist="uniform", seed=s), with_acts=False,
                                                   fill_content=False)))) for s in range(8)]
    assert abs(np.mean(got) - expect) < 8.0, (got, expect)


def test_skewed_is_a_rounded_clipped_normal():
    step = wl.make_step(cfg(adapter_dist="skewed", skew_std=20.0, n_seqs=4000, n_dev_blocks=60000), with_acts=False,
                        fill_content=False)
    a = seq_adapters(step).astype(np.float64)
    assert abs(a.mean() - 500.0) < 1.5 and abs(a.std() - 20.0) < 1.0
    assert a.min() >= 0 and a.max() <= 999
    within = np.mean(np.abs(a - 500.0) <= 20.0)
    assert 0.64 < within < 0.73                             # one standard deviation holds about 68 %
    # a wide deviate is clipped into the id range
    step = wl.make_step(cfg(adapter_dist="skewed", skew_std=1000.0, n_adapters=16, n_seqs=300), with_acts=False,
                        fill_content=False)
    assert set(np.unique(seq_adapters(step))) <= set(range(16))


@pytest.mark.parametrize("dist", ["uniform", "zipf", "distinct", "skewed"])
def test_step_invariants(dist):
    step = wl.make_step(cfg(adapter_dist=dist, n_seqs=50), with_acts=False, fill_content=False)
    a = seq_adapters(step)
    assert np.array_equal(step.token_adapter, np.repeat(a, np.diff(step.cu_new)))
    present = np.unique(a)
    assert np.array_equal(np.flatnonzero(step.rank > 0), present)       # exactly the adapters in the batch are resident
    # every page table entry of a resident adapter is a distinct device block
    ids = np.asarray(step.lora_block_ids)
    assert len(np.unique(ids)) == len(ids)
    # same seed, same step
    again = wl.make_step(cfg(adapter_dist=dist, n_seqs=50), with_acts=False, fill_content=False)
    assert np.array_equal(again.token_adapter, step.token_adapter) and np.array_equal(again.lora_tables, step.lora_tables)


def test_shared_prefix_blocks_stay_within_one_adapter():
    """share_frac > 0 (paper section 4.1: queries of one LoRA with a common beginning hang below the same nodes;
    section 2.1: KV of different LoRAs is never shared): a physical block may sit in several tables, but only of
    sequences with the same adapter, only as a leading full prefix block at the same index, and never the block
    that a sequence's own new tokens are written to."""
    cfg = wl.LayerConfig("share", "f16", 512, 4, 4, 128, 3000, 900, 3, (8,), ("q",), 60, (0, 400), (1, 40),
                         share_frac=0.8, swap_in_frac=0.3, seed=5)
    st = wl.make_step(cfg)
    bt = cfg.block_tokens
    owners = {}
    for i in range(cfg.n_seqs):
        nb = -(-(int(st.prefix_len[i]) + int(st.new_len[i])) // bt)
        for k, b in enumerate(st.kv_tables[i, :nb]):
            owners.setdefault(int(b), []).append((i, k))
    shared = {b: o for b, o in owners.items() if len(o) > 1}
    assert len(shared) > 20
    for b, o in shared.items():
        assert len({int(st.seq_adapter[i]) for i, _ in o}) == 1          # one adapter
        assert len({k for _, k in o}) == 1                                # the same place in every table
        for i, k in o:
            assert (k + 1) * bt <= int(st.prefix_len[i])                  # a full prefix block, not the append target
    assert len(np.unique(st.content_ids)) == len(st.content_ids)          # every block has one content row
    assert not np.isin(st.fresh_block_ids, list(shared)).any()
    # the knob off: the same seed shares nothing
    st0 = wl.make_step(cfg.scaled(share_frac=0.0))
    ids, counts = np.unique(st0.kv_tables[st0.kv_tables >= 0], return_counts=True)
    assert counts.max() == 1
    assert np.array_equal(st0.prefix_len, st.prefix_len) and np.array_equal(st0.seq_adapter, st.seq_adapter)
