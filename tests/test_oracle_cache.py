"""Pins of the cache-manager / cache-swapper oracle against what the paper and the mathematics fix
(sections 4.1-4.3, 5.1-5.3, Eq. 3-6): closed forms, invariants, brute force on small trees."""
import itertools
import math

import numpy as np
import pytest

from oracle.cache_oracle import HBM, HOST, KV, LORA, CacheOracle
from tests.cache_trace import run_trace


class OracleDriver(CacheOracle):
    def alloc_dev(self, n):
        return self.free[HBM].alloc(n)

    def free_dev(self, ids):
        self.free[HBM].free(ids)


def make(n_dev, n_host, bt, **cfg):
    return OracleDriver(n_dev, n_host, block_tokens=bt, block_bytes=4096, **cfg)


def fresh(n_loras, visits, **cfg):
    c = make(256, 256, 4, **cfg)
    for a in range(n_loras):
        c.add_lora(a, 1, HBM, 0.0)
    for a, v in enumerate(visits):
        for _ in range(v):
            q, *_ = c.match(a, [], 0.0)
            c.release(q)
    return c


# ------------------------------------------------------------------ Eq. 3
@pytest.mark.parametrize("n,bs", [(1, 1), (4, 1), (4, 8), (10, 3), (50, 32)])
def test_low_lora_uniform_closed_form(n, bs):
    c = fresh(n, [3] * n)
    assert c.low_lora(bs) == pytest.approx(n * (1 - (1 - 1 / n) ** bs), rel=1e-12)


def test_low_lora_limits():
    c = fresh(5, [1, 2, 3, 4, 5])
    assert c.low_lora(1) == pytest.approx(1.0, rel=1e-12)          # one query uses exactly one LoRA
    assert c.low_lora(10 ** 6) == pytest.approx(5.0, rel=1e-9)     # a huge batch uses all of them
    c = fresh(3, [7, 0, 0])
    assert c.low_lora(4) == pytest.approx(1.0, rel=1e-12)          # only one LoRA is ever used
    # monotone in the batch size, and equal to the expectation estimated by brute-force enumeration
    c = fresh(3, [1, 2, 5])
    p = [1 / 8, 2 / 8, 5 / 8]
    for bs in (1, 2, 3):
        exp = 0.0
        for combo in itertools.product(range(3), repeat=bs):
            exp += len(set(combo)) * math.prod(p[i] for i in combo)
        assert c.low_lora(bs) == pytest.approx(exp, rel=1e-12)


# ------------------------------------------------------------------ Eq. 4
def test_lora_eval_reward():
    c = fresh(1, [1])
    assert c.lora_eval(3.0, 6) == 1.0
    assert c.lora_eval(3.0, 3) == 1.0
    assert c.lora_eval(3.0, 2) == 1.5
    assert c.lora_eval(3.0, 0) == 3.0           # nothing loaded: taken as one loaded


# ------------------------------------------------------------------ Eq. 5, Eq. 6
def test_retain_eval_closed_forms():
    c = make(64, 64, 4, pcie_bytes_per_s=4096.0, time_scale_s=2.0)
    c.add_lora(0, 3, HBM, 0.0)
    c.add_lora(1, 1, HBM, 0.0)
    for a, v in ((0, 3), (1, 1)):
        for _ in range(v):
            q, *_ = c.match(a, [], 10.0)
            c.release(q)
    n0, n1 = c.root.children[0], c.root.children[1]
    # t = 0: sigmoid = 1/2; cost = size / bandwidth = 3 blocks * 4096 B / 4096 B/s = 3 s; prob = 3/4
    assert c.retain_eval(n0, 10.0) == pytest.approx(3.0 * 0.75 * 0.5, rel=1e-12)
    assert c.retain_eval(n1, 10.0) == pytest.approx(1.0 * 0.25 * 0.5, rel=1e-12)
    # decay: t = (now - last use) / time scale
    assert c.retain_eval(n0, 14.0) == pytest.approx(3.0 * 0.75 * (1 - 1 / (1 + math.exp(-2.0))), rel=1e-12)
    vals = [c.retain_eval(n0, 10.0 + d) for d in range(0, 40, 4)]
    assert all(x > y > 0 for x, y in zip(vals, vals[1:]))
    # Eq. 6: product with the reward (LoRA nodes only)
    assert c.eval(n0, 10.0, 4.0, 2) == pytest.approx(2.0 * c.retain_eval(n0, 10.0), rel=1e-12)
    assert c.eval(n0, 10.0, 1.0, 2) == pytest.approx(c.retain_eval(n0, 10.0), rel=1e-12)


def test_reward_applies_to_lora_nodes_only_and_can_be_switched_off():
    for no_reward in (False, True):
        c = make(64, 64, 4, no_lora_reward=no_reward)
        c.add_lora(0, 1, HBM, 0.0)
        q, _, kv, _ = c.match(0, [1, 2, 3, 4], 0.0)
        c.insert(q, [1, 2, 3, 4], c.alloc_dev(1), 0.0)
        c.release(q)
        lora = c.root.children[0]
        kvn = next(iter(lora.children.values()))
        assert c.eval(kvn, 1.0, 5.0, 1) == c.retain_eval(kvn, 1.0)
        want = c.retain_eval(lora, 1.0) * (1.0 if no_reward else 5.0)
        assert c.eval(lora, 1.0, 5.0, 1) == pytest.approx(want, rel=1e-12)


# ------------------------------------------------------------------ tree: match / insert (sections 4.1, 4.2)
def test_match_is_longest_stored_prefix_in_whole_blocks():
    rng = np.random.default_rng(5)
    bt = 4
    c = make(4096, 64, bt)
    stored = {0: [], 1: []}
    for a in stored:
        c.add_lora(a, 1, HBM, 0.0)
    for it in range(200):
        a = int(rng.integers(0, 2))
        toks = [int(t) for t in rng.integers(0, 2, size=int(rng.integers(0, 30)))]
        q, lb, kv, si = c.match(a, toks, float(it))
        # brute force: longest common whole-block prefix with anything stored under the same LoRA
        best = 0
        for s in stored[a]:
            k = 0
            while (k + 1) * bt <= min(len(s), len(toks)) and s[k * bt:(k + 1) * bt] == toks[k * bt:(k + 1) * bt]:
                k += 1
            best = max(best, k)
        assert len(kv) == best and si == []
        n_new = len(toks) // bt - best
        back = c.insert(q, toks, c.alloc_dev(n_new), float(it))
        assert back == []
        c.release(q)
        stored[a].append(toks[:len(toks) // bt * bt])
    # the same tokens under another LoRA share nothing (section 2.1: KV caches are per LoRA)
    c.add_lora(2, 1, HBM, 0.0)
    q, lb, kv, si = c.match(2, stored[0][0] if stored[0] else [0] * 8, 999.0)
    assert kv == []


def test_insert_then_match_returns_the_same_blocks_and_updates_statistics():
    c = make(64, 64, 4)
    c.add_lora(9, 2, HBM, 0.0)
    toks = list(range(11))
    q, lb, kv, _ = c.match(9, toks, 1.0)
    blocks = c.alloc_dev(2)
    assert c.insert(q, toks, blocks, 1.0) == []
    c.release(q)
    q2, lb2, kv2, si2 = c.match(9, toks, 5.0)
    assert kv2 == blocks and lb2 == lb and si2 == []
    snap = {s[0]: s for s in c.snapshot()}
    assert [snap[i][5] for i in (1, 2, 3)] == [2, 2, 2]              # visit counts
    assert [snap[i][6] for i in (1, 2, 3)] == [5.0, 5.0, 5.0]        # last use
    assert [snap[i][7] for i in (1, 2, 3)] == [1, 1, 1]              # pinned by the running query
    # a second query inserting the same continuation gets its block back
    q3, _, kv3, _ = c.match(9, toks[:4], 6.0)
    extra = c.alloc_dev(1)
    assert c.insert(q3, toks[:8], extra, 6.0) == extra


# ------------------------------------------------------------------ swapper (sections 4.2, 5.3)
def build_chain(c, lora, n_blocks, now, tokens_base=0):
    toks = [tokens_base + i for i in range(n_blocks * c.bt)]
    q, *_ = c.match(lora, toks, now)
    c.insert(q, toks, c.alloc_dev(n_blocks), now)
    c.release(q)


def test_nothing_moves_between_the_thresholds():
    c = make(100, 100, 4)
    c.add_lora(0, 10, HBM, 0.0)
    build_chain(c, 0, 70, 1.0)                       # usage 0.80
    assert c.tick(2.0, 4) == ([], [], [])


def test_swap_out_takes_leaves_in_increasing_eval_until_usage_is_at_most_upper():
    c = make(100, 100, 4, upper=0.90, lower=0.10)
    c.add_lora(0, 2, HBM, 0.0)
    c.add_lora(1, 2, HBM, 0.0)
    build_chain(c, 0, 50, 1.0)
    build_chain(c, 1, 43, 50.0, tokens_base=1000)    # 97 blocks in use
    before = {s[0]: s for s in c.snapshot()}
    out, inn, dropped = c.tick(60.0, 4)
    assert inn == [] and dropped == [] and len(out) == 7
    assert c.usage() <= 0.90 < (100 - c.free[HBM].num_free() + 1) / 100
    # victims: each one was a leaf among the HBM nodes at the time it was taken (children always go first)
    dev_to_node = {before[i][4][0]: i for i in before if before[i][1] == KV}
    victims = [dev_to_node[d] for d, _ in out]
    chain0 = sorted(i for i in before if before[i][1] == KV and before[i][6] == 1.0)
    # the older chain has the lower Eval everywhere (same size and frequency, larger t): its tail goes, leaf first
    assert victims == chain0[::-1][:7]
    assert c.invalid_kv_blocks() == 0


def test_first_victim_is_the_arg_min_of_eval_over_all_leaves_brute_force():
    rng = np.random.default_rng(11)
    for trial in range(20):
        c = make(64, 64, 2, upper=0.5, lower=0.1, time_scale_s=float(rng.integers(1, 20)))
        for a in range(3):
            c.add_lora(a, int(rng.integers(1, 4)), HBM, 0.0)
        now = 0.0
        for _ in range(12):
            now += float(rng.integers(1, 10))
            a = int(rng.integers(0, 3))
            toks = [int(t) for t in rng.integers(0, 2, size=int(rng.integers(2, 9)))]
            q, lb, kv, _ = c.match(a, toks, now)
            n_new = len(toks) // 2 - len(kv)
            ids = c.alloc_dev(n_new) or []
            c.insert(q, toks, ids, now)
            c.release(q)
        if c.usage() <= 0.5:
            continue
        now += 3.0
        low, nl = c.low_lora(4), c.now_lora()
        leaves = [n for n in c.nodes.values() if n is not c.root and n.tier == HBM
                  and not any(ch.tier == HBM for ch in n.children.values())]
        best = min(leaves, key=lambda n: (c.eval(n, now, low, nl), n.id))
        want = best.blocks[0]
        out, _, _ = c.tick(now, 4)
        assert out[0][0] == want


def test_swap_in_takes_host_roots_in_decreasing_eval_and_stops_at_lower():
    c = make(100, 100, 4, upper=0.95, lower=0.50)
    c.add_lora(0, 2, HOST, 0.0)
    c.add_lora(1, 2, HOST, 0.0)
    for _ in range(3):                                # LoRA 1 is used three times as often
        q, *_ = c.match(1, [], 1.0)
        c.release(q)
    q, *_ = c.match(0, [], 1.0)
    c.release(q)
    # matching brought both into HBM; push both out again with a very low upper threshold
    c.upper, c.lower = 0.0, -1.0
    out, _, _ = c.tick(2.0, 4)
    assert len(out) == 4 and c.usage() == 0.0
    c.upper, c.lower = 0.95, 0.02
    out, inn, _ = c.tick(3.0, 4)
    assert out == [] and len(inn) == 2                # one LoRA (2 blocks) reaches the lower threshold
    assert c.root.children[1].tier == HBM and c.root.children[0].tier == HOST


def test_lru_variant_evicts_the_least_recently_used_leaf():
    c = make(40, 40, 4, upper=0.5, lower=0.0, use_lru=True)
    c.add_lora(0, 1, HBM, 0.0)
    c.add_lora(1, 1, HBM, 0.0)
    build_chain(c, 0, 10, 5.0)
    build_chain(c, 1, 10, 2.0, tokens_base=500)       # older
    out, _, _ = c.tick(9.0, 4)
    oldest_chain = [n for n in c.nodes.values() if n.kind == KV and n.last_use == 2.0]
    assert len(out) == 2 and all(n.tier == HOST for n in sorted(oldest_chain, key=lambda n: -n.id)[:2])


def test_pinned_nodes_stay():
    c = make(20, 20, 4, upper=0.1, lower=0.0)
    c.add_lora(0, 1, HBM, 0.0)
    toks = list(range(16))
    q, *_ = c.match(0, toks, 1.0)
    c.insert(q, toks, c.alloc_dev(4), 1.0)
    out, _, _ = c.tick(2.0, 4)
    assert out == []                                  # everything is in use
    c.release(q)
    out, _, _ = c.tick(3.0, 4)
    assert len(out) == 3 and c.usage() <= 0.1 + 1e-12         # 5 of 20 blocks held; 2 may stay


def test_dependencies_keep_every_resident_kv_valid_and_ignoring_them_does_not():
    for seed in range(6):
        c, _ = run_trace(make, seed, n_steps=300)
        assert c.invalid_kv_blocks() == 0
        for n in c.nodes.values():
            if n is not c.root and n.tier == HBM and n.parent is not c.root:
                assert n.parent.tier == HBM
    bad = 0
    for seed in range(6):
        c, _ = run_trace(make, seed, n_steps=300, ignore_dependencies=True)
        bad += c.invalid_kv_blocks()
    assert bad > 0


def test_blocks_are_conserved_and_thresholds_hold_on_random_traces():
    for seed in range(8):
        c, log = run_trace(make, 100 + seed, n_steps=300)
        for tier in (HBM, HOST):
            held = sum(len(n.blocks) for n in c.nodes.values() if n is not c.root and n.tier == tier)
            assert held + c.free[tier].num_free() == c.free[tier].n
        for rec in log:
            if rec[0] == "tick":
                _, out, inn, dropped, usage = rec
                assert not (out and inn)
                if inn:
                    assert usage <= c.upper + 1e-9
