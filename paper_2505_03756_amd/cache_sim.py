"""Trace-driven run of the cache manager / cache swapper (include/flcache.h) on a synthetic multi-LoRA
chat workload: host logic only, block ids only (no block contents are touched, no GPU needed).

Stands in for the paper's chatbot scenario (section 6.2: multi-turn conversations, tens of LoRAs with
skewed popularity, about two queries per second); none of the paper's traces is reproduced.  Recipe,
all seeded: conversations arrive as a Poisson process; each picks a LoRA by Zipf(1) over a seeded
permutation, starts from that LoRA's shared 128-token system prompt and has a geometric number of
turns; a turn appends a prompt and a response of uniform random lengths (fresh random token ids) to
the conversation's history and is sent after an exponential think time; a query holds its nodes while
it runs (a time proportional to its new tokens); the swapper ticks every 100 ms (section 5.3).

Reported per variant (the paper's ablations: section 6.6 no dependencies, 6.7 LRU, 6.8 no LoRA reward):
KV hit ratio in blocks, LoRA cold starts, bytes swapped in on the critical path of a query (what Eq. 5
calls the cold-start cost), bytes moved by the swapper, the share of HBM-resident KV blocks that cannot
be matched because an ancestor is not resident ("invalid KV caches", sections 2.3 / 6.6), and the
manager's own overheads against the paper's budget (section 6.10: < 0.5 ms per match and update, <= 5 ms
per swapping decision).
"""
import heapq
import time

import numpy as np

from . import flcache, flpool

VARIANTS = {
    "full": {},
    "no_dependencies": {"ignore_dependencies": True},
    "lru": {"use_lru": True},
    "no_lora_reward": {"no_lora_reward": True},
}


def _host_pool(n_dev, n_host, bt):
    # ids only: the two regions are zero pages that nothing touches
    be = 2 * bt * 64
    dev = np.zeros(n_dev * be + 256, np.uint16)
    host = np.zeros(n_host * be + 256, np.uint16)
    al = lambda a: (a.ctypes.data + 255) & ~255
    p = flpool.Pool("f16", 1, 64, n_dev, n_host, block_tokens=bt, dev=al(dev), host=al(host))
    p._bufs = (dev, host)
    return p


def simulate(variant="full", seed=20250601, duration_s=600.0, rate_per_s=2.0, n_loras=50, lora_blocks=8,
             n_dev_blocks=16384, n_host_blocks=131072, bt=16, block_bytes=262144, pcie_bytes_per_s=57e9,
             mean_turns=4.0, think_s=30.0):
    rng = np.random.default_rng(seed)
    pool = _host_pool(n_dev_blocks, n_host_blocks, bt)
    cache = flcache.Cache(pool, block_tokens=bt, upper=0.95, lower=0.70, pcie_bytes_per_s=pcie_bytes_per_s,
                          time_scale_s=60.0, **VARIANTS[variant])
    perm = rng.permutation(n_loras)
    w = 1.0 / np.arange(1, n_loras + 1)
    w /= w.sum()
    system = [rng.integers(0, 32000, size=128).astype(np.int32) for _ in range(n_loras)]
    for a in range(n_loras):
        cache.add_lora(a, lora_blocks, 1, 0.0)                     # every adapter starts on the host tier

    events = []                                                    # (time, seq, kind, payload)
    seq = 0

    def push(t, kind, payload):
        nonlocal seq
        heapq.heappush(events, (t, seq, kind, payload))
        seq += 1

    t = 0.0
    while t < duration_s:
        t += float(rng.exponential(1.0 / rate_per_s))
        a = int(perm[int(rng.choice(n_loras, p=w))])
        push(t, "turn", {"lora": a, "history": system[a], "turns_left": int(rng.geometric(1.0 / mean_turns))})
    tick_t = 0.1
    while tick_t < duration_s:
        push(tick_t, "tick", None)
        tick_t += 0.1

    m = dict(queries=0, blocks_needed=0, blocks_hit=0, blocks_hit_hbm=0, lora_cold=0, cold_blocks=0, swapper_out=0, swapper_in=0,
             dropped=0, waits=0, alloc_fail=0, invalid_samples=[], usage_samples=[])
    t_match, t_tick = [], []
    recent = []                                                    # query start times of the last 5 s (batch size of Eq. 3)
    while events:
        now, _, kind, ev = heapq.heappop(events)
        if kind == "tick":
            recent = [x for x in recent if x > now - 5.0]
            t0 = time.perf_counter()
            (od, oh), (ih, idv), dr = cache.tick(now, max(1, len(recent)), cap=65536)
            t_tick.append(time.perf_counter() - t0)
            m["swapper_out"] += len(od)
            m["swapper_in"] += len(ih)
            m["dropped"] += len(dr)
            if int(round(now * 10)) % 50 == 0:
                s = cache.stats()
                kv_hbm = s["hbm_blocks_held"] - s["n_lora_hbm"] * lora_blocks
                m["invalid_samples"].append(s["invalid_kv_blocks"] / kv_hbm if kv_hbm > 0 else 0.0)
                m["usage_samples"].append(s["usage"])
        elif kind == "turn":
            if now >= duration_s:                                  # the run is over: later turns are not sent
                continue
            prompt = rng.integers(0, 32000, size=int(rng.integers(64, 513))).astype(np.int32)
            toks = np.concatenate([ev["history"], prompt])
            t0 = time.perf_counter()
            q, lb, kv, sh, sd = cache.match(ev["lora"], toks, now)
            if lb is None:                                         # not even the LoRA fits: retry after the next ticks
                cache.release(q)
                m["waits"] += 1
                if now < duration_s:
                    push(now + 0.2, "turn", ev)
                continue
            response = rng.integers(0, 32000, size=int(rng.integers(64, 257))).astype(np.int32)
            full = np.concatenate([toks, response])
            n_new = len(full) // bt - len(kv)
            try:
                new = pool.alloc(n_new, 0)
            except flpool.FlpError:
                cache.release(q)
                m["alloc_fail"] += 1
                if now < duration_s:
                    push(now + 0.2, "turn", ev)
                continue
            back = cache.insert(q, full, new, now)
            if len(back):
                pool.free(back, 0)
            t_match.append(time.perf_counter() - t0)
            m["queries"] += 1
            m["blocks_needed"] += len(toks) // bt
            m["blocks_hit"] += len(kv)
            lora_cold = len(sd) >= lora_blocks and set(int(x) for x in sd[:lora_blocks]) == set(int(x) for x in lb)
            m["lora_cold"] += int(lora_cold)
            m["cold_blocks"] += len(sh)
            m["blocks_hit_hbm"] += len(kv) - (len(sh) - (lora_blocks if lora_cold else 0))
            recent.append(now)
            push(now + 0.5 + len(prompt) / 4000.0 + len(response) / 100.0, "done", q)
            if ev["turns_left"] > 1:
                push(now + 0.5 + len(response) / 100.0 + float(rng.exponential(think_s)), "turn",
                     {"lora": ev["lora"], "history": full, "turns_left": ev["turns_left"] - 1})
        else:
            cache.release(ev)
    s = cache.stats()
    bw = pcie_bytes_per_s
    return {
        "variant": variant,
        "queries": m["queries"],
        "kv_hit_ratio": round(m["blocks_hit"] / max(1, m["blocks_needed"]), 4),
        "kv_hit_ratio_hbm": round(m["blocks_hit_hbm"] / max(1, m["blocks_needed"]), 4),
        "lora_cold_starts": m["lora_cold"],
        "cold_start_ms_per_query": round(1e3 * m["cold_blocks"] * block_bytes / bw / max(1, m["queries"]), 3),
        "swapper_out_GB": round(m["swapper_out"] * block_bytes / 1e9, 3),
        "swapper_in_GB": round(m["swapper_in"] * block_bytes / 1e9, 3),
        "forgotten_nodes": m["dropped"],
        "waits": m["waits"] + m["alloc_fail"],
        "invalid_kv_share_mean": round(float(np.mean(m["invalid_samples"])) if m["invalid_samples"] else 0.0, 4),
        "hbm_usage_mean": round(float(np.mean(m["usage_samples"])) if m["usage_samples"] else 0.0, 4),
        "nodes_at_end": s["n_nodes"],
        "match_update_us_mean": round(1e6 * float(np.mean(t_match)), 1),
        "match_update_us_p99": round(1e6 * float(np.percentile(t_match, 99)), 1),
        "tick_ms_mean": round(1e3 * float(np.mean(t_tick)), 4),
        "tick_ms_max": round(1e3 * float(np.max(t_tick)), 3),
    }


if __name__ == "__main__":
    import json
    import sys
    names = sys.argv[1:] or list(VARIANTS)
    for name in names:
        print(json.dumps(simulate(name)), flush=True)
