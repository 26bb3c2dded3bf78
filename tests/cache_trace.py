"""Seeded random traces that drive a cache manager (the oracle or the library binding) through the
same sequence of calls and record everything they return.  No arithmetic of the method lives here."""
import numpy as np


def run_trace(make, seed, n_steps=300, n_dev=96, n_host=160, bt=4, n_loras=6, vocab=3, max_len=40, **cfg):
    """`make(n_dev, n_host, bt, **cfg)` returns an object with add_lora / match / insert / release / tick /
    alloc_dev / free_dev / snapshot / usage.  Conversations draw tokens from a tiny vocabulary so that
    prefixes collide often; LoRA ids follow a skewed distribution."""
    rng = np.random.default_rng(seed)
    m = make(n_dev, n_host, bt, **cfg)
    log = []
    now = 0.0
    for a in range(n_loras):
        ids = m.add_lora(100 + a, 1 + a % 3, 1 if a % 2 else 0, now)
        log.append(("add_lora", a, ids))
    weights = 1.0 / np.arange(1, n_loras + 1)
    weights /= weights.sum()
    running = []
    for step in range(n_steps):
        now += float(rng.integers(1, 50)) / 10.0
        op = rng.random()
        if op < 0.55:
            a = int(rng.choice(n_loras, p=weights))
            n_tok = int(rng.integers(1, max_len))
            tokens = [int(t) for t in rng.integers(0, vocab, size=n_tok)]
            q, lora_blocks, kv_blocks, swap_in = m.match(100 + a, tokens, now)
            log.append(("match", a, tuple(tokens), lora_blocks, tuple(kv_blocks), tuple(swap_in)))
            if lora_blocks is None:
                m.release(q)
                continue
            n_new = n_tok // bt - len(kv_blocks)
            new = m.alloc_dev(n_new) if n_new > 0 else []
            if new is None:
                new = []
            back = m.insert(q, tokens, new, now) if new else []
            if back:
                m.free_dev(back)
            log.append(("insert", tuple(new), tuple(back)))
            running.append(q)
        elif op < 0.80 and running:
            q = running.pop(int(rng.integers(0, len(running))))
            m.release(q)
            log.append(("release", q))
        else:
            out, inn, dropped = m.tick(now, int(rng.integers(1, 9)))
            log.append(("tick", tuple(out), tuple(inn), tuple(dropped), round(m.usage(), 9)))
    for q in running:
        m.release(q)
    out, inn, dropped = m.tick(now + 1.0, 4)
    log.append(("tick", tuple(out), tuple(inn), tuple(dropped), round(m.usage(), 9)))
    log.append(("snapshot", tuple(m.snapshot())))
    return m, log
