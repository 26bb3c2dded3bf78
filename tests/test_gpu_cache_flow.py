"""The cache manager driving the pool on the GPU: its match / tick lists are executed by
flp_pool_swap_in / flp_pool_swap_out, fresh KV is appended by flp_kv_append into the blocks it
handed over, and after any number of manager-decided round trips between the tiers every cached
block holds the bytes it was given and attention over the re-matched prefix agrees with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2505_03756_amd import flcache, flpool
from tests.helpers import TOL, close

pytestmark = pytest.mark.gpu

BT, N_KV, D, N_H = 16, 2, 128, 4
BE = 2 * BT * N_KV * D


def test_manager_driven_swaps_preserve_every_block_and_attention_matches():
    rng = np.random.default_rng(2025)
    n_dev, n_host = 48, 256
    dev = torch.zeros(n_dev, BE, dtype=torch.int16, device="cuda")
    host = torch.zeros(n_host, BE, dtype=torch.int16).pin_memory()
    pool = flpool.Pool("f16", N_KV, D, n_dev, n_host, block_tokens=BT, dev=dev, host=host)
    cache = flcache.Cache(pool, block_tokens=BT, upper=0.60, lower=0.30, time_scale_s=5.0)
    st = torch.cuda.Stream()
    content = {}                                   # node id of a block's owner is not visible: key by (lora, token prefix)

    # adapters arrive on the host tier with recognisable pages
    lora_pages = {}
    for a in range(3):
        ids = cache.add_lora(a, 2, 1, 0.0)
        for k, b in enumerate(ids):
            page = torch.from_numpy(rng.integers(-2000, 2000, size=BE, dtype=np.int16))
            host[int(b)] = page
            lora_pages[(a, k)] = page.clone()

    convs = []
    now = 0.0
    for it in range(60):
        now += 1.0
        a = int(rng.integers(0, 3))
        if convs and rng.random() < 0.6:
            base = convs[int(rng.integers(0, len(convs)))]
            a, toks = base[0], list(base[1]) + [int(t) for t in rng.integers(0, 50, size=int(rng.integers(8, 40)))]
        else:
            toks = [int(t) for t in rng.integers(0, 50, size=int(rng.integers(20, 90)))]
        q, lb, kv, sh, sd = cache.match(a, toks, now)
        if lb is None:
            cache.release(q)
            continue
        pool.swap_in(sh, sd, stream=st)
        st.synchronize()
        # the LoRA's pages and every matched KV block hold what they were given
        for k, b in enumerate(lb):
            assert torch.equal(dev[int(b)].cpu(), lora_pages[(a, k)])
        for j, b in enumerate(kv):
            assert torch.equal(dev[int(b)].cpu(), content[(a, tuple(toks[:(j + 1) * BT]))]), (it, j)
        # fresh KV for the rest of the tokens, appended through a table of matched + new blocks
        P = len(kv) * BT
        N = len(toks) - P
        n_new_blocks = (len(toks) + BT - 1) // BT - len(kv)
        try:
            new = pool.alloc(n_new_blocks, 0)
        except flpool.FlpError:
            cache.release(q)
            (od, oh), (ih, idv), dr = cache.tick(now, 4)
            pool.swap_out(od, oh, stream=st)
            pool.swap_in(ih, idv, stream=st)
            st.synchronize()
            continue
        table = torch.tensor([list(kv) + list(new)], dtype=torch.int32, device="cuda")
        k_new = torch.from_numpy(rng.standard_normal((N, N_KV, D)).astype(np.float16).view(np.int16)).cuda()
        v_new = torch.from_numpy(rng.standard_normal((N, N_KV, D)).astype(np.float16).view(np.int16)).cuda()
        cu, pl = np.array([0, N], np.int32), np.array([P], np.int32)
        pool.kv_append(k_new, v_new, cu, pl, table, stream=st)
        # attention of the new tokens over the reused prefix + their own KV, against the oracle on a host image
        qv = torch.from_numpy(rng.standard_normal((N, N_H, D)).astype(np.float16).view(np.int16)).cuda()
        out = torch.zeros_like(qv)
        pool.paged_prefix_attention(qv, out, cu, pl, table, N_H, stream=st)
        st.synchronize()
        img = dev.cpu().numpy().view(np.uint16)
        want = oracle.paged_attention(img, "f16", BT, N_KV, D, N_H, cu, pl, table.cpu().numpy(),
                                      qv.cpu().numpy().view(np.uint16))
        got = out.cpu().numpy().view(np.float16).astype(np.float64)
        ok, worst, nbad = close(got.reshape(want.shape), want, *TOL["f16"])
        assert ok, (it, worst, nbad)
        # full new blocks become nodes; the partial last block stays with the caller and is freed
        n_full = len(toks) // BT - len(kv)
        back = cache.insert(q, toks, new[:n_full], now)
        for j in range(n_full):
            key = (a, tuple(toks[:(len(kv) + j + 1) * BT]))
            if key not in content:
                content[key] = dev[int(new[j])].cpu().clone()
        pool.free(np.concatenate([back, new[n_full:]]).astype(np.int32), 0)
        cache.release(q)
        convs.append((a, toks))
        # the swapper's decisions, executed in the order it gives them
        (od, oh), (ih, idv), dr = cache.tick(now, 4)
        pool.swap_out(od, oh, stream=st)
        pool.swap_in(ih, idv, stream=st)
        st.synchronize()
        s = cache.stats()
        assert s["invalid_kv_blocks"] == 0
    s = cache.stats()
    assert s["n_kv_nodes"] > 30 and s["host_blocks_held"] > 0, s     # the run did move blocks between the tiers
