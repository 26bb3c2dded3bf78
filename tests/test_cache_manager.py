"""The library's cache manager / cache swapper (include/flcache.h) against the oracle: the same seeded
traces of add / match / insert / release / tick must produce the same block lists, in the same order,
and the same tree.  Host logic only: runs without a GPU on a pool over caller-owned host memory."""
import ctypes as C
import os
import re
import time

import numpy as np
import pytest

from oracle.cache_oracle import HBM, CacheOracle
from paper_2505_03756_amd import flcache, flpool
from tests.cache_trace import run_trace

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BLOCK_BYTES = 2 * 4 * 1 * 64 * 2          # bt = 4, one kv head of 64 channels, 16 bit


def host_pool(n_dev, n_host, bt):
    be = 2 * bt * 1 * 64
    dev = np.zeros(n_dev * be + 256, np.uint16)
    host = np.zeros(n_host * be + 256, np.uint16)
    al = lambda a: (a.ctypes.data + 255) & ~255
    p = flpool.Pool("f16", 1, 64, n_dev, n_host, block_tokens=bt, dev=al(dev), host=al(host))
    p._bufs = (dev, host)
    return p


class LibDriver:
    """The binding behind the interface of tests/cache_trace.py."""

    def __init__(self, n_dev, n_host, bt, **cfg):
        self.pool = host_pool(n_dev, n_host, bt)
        self.c = flcache.Cache(self.pool, block_tokens=bt, **cfg)
        self.upper = cfg.get("upper", 0.95)

    def add_lora(self, lora_id, n_blocks, tier, now):
        try:
            return [int(i) for i in self.c.add_lora(lora_id, n_blocks, tier, now)]
        except flpool.FlpError as e:
            assert e.code == flpool.FLP_ENOSPC
            return None

    def match(self, lora_id, tokens, now):
        q, lb, kv, sh, sd = self.c.match(lora_id, tokens, now)
        return (q, None if lb is None else [int(i) for i in lb], [int(i) for i in kv],
                list(zip([int(i) for i in sh], [int(i) for i in sd])))

    def insert(self, q, tokens, new, now):
        return [int(i) for i in self.c.insert(q, tokens, new, now)]

    def release(self, q):
        self.c.release(q)

    def tick(self, now, bs):
        (od, oh), (ih, idv), dr = self.c.tick(now, bs)
        return (list(zip([int(i) for i in od], [int(i) for i in oh])),
                list(zip([int(i) for i in ih], [int(i) for i in idv])), [int(i) for i in dr])

    def alloc_dev(self, n):
        try:
            return [int(i) for i in self.pool.alloc(n, 0)]
        except flpool.FlpError:
            return None

    def free_dev(self, ids):
        self.pool.free(np.asarray(ids, np.int32), 0)

    def usage(self):
        return self.c.stats()["usage"]

    def snapshot(self):
        # (id, kind, parent, tier, blocks..., visits, last use, pins) with the oracle's field order
        return [(i, k, p, t, fb, nb, v, lu, pins) for i, k, p, t, fb, nb, v, lu, pins in self.c.snapshot()]


class OracleDriver(CacheOracle):
    def alloc_dev(self, n):
        return self.free[HBM].alloc(n)

    def free_dev(self, ids):
        self.free[HBM].free(ids)

    def snapshot(self):
        return [(i, k, p, t, b[0] if b else -1, len(b), v, lu, pins) for i, k, p, t, b, v, lu, pins in super().snapshot()]


def make_oracle(n_dev, n_host, bt, **cfg):
    return OracleDriver(n_dev, n_host, block_tokens=bt, block_bytes=BLOCK_BYTES, **cfg)


VARIANTS = [dict(), dict(use_lru=True), dict(ignore_dependencies=True), dict(no_lora_reward=True),
            dict(upper=0.6, lower=0.3, time_scale_s=3.0), dict(pcie_bytes_per_s=1e6, time_scale_s=0.5)]


def test_library_exports_every_declared_symbol():
    lib = flpool.load()
    header = open(os.path.join(ROOT, "include", "flcache.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(flc_[a-z_0-9]+)\s*\(", header))
    assert declared == set(flcache.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert C.sizeof(flcache.Config) == 16 + 4 * 8
    assert C.sizeof(flcache.Stats) == 10 * 8
    assert C.sizeof(flcache.NodeInfo) == 8 * 4 + 16


@pytest.mark.parametrize("variant", range(len(VARIANTS)))
@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_traces_agree_with_the_oracle_block_for_block(seed, variant):
    cfg = VARIANTS[variant]
    _, want = run_trace(make_oracle, 1000 * variant + seed, **cfg)
    _, got = run_trace(LibDriver, 1000 * variant + seed, **cfg)
    assert len(want) == len(got)
    for k, (w, g) in enumerate(zip(want, got)):
        assert w == g, "record %d: oracle %r, library %r" % (k, w, g)


def test_host_tier_full_forgets_victims_like_the_oracle():
    for seed in range(4):
        _, want = run_trace(make_oracle, 50 + seed, n_dev=64, n_host=12, n_steps=400)
        _, got = run_trace(LibDriver, 50 + seed, n_dev=64, n_host=12, n_steps=400)
        assert want == got
        assert any(r[0] == "tick" and r[3] for r in want), "the trace was meant to drop nodes"


def test_cost_model_values_agree_with_the_oracle():
    o, _ = run_trace(make_oracle, 7, n_steps=200)
    l, _ = run_trace(LibDriver, 7, n_steps=200)
    for bs in (1, 4, 32):
        assert l.c.low_lora(bs) == o.low_lora(bs)
    now = 5000.0
    low, nl = o.low_lora(4), o.now_lora()
    for n in o.nodes.values():
        if n is not o.root:
            assert l.c.eval(n.id, now, 4) == o.eval(n, now, low, nl)
    s = l.c.stats()
    assert s["invalid_kv_blocks"] == o.invalid_kv_blocks() == 0
    assert s["n_nodes"] == len(o.nodes) - 1 and s["n_lora_hbm"] == o.now_lora() and s["n_queries"] == o.n_queries


def test_errors_leave_the_cache_unchanged():
    d = LibDriver(32, 32, 4)
    c = d.c
    c.add_lora(1, 2, 0, 0.0)
    with pytest.raises(flpool.FlpError) as e:
        c.add_lora(1, 2, 0, 0.0)
    assert e.value.code == flpool.FLP_EDUP
    with pytest.raises(flpool.FlpError) as e:
        c.add_lora(2, 100, 0, 0.0)
    assert e.value.code == flpool.FLP_ENOSPC
    with pytest.raises(flpool.FlpError) as e:
        c.match(99, [1, 2, 3, 4], 0.0)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        c.release(12345)
    assert e.value.code == flpool.FLP_EINVAL
    q, lb, kv, sh, sd = c.match(1, list(range(8)), 1.0)
    with pytest.raises(flpool.FlpError) as e:
        c.insert(q, list(range(4)), [5, 6], 1.0)            # tokens do not cover two new blocks
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        c.insert(q, list(range(8)), [5, 600], 1.0)          # id outside the pool
    assert e.value.code == flpool.FLP_ERANGE
    assert c.stats()["n_nodes"] == 1 and d.pool.num_free(0) == 30


def test_overheads_stay_within_the_papers_budget():
    """Section 6.10 of the paper: matching and updating below 0.5 ms, the swapping decision within 5 ms.
    Tree of 100 LoRAs and 60 000 KV blocks (a 15 GiB pool of 256 KiB blocks), queries of 1024 tokens."""
    bt = 16
    n_dev, n_host = 60000, 60000
    pool = host_pool(n_dev, n_host, bt)        # (zero pages that are never touched: only ids are used)
    c = flcache.Cache(pool, block_tokens=bt, upper=0.95, lower=0.70)
    rng = np.random.default_rng(0)
    for a in range(100):
        c.add_lora(a, 4, 0, 0.0)
    convs = []
    now = 0.0
    t_match = []
    while pool.num_free(0) > 0.03 * n_dev:
        now += 0.01
        a = int(rng.integers(0, 100))
        if convs and rng.random() < 0.5:
            base = convs[int(rng.integers(0, len(convs)))]
            a, toks = base[0], np.concatenate([base[1], rng.integers(0, 32000, size=256)]).astype(np.int32)
        else:
            toks = rng.integers(0, 32000, size=1024).astype(np.int32)
        t0 = time.perf_counter()
        q, lb, kv, sh, sd = c.match(a, toks, now)
        n_new = len(toks) // bt - len(kv)
        new = pool.alloc(n_new, 0)
        back = c.insert(q, toks, new, now)
        c.release(q)
        t_match.append(time.perf_counter() - t0)
        assert len(back) == 0
        convs.append((a, toks))
    t0 = time.perf_counter()
    (od, oh), (ih, idv), dr = c.tick(now + 1.0, 16, cap=65536)
    t_tick = time.perf_counter() - t0
    s = c.stats()
    assert len(od) > 0 and s["usage"] <= 0.95 + 1e-9 and s["invalid_kv_blocks"] == 0
    mean_match = sum(t_match) / len(t_match)
    print("nodes %d: match+insert+release mean %.3f ms, max %.3f ms; tick (%d moves) %.3f ms" %
          (s["n_nodes"], mean_match * 1e3, max(t_match) * 1e3, len(od), t_tick * 1e3))
    assert mean_match < 0.5e-3
    assert t_tick < 5e-3


def _build_host_driver(tmp_path, source, sanitize):
    """g++ build of a tests/*.cpp driver with the library's host sources (pool.cpp, cache_manager.cpp)."""
    import shutil
    import subprocess
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    csrc = os.path.join(ROOT, "paper_2505_03756_amd", "csrc")
    exe = str(tmp_path / os.path.splitext(source)[0])
    cmd = [gxx, "-std=c++17", "-O1", "-g"] + sanitize + [
        "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-I/opt/rocm/include",
        os.path.join(ROOT, "tests", source), os.path.join(csrc, "pool.cpp"), os.path.join(csrc, "cache_manager.cpp"),
        "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-pthread", "-o", exe]
    b = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert b.returncode == 0, b.stderr[-3000:]
    return exe


def test_four_threads_on_one_cache_under_thread_sanitizer(tmp_path):
    """tests/cache_threads.cpp: four threads match, insert, release and allocate on one cache and one pool while
    one of them runs the monitor intervals, built with ThreadSanitizer: no report (the internal locks of
    include/flcache.h and include/flpool.h hold), accounting intact at the end."""
    import subprocess
    exe = _build_host_driver(tmp_path, "cache_threads.cpp", ["-fsanitize=thread"])
    r = subprocess.run([exe, "3000"], capture_output=True, text=True, timeout=300)
    if "unexpected memory mapping" in r.stderr:
        pytest.skip("ThreadSanitizer cannot run in this address-space layout")
    assert r.returncode == 0 and "ThreadSanitizer" not in r.stderr, (r.stdout + r.stderr)[-3000:]
    assert "accounting intact" in r.stdout


def test_random_walk_over_the_host_abi_under_sanitizers(tmp_path):
    """tests/cache_fuzz.cpp (a seeded random walk over every entry point of include/flcache.h, legal and illegal
    arguments, all four policy variants, roomy and tight tiers) built from the library's own host sources with
    AddressSanitizer and UndefinedBehaviorSanitizer: no report, block accounting intact after every call, blocks
    back in the pool after flc_destroy."""
    import subprocess
    exe = _build_host_driver(tmp_path, "cache_fuzz.cpp", ["-fsanitize=address,undefined",
                                                          "-fno-sanitize-recover=undefined", "-static-libasan"])
    # where a GPU is present the pool's one look at its host base starts the HIP / HSA runtimes, which keep a few
    # allocations until the process ends: not this library's, so the leak check leaves those two out
    supp = tmp_path / "lsan.supp"
    supp.write_text("leak:libhsa-runtime64\nleak:libamdhip64\n")
    env = dict(os.environ, LSAN_OPTIONS="suppressions=%s:print_suppressions=0" % supp)
    r = subprocess.run([exe, "3000"], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "accounting held after every call" in r.stdout


def test_closing_the_pool_first_closes_its_caches():
    """flc_destroy returns the nodes' blocks to the pool, so the pool must outlive the cache: the binding closes
    the caches of a pool before the pool itself, whatever order the caller (or the garbage collector) picks."""
    pool = host_pool(16, 16, 4)
    c = flcache.Cache(pool, 4)
    c.add_lora(1, 3, 0, 0.0)
    assert pool.num_free(0) == 13
    pool.close()
    assert c._h is None and pool._h is None
    c.close()                                   # a second time: nothing left to do
    pool2 = host_pool(16, 16, 4)
    c2 = flcache.Cache(pool2, 4)
    c2.add_lora(1, 3, 0, 0.0)
    c2.close()
    assert pool2.num_free(0) == 16              # the LoRA's blocks came back
    pool2.close()
