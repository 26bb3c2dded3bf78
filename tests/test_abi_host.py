"""Host-side checks of the C-ABI library that need no GPU: it loads, exports what the header
declares, and its free lists / argument validation agree with the oracle's allocator model."""
import ctypes as C
import os
import re
import subprocess
import sys

import numpy as np
import pytest

import oracle
from oracle import OracleError
from paper_2505_03756_amd import flpool

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _host_pool(n_dev=64, n_host=16, dtype="f16", n_kv=2, d=64):
    be = 2 * 16 * n_kv * d
    sd = np.float32 if dtype == "f32" else np.uint16
    # over-allocate so that a 256-byte aligned base exists inside each buffer
    dev = np.zeros(n_dev * be + 256, sd)
    host = np.zeros(n_host * be + 256, sd)

    def aligned(a):
        return (a.ctypes.data + 255) & ~255
    p = flpool.Pool(dtype, n_kv, d, n_dev, n_host, dev=aligned(dev), host=aligned(host))
    p._bufs = (dev, host)
    return p


def test_library_exports_every_declared_symbol():
    lib = flpool.load()
    header = open(os.path.join(ROOT, "include", "flpool.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(flp_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations parsed"
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(flpool.EXPORTS)
    assert b"flpool" in lib.flp_version()


def test_layer_header_symbols_and_structs():
    from paper_2505_03756_amd import fllayer
    lib = flpool.load()
    header = open(os.path.join(ROOT, "include", "fllayer.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(fll_[a-z_0-9]+)\s*\(", header))
    assert declared == set(fllayer.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert C.sizeof(fllayer.LayerConfig) == 24
    assert C.sizeof(fllayer.LayerWeights) == 9 * 8
    assert C.sizeof(fllayer.LoraPlace) == 32
    assert C.sizeof(fllayer.LayerBatch) == 24 + 8 * 8 + 7 * 32
    # argument checks that need no GPU
    assert lib.fll_rmsnorm(1, None, None, None, 4, 64, C.c_float(1e-5), None) == flpool.FLP_EINVAL
    assert lib.fll_rope(1, None, None, None, 4, 2, 2, 128, C.c_float(1e4), None) == flpool.FLP_EINVAL
    buf = np.zeros(64, np.float32)
    fllayer._lib()
    assert lib.fll_rope(0, buf.ctypes.data, None, buf.ctypes.data, 1, 1, 1, 96, C.c_float(1e4), None) == flpool.FLP_ENOTSUP
    assert lib.fll_silu_mul(1, buf.ctypes.data, 7, buf.ctypes.data, 7, buf.ctypes.data, 7, 1, 7, None) == flpool.FLP_ENOTSUP
    assert lib.fll_rmsnorm(1, buf.ctypes.data, buf.ctypes.data, buf.ctypes.data, 0, 64, C.c_float(1e-5), None) == flpool.FLP_OK


def test_struct_sizes_match_header_layout():
    # natural alignment of the C structs in include/flpool.h
    assert C.sizeof(flpool.PoolConfig) == 48
    assert C.sizeof(flpool.AttnBatch) == 16 + 7 * 8
    assert C.sizeof(flpool.LoraProj) == 16 + 6 * 8
    assert C.sizeof(flpool.LoraBatch) == 32 + 5 * 8 + 4 * C.sizeof(flpool.LoraProj)


def test_alloc_free_match_oracle_model_bit_exactly():
    rng = np.random.default_rng(100)
    for tier, n in ((0, 64), (1, 16)):
        pool = _host_pool()
        model = oracle.Allocator(n)
        held = []
        for _ in range(1500):
            if rng.random() < 0.55:
                k = int(rng.integers(0, 7))
                try:
                    want = model.alloc(k)
                except OracleError as e:
                    with pytest.raises(flpool.FlpError) as g:
                        pool.alloc(k, tier)
                    assert g.value.code == e.code == flpool.FLP_ENOSPC
                    continue
                got = pool.alloc(k, tier)
                assert np.array_equal(got, want)
                held += list(got)
            elif held:
                k = int(rng.integers(1, min(len(held), 5) + 1))
                pick = [held.pop(int(rng.integers(0, len(held)))) for _ in range(k)]
                model.free(pick)
                pool.free(pick, tier)
            assert pool.num_free(tier) == model.num_free
        pool.close()


def test_shuffled_free_list_recipe():
    # "random block permutation": allocate everything, free in a seeded shuffled order,
    # then allocations come back in the reverse of that order - identical in model and library
    rng = np.random.default_rng(101)
    pool = _host_pool()
    model = oracle.Allocator(64)
    order = rng.permutation(64).astype(np.int32)
    for a in (pool, model):
        a.alloc(64)
        a.free(order)
    got, want = pool.alloc(20), model.alloc(20)
    assert np.array_equal(got, want) and np.array_equal(got, order[::-1][:20])


def test_alloc_free_error_codes_leave_state_unchanged():
    pool = _host_pool(n_dev=8)
    ids = pool.alloc(6)
    with pytest.raises(flpool.FlpError) as e:
        pool.alloc(3)
    assert e.value.code == flpool.FLP_ENOSPC and pool.num_free() == 2
    for bad, code in (([8], flpool.FLP_ERANGE), ([-1], flpool.FLP_ERANGE), ([7], flpool.FLP_EDUP),
                      ([ids[0], ids[1], ids[0]], flpool.FLP_EDUP)):
        with pytest.raises(flpool.FlpError) as e:
            pool.free(bad)
        assert e.value.code == code
        assert pool.num_free() == 2
    with pytest.raises(flpool.FlpError) as e:
        pool.alloc(-1)
    assert e.value.code == flpool.FLP_EINVAL
    pool.free(ids)
    assert pool.num_free() == 8
    assert "flp_pool" in str(e.value)


def test_swap_list_validation_without_touching_memory():
    pool = _host_pool(n_dev=8, n_host=4)
    for fn, a, b, code in (
            (pool.swap_in, [0, 1], [3, 3], flpool.FLP_EDUP),       # duplicate destination (device side)
            (pool.swap_in, [4], [0], flpool.FLP_ERANGE),           # host id out of range
            (pool.swap_in, [0], [8], flpool.FLP_ERANGE),
            (pool.swap_out, [0, 1], [2, 2], flpool.FLP_EDUP),      # duplicate destination (host side)
            (pool.swap_out, [8], [0], flpool.FLP_ERANGE),
            (pool.swap_out, [0], [-1], flpool.FLP_ERANGE)):
        with pytest.raises(flpool.FlpError) as e:
            fn(a, b, stream=0)
        assert e.value.code == code
    pool.swap_in([], [], stream=0)          # empty list: success, nothing enqueued
    pool.swap_out([], [], stream=0)
    with pytest.raises(flpool.FlpError) as e:
        pool.swap_in([0, 1], [2], stream=0)
    assert e.value.code == flpool.FLP_EINVAL


def test_attention_argument_checks():
    pool = _host_pool(n_kv=2, d=64)
    fake = 0x1000                      # never dereferenced: the checks fail first
    tables = np.zeros((2, 3), np.int32)
    with pytest.raises(flpool.FlpError) as e:    # 40 + 9 positions > 3 blocks * 16
        pool.paged_prefix_attention(fake, fake, [0, 4, 13], [10, 40], tables.ctypes.data, 4, max_blocks=3, stream=0)
    assert e.value.code == flpool.FLP_ERANGE
    with pytest.raises(flpool.FlpError) as e:    # 3 query heads over 2 kv heads
        pool.paged_prefix_attention(fake, fake, [0, 4], [10], tables.ctypes.data, 3, max_blocks=3, stream=0)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:    # cu_new decreasing
        pool.paged_prefix_attention(fake, fake, [0, 4, 2], [1, 1], tables.ctypes.data, 4, max_blocks=3, stream=0)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:    # misaligned q
        pool.paged_prefix_attention(fake + 2, fake, [0, 4], [1], tables.ctypes.data, 4, max_blocks=3, stream=0)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:    # append without v_new
        pool.kv_append(fake, None, [0, 4], [1], tables.ctypes.data, max_blocks=3, stream=0)
    assert e.value.code == flpool.FLP_EINVAL
    odd = flpool.Pool("f16", 2, 80, 4, 0, dev=pool.base(0), host=None)
    with pytest.raises(flpool.FlpError) as e:
        odd.paged_prefix_attention(fake, fake, [0, 1], [1], tables.ctypes.data, 2, max_blocks=3, stream=0)
    assert e.value.code == flpool.FLP_ENOTSUP


def test_lora_argument_checks():
    pool = _host_pool(n_kv=2, d=64)            # block = 4096 elements
    fake = 0x1000
    proj = dict(y=fake, d_out=64, a_tab_off=fake, a_row_base=fake, b_tab_off=fake, b_row_base=fake)
    kw = dict(x=fake, token_adapter=fake, rank=fake, scale=fake, block_tables=fake, n_tokens=4, d_in=64,
              n_adapters=2, max_rank=8, stream=0)
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[proj], **{**kw, "max_rank": 65})
    assert e.value.code == flpool.FLP_ERANGE
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[proj], **{**kw, "d_in": 8192})     # a page-row longer than a block
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[dict(proj, d_out=60)], **kw)       # not a multiple of 8 elements
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[dict(proj, y=None)], **kw)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[proj] * 5, **kw)
    assert e.value.code == flpool.FLP_EINVAL
    pool.lora_apply_paged(projs=[proj], **{**kw, "n_tokens": 0})        # empty batch: success
    # the limits the header states next to the declarations: 1..64 for max_rank, 2048 adapters for both calls
    for bad_rank in (0, -1, 65):
        with pytest.raises(flpool.FlpError) as e:
            pool.lora_apply_paged(projs=[proj], **{**kw, "max_rank": bad_rank})
        assert e.value.code == flpool.FLP_ERANGE
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[proj], **{**kw, "n_adapters": 2049})
    assert e.value.code == flpool.FLP_ERANGE and "2048" in str(e.value)


def test_static_lora_entry_point_refuses_oversized_batches_on_the_host():
    """The entry point that allocates nothing checks the batch against its fixed 64 MiB before it touches the GPU."""
    pool = _host_pool(n_kv=8, d=128)           # block = 32768 elements
    fake = 0x1000
    proj = dict(y=fake, d_out=16384, w_base=fake, a_tab_off=fake, a_row_base=fake, b_tab_off=fake, b_row_base=fake)
    kw = dict(x=fake, token_adapter=fake, rank=fake, scale=fake, block_tables=fake, n_tokens=1000, d_in=16384,
              n_adapters=2, max_rank=8, stream=0)
    assert flpool.static_scratch_bytes() == 64 << 20
    with pytest.raises(flpool.FlpError) as e:
        pool.lora_apply_paged(projs=[proj], static=True, **kw)
    assert e.value.code == flpool.FLP_ENOSPC and "fixed buffer" in str(e.value)


def test_header_and_code_state_the_same_adapter_limit():
    hdr = open(os.path.join(ROOT, "include", "flpool.h")).read()
    assert "4096" not in hdr.split("flp_lora_segment")[0].split("FLP_MAX_PROJ")[-1]
    assert hdr.count("n_adapters <= 2048") >= 2
    lib = flpool.load()
    import ctypes
    fake = ctypes.c_void_p(0x1000)
    pool = _host_pool(n_kv=2, d=64)
    rc = lib.flp_lora_segment(pool._h, 4, fake, 2049, fake, fake, fake, fake, None)
    assert rc == flpool.FLP_ERANGE


def test_pool_create_rejects_bad_geometry():
    with pytest.raises(flpool.FlpError) as e:
        flpool.Pool("f16", 0, 64, 4, 0, dev=0x1000)
    assert e.value.code == flpool.FLP_EINVAL
    with pytest.raises(flpool.FlpError) as e:
        flpool.Pool("f16", 2, 64, 4, 0, dev=0x1010)       # not 256-byte aligned
    assert e.value.code == flpool.FLP_EINVAL


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_build_rejects_kernels_that_left_the_registers():
    """The build parses the compiler's per-kernel resource report and stops when a kernel uses more than a few
    spilled registers' worth of private memory (an accumulator array in scratch memory is many times slower and
    fails no parity test): the parser on a report with one good and one bad kernel."""
    from paper_2505_03756_amd import build as b
    report = """
x.hip:1:1: remark: Function Name: good_kernel [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     VGPRs: 64 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     ScratchSize [bytes/lane]: 56 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     Occupancy [waves/SIMD]: 8 [-Rpass-analysis=kernel-resource-usage]
x.hip:1:1: remark:     LDS Size [bytes/block]: 1024 [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark: Function Name: bad_kernel [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark:     VGPRs: 103 [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark:     AGPRs: 256 [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark:     ScratchSize [bytes/lane]: 1088 [-Rpass-analysis=kernel-resource-usage]
x.hip:9:1: remark:     Occupancy [waves/SIMD]: 1 [-Rpass-analysis=kernel-resource-usage]
"""
    res = b._resources(report)
    assert res["good_kernel"] == {"vgprs": 64, "agprs": 0, "scratch": 56, "occupancy": 8, "lds": 1024}
    assert res["bad_kernel"]["scratch"] == 1088 and res["bad_kernel"]["agprs"] == 256
    assert [k for k, v in res.items() if v["scratch"] > b.MAX_SCRATCH_BYTES] == ["bad_kernel"]


def test_binding_fails_loudly_without_the_library(tmp_path):
    """The product path has no fallback: with no built library the binding raises at load (in a fresh process, with
    the library path pointed at a file that does not exist) instead of computing anything some other way."""
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2505_03756_amd import flpool\n"
            "flpool.LIB_PATH = %r\n"
            "try:\n"
            "    flpool.Pool('f16', 1, 64, 4, 4)\n"
            "except flpool.FlpError as e:\n"
            "    print('raised:', e); sys.exit(7)\n"
            "sys.exit(0)\n") % (ROOT, str(tmp_path / "libflpool.so"))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert r.returncode == 7, r.stdout + r.stderr
    assert "not built" in r.stdout
