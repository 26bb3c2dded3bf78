"""The trace-driven run of the library's cache manager (paper_2505_03756_amd/cache_sim.py): a short
seeded trace per variant; checks what holds for any trace."""
import pytest

from paper_2505_03756_amd import cache_sim


@pytest.mark.parametrize("variant", list(cache_sim.VARIANTS))
def test_short_trace(variant):
    r = cache_sim.simulate(variant, duration_s=60.0, n_dev_blocks=2048, n_host_blocks=32768)
    assert r["queries"] > 100
    assert 0.0 <= r["kv_hit_ratio_hbm"] <= r["kv_hit_ratio"] <= 1.0
    assert r["hbm_usage_mean"] <= 0.97
    if variant != "no_dependencies":
        assert r["invalid_kv_share_mean"] == 0.0          # section 4.2: every resident KV cache is a valid one
    assert r["match_update_us_mean"] < 500.0              # the paper's budget (section 6.10)
    assert r["tick_ms_mean"] < 5.0


def test_same_seed_same_decisions():
    a = cache_sim.simulate("full", duration_s=30.0, n_dev_blocks=1024, n_host_blocks=16384)
    b = cache_sim.simulate("full", duration_s=30.0, n_dev_blocks=1024, n_host_blocks=16384)
    for k in ("queries", "kv_hit_ratio", "lora_cold_starts", "swapper_out_GB", "nodes_at_end"):
        assert a[k] == b[k]
