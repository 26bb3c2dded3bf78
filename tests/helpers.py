"""Shared test plumbing: turn a synthetic Step into host-side pool arrays."""
import numpy as np

from paper_2505_03756_amd import workload as wl


def poison_value(dtype):
    return np.float32(np.nan) if dtype == "f32" else (0x7E00 if dtype == "f16" else 0x7FC0)


def build_pools(step, poison_rest=False):
    """Device-tier and host-tier pool images ([n_blocks, block_elems] storage arrays) at
    the start of the step: blocks on the swap-in list have their content on the host tier
    and poison on the device tier."""
    cfg = step.cfg
    sd = wl.storage_dtype(cfg.dtype)
    dev = np.zeros((cfg.n_dev_blocks, cfg.block_elems), dtype=sd)
    host = np.zeros((cfg.n_host_blocks, cfg.block_elems), dtype=sd)
    if poison_rest:
        dev[:] = poison_value(cfg.dtype)
    dev[step.content_ids] = step.content
    if len(step.swap_in_dev):
        host[step.swap_in_host] = dev[step.swap_in_dev]
        dev[step.swap_in_dev] = poison_value(cfg.dtype)
    return dev, host


def resident_pool(step):
    """Device pool image with every needed block resident (swap already done)."""
    cfg = step.cfg
    dev = np.zeros((cfg.n_dev_blocks, cfg.block_elems), dtype=wl.storage_dtype(cfg.dtype))
    dev[step.content_ids] = step.content
    return dev


def close(got, ref, rtol, atol):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    tol = atol + rtol * np.abs(ref)
    bad = ~(err <= tol)
    return not bad.any(), float(err.max() if err.size else 0.0), int(bad.sum())


TOL = {"f32": (1e-4, 1e-5), "f16": (2e-3, 1e-2), "bf16": (2e-3, 1e-2)}
