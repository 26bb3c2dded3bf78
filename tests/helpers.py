"""Test-side helpers: the harness plumbing lives in the package; only the comparison rule and the
tolerances are defined here."""
import numpy as np

from paper_2505_03756_amd.harness import (GpuPool, GpuStep, SparseGpuPool, build_pools, compact_step,  # noqa: F401
                                          poison_value, resident_pool, to_dev, to_np)


def close(got, ref, rtol, atol):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    tol = atol + rtol * np.abs(ref)
    bad = ~(err <= tol)
    return not bad.any(), float(err.max() if err.size else 0.0), int(bad.sum())


TOL = {"f32": (1e-4, 1e-5), "f16": (2e-3, 1e-2), "bf16": (2e-3, 1e-2)}
