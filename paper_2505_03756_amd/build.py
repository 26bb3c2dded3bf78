"""Build libflpool.so (HIP, gfx950) in-tree with hipcc.  No GPU needed to compile."""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflpool.so")
SOURCES = ["pool.cpp", "dispatch.cpp", "cache_manager.cpp", "sched.cpp", "swap.hip", "attention.hip", "attention_mfma.hip", "lora.hip", "lora_mfma.hip", "gemm.hip", "layer.hip", "static_scratch.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics"]
# Private (scratch) memory a kernel may use, bytes per lane.  A few dozen spilled registers in an epilogue are fine
# (the large-batch GEMM holds 256 accumulators and spills up to 36 registers after its loop); an accumulator array
# that the compiler could not keep in registers (a loop it did not unroll, an index it could not resolve) is a
# kilobyte and makes the kernel many times slower without failing any test, so the build stops.
MAX_SCRATCH_BYTES = 256
RESOURCES = {}      # kernel name -> dict(vgprs, agprs, scratch, occupancy), filled by build()


def _resources(stderr):
    """Parse hipcc's kernel-resource-usage remarks: {mangled kernel name: figures}."""
    out, cur = {}, None
    for line in stderr.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        if cur is None:
            continue
        for key, pat in (("vgprs", r" VGPRs: (\d+)"), ("agprs", r"AGPRs: (\d+)"),
                         ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"), ("occupancy", r"Occupancy \[waves/SIMD\]: (\d+)"),
                         ("lds", r"LDS Size \[bytes/block\]: (\d+)")):
            m = re.search(pat, line)
            if m:
                cur[key] = int(m.group(1))
    return out


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "is not a recognized feature" not in l and "-Rpass-analysis=kernel-resource-usage" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    res = _resources(r.stderr)
    bad = {k: v["scratch"] for k, v in res.items() if v.get("scratch", 0) > MAX_SCRATCH_BYTES}
    if bad:
        raise RuntimeError("%s: kernels with more than %d bytes of private memory per lane (an array that left the "
                           "registers): %s" % (src, MAX_SCRATCH_BYTES, bad))
    return obj, res


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        done = list(ex.map(_compile, srcs))
    objs = [o for o, _ in done]
    RESOURCES.clear()
    for _, res in done:
        RESOURCES.update(res)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
