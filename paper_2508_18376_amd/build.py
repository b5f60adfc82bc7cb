"""Builds libdsmoe.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdsmoe.so")
SOURCES = ["api.hip", "route_plan.hip", "pack.hip", "gemm_generic.hip", "gemm_mfma.hip", "importance.hip", "thresholds.hip", "router.hip", "transform.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(HERE, "..", "include", "dsmoe.h")]
    return any(os.path.getmtime(d) > t for d in deps)


# The MFMA GEMM kernels use the whole register file (256 accumulators + 256 others per lane).  A
# spill to scratch memory inside a main loop makes the loop wait for every outstanding load each
# time round, and a small edit of the kernel is enough to cause one: the build refuses it.
NO_SCRATCH = {"gemm_mfma.hip": ("gemm1_mfma_kernel", "gemm2_mfma_kernel")}


def _scratch_users(remarks: str, kernels) -> list:
    """Kernels among `kernels` whose 'ScratchSize [bytes/lane]' remark is not 0."""
    bad, name = [], None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name is not None:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size != 0 and any(k in name for k in kernels):
                bad.append("%s: %d bytes/lane" % (name, size))
    return bad


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link the shared library.  Returns its path."""
    if not force and not _needs_build():
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def cc(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if src in NO_SCRATCH:
            cmd.append("-Rpass-analysis=kernel-resource-usage")
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if src in NO_SCRATCH:
            bad = _scratch_users(r.stderr, NO_SCRATCH[src])
            if bad:
                raise RuntimeError("%s: kernels that must not spill use scratch memory: %s" % (src, "; ".join(bad)))
        elif verbose and r.stderr.strip():
            sys.stderr.write(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(cc, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
