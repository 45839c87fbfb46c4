"""Builds libdrcgnn.so (the C-ABI library of hand-written HIP kernels) in-tree for gfx950."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdrcgnn.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC",
    "--offload-arch=gfx950",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = True) -> str:
    """Compile every HIP translation unit (one hipcc process each, side by side) and link the shared library.
    Always recompiles; the objects live in a temporary directory and are not kept."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    with tempfile.TemporaryDirectory(prefix="drcgnn_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, *inc, "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True)
            return obj
        with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as pool:
            objs = list(pool.map(compile_one, sources()))
        link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


def kernel_resources(source: str) -> dict:
    """{mangled kernel name: {"VGPRs", "ScratchSize", "Occupancy", "LDS Size", ...}} of one translation unit of csrc/, as
    the compiler reports them (-Rpass-analysis=kernel-resource-usage; device code only, nothing is written).  A kernel
    whose ScratchSize is not 0 keeps something in scratch memory: every access to it is a vector-memory operation whose
    wait also waits for the loads in flight."""
    import re
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only",
           "-Rpass-analysis=kernel-resource-usage", "-c", os.path.join(CSRC, source), "-o", os.devnull]
    err = subprocess.run(cmd, check=True, capture_output=True, text=True).stderr
    out, cur = {}, None
    for line in err.splitlines():
        m = re.search(r"remark:\s+(Function Name|[A-Za-z ]+(?:\[[^\]]*\])?):\s+(\S+)", line)
        if not m:
            continue
        key, val = m.group(1).strip(), m.group(2)
        if key == "Function Name":
            cur = out.setdefault(val, {})
        elif cur is not None:
            key = re.sub(r"\s*\[.*\]", "", key)
            cur[key] = int(val) if val.lstrip("-").isdigit() else val
    return out


if __name__ == "__main__":
    build()
    print(LIB)
    sys.exit(0)
