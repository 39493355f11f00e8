"""Builds libxsv.so (the HIP library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libxsv.so")
ISSUE_BENCH = os.path.join(_HERE, "issue_bench")   # standalone microbenchmark program (csrc/issue_bench.hip)
BUILD_DIR = os.path.join(_HERE, "_build")

# packed-fp32 instructions are switched off for every kernel (target feature): some of their forms have
# given wrong results on this hardware, and hipcc would otherwise form them from ordinary float code
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# bit-exact kernels: one rounding per operation, like the definition
SOURCES = {
    "xsv_api.hip": [],
    # plain v_max3 in the softmax (inputs are finite); MFMA results in VGPRs so the softmax reads them
    # without accumulator-register moves
    "attend.hip": ["-fno-honor-nans", "-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "score_select.hip": ["-ffp-contract=off"],
    "requant.hip": ["-ffp-contract=off"],
    "peaks.hip": [],
}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    os.makedirs(BUILD_DIR, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(item):
        src, extra = item
        obj = os.path.join(BUILD_DIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
        if verbose and r.stderr:
            print(r.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES.items()))
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stderr}")
    r = subprocess.run([hipcc, *[f for f in COMMON if f != "-fPIC"], "-Wno-unused-result", "-mllvm", "-amdgpu-mfma-vgpr-form=1",
                        os.path.join(CSRC, "issue_bench.hip"), "-o", ISSUE_BENCH], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"issue_bench failed to build:\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
