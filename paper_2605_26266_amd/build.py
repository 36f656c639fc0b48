"""Compile the HIP sources of the library for gfx950 into paper_2605_26266_amd/libkvq.so.

`python -m paper_2605_26266_amd.build` builds the library; with `--microbench` it also builds the stand-alone
issue-rate microbenchmarks (paper_2605_26266_amd/kvq_microbench, a measuring tool that is not part of the library)."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

try:                                     # `python -m paper_2605_26266_amd.build` and a plain script run both work
    from . import mfma_hazard_check
except ImportError:                      # pragma: no cover
    import mfma_hazard_check

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkvq.so")
MICROBENCH = os.path.join(HERE, "kvq_microbench")   # stand-alone issue-rate microbenchmarks

# Packed-FP32 code generation is switched off for every device translation unit.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-constant-logical-operand",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# Sources with MFMAs written as inline assembly: the wait states around them are placed in the source, and every
# build checks the device assembly for them (mfma_hazard_check) before the object is accepted.
HAZARD_CHECKED = {"kvq_attention_mfma.hip"}
SOURCES = {
    "kvq_api.hip": [],
    # the quantizer's rounding decisions follow a fixed sequence of IEEE operations: no contraction
    "kvq_quantize.hip": ["-ffp-contract=off"],
    "kvq_attention_simt.hip": [],
    "kvq_attention_mfma.hip": [],
    "kvq_attention_mfma_group.hip": [],
}


def _compile(item):
    src, extra = item
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    temps = os.path.join(OBJ, "asm_" + src.replace(".hip", ""))
    if src in HAZARD_CHECKED:            # keep the intermediate files of this compile, among them the device assembly
        shutil.rmtree(temps, ignore_errors=True)
        os.makedirs(temps)
        obj_tmp = os.path.join(temps, os.path.basename(obj))
        cmd = ["hipcc", *COMMON, *extra, "-save-temps=obj", "-c", os.path.join(CSRC, src), "-o", obj_tmp]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    if src in HAZARD_CHECKED:
        listings = glob.glob(os.path.join(temps, "*-hip-amdgcn-amd-amdhsa-gfx950.s"))
        if len(listings) != 1:
            raise RuntimeError("no device assembly found for %s in %s" % (src, temps))
        count, problems = mfma_hazard_check.check_file(listings[0])
        if problems or count == 0:
            raise RuntimeError("wait-state check failed for %s (%d MFMAs):\n%s" % (src, count, "\n".join(problems[:20])))
        os.replace(obj_tmp, obj)
        shutil.rmtree(temps, ignore_errors=True)
    return obj


def build_microbench(verbose: bool = False) -> str:
    cmd = ["hipcc", *COMMON, os.path.join(CSRC, "kvq_microbench.hip"), "-o", MICROBENCH]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for kvq_microbench.hip:\n" + r.stderr)
    if verbose:
        print("built", MICROBENCH)
    return MICROBENCH


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as pool:
        objs = list(pool.map(_compile, SOURCES.items()))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
    if "--microbench" in sys.argv[1:]:
        build_microbench(verbose=True)
