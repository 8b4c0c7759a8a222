"""Build the HIP libraries (gfx950) in-tree with hipcc.

libcfdecode.so is the product.  libcfdecode_trace.so is the same code with the per-phase time stamps compiled in
(-DCF_STAMPS=1; cf_debug_export what = 2): a profiling aid, about 0.25 us slower per step, loaded only when the
environment variable CFDECODE_LIB points to it.
"""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libcfdecode.so")
TRACE_LIB = os.path.join(PKG, "libcfdecode_trace.so")
SOURCES = ["cf_api.hip", "cf_fused_kernel.hip", "cf_team.hip", "cf_mla.hip", "cf_mla_heads.hip", "cf_splithead.hip", "cf_ffn.hip"]
# -ffp-contract=on: multiply-adds are fused where one source expression holds both, never across statements at the
# optimiser's choice, so every instantiation of a template rounds alike (the multi-layer kernel and the single-block
# kernel then give the same bits); measured cost against the default "fast": none to 0.2 us per step.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=on",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link both shared libraries.  Always recompiles."""
    obj_dir = os.path.join(PKG, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()
    variants = (("", ["-DCF_STAMPS=0"], LIB), ("_trace", ["-DCF_STAMPS=1"], TRACE_LIB))
    # (object suffix, extra definitions, source): the fused kernel is compiled a second time with -DCF_LAYER=1
    units = [("", [], src) for src in SOURCES] + [("_layer", ["-DCF_LAYER=1"], "cf_fused_kernel.hip")]

    def compile_one(job):
        suffix, defs, src = job
        obj = os.path.join(obj_dir, src.replace(".hip", suffix + ".o"))
        cmd = [hipcc, *HIPCC_FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr))
        if verbose:
            print(res.stderr)
        return obj

    jobs = [(usuf + suffix, defs + udefs, src) for (suffix, defs, _) in variants for (usuf, udefs, src) in units]
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(compile_one, jobs))
    for k, (_, _, lib) in enumerate(variants):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs[k * len(units):(k + 1) * len(units)]]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
