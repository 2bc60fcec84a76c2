"""Compile the HIP sources into libattn.so (the attention library) and libattn_probes.so (measurement
probes, a library of their own) next to this file (hipcc, gfx950 only)."""
from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libattn.so")
PROBES_LIB = os.path.join(HERE, "libattn_probes.so")
# VGPR_FORM: kernels that run one wave per SIMD may use the accumulation registers (AGPRs) next to
# the 256 vector registers; by default the compiler then gives every MFMA an AGPR accumulator,
# and where vector instructions read those accumulators every tile (softmax on the scores, dS from
# dP) it shuttles hundreds of registers per tile between the two files.  With VGPR-form MFMAs the
# AGPRs only hold spilled loop invariants.  Applied to the forward kernels (only head dim 256 runs
# one wave per SIMD: +7 %, no other forward kernel changes) and to the kernels attn_bwd_all.inc
# lists for the second pass over attn_bwd.hip.  The dK/dV kernels of d = 192 / 256 keep dK and dV,
# which no vector instruction touches inside the loop, in AGPRs: they want the default.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=true"]
# (source, object, additional flags)
SOURCES = [("attn_api.hip", "attn_api.o", []),
           ("attn_fwd.hip", "attn_fwd.o", VGPR_FORM),
           ("attn_fwd_q64.hip", "attn_fwd_q64.o", []),
           ("attn_bwd.hip", "attn_bwd.o", []),
           ("attn_bwd.hip", "attn_bwd_vgpr_form.o", ["-DATTN_BWD_VGPR_FORM_PART=1", *VGPR_FORM]),
           ("attn_bwd_dq_q64.hip", "attn_bwd_dq_q64.o", []),
           ("attn_varlen.hip", "attn_varlen.o", []),
           ("exp2_emulated.hip", "exp2_emulated.o", [])]
PROBE_SOURCES = [("probes.hip", "probes.o", [])]
# packed-fp32 instruction selection is switched off on purpose (device passes only; the
# host pass prints a harmless "not a recognized feature" note).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument"]

def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        keep = [ln for ln in (res.stdout + res.stderr).splitlines() if "packed-fp32-ops" not in ln]
        if keep:
            print("\n".join(keep))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libattn.so: " + " ".join(cmd[-3:]))


def build_library(verbose: bool = False) -> str:
    """One hipcc process per source file (the attention files dominate: every kernel body is
    instantiated per head dim, mask, mode and element type), then one link step per library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="libattn_build_")
    try:
        every = SOURCES + PROBE_SOURCES
        jobs = [[hipcc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", os.path.join(tmp, obj)]
                for src, obj, extra in every]
        with ThreadPoolExecutor(max_workers=min(len(jobs), os.cpu_count() or 1, 8)) as pool:
            list(pool.map(lambda c: _run(c, verbose), jobs))
        for lib, sources in ((LIB, SOURCES), (PROBES_LIB, PROBE_SOURCES)):
            objs = [os.path.join(tmp, obj) for _, obj, _ in sources]
            _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib + ".tmp", *objs], verbose)
            os.replace(lib + ".tmp", lib)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
