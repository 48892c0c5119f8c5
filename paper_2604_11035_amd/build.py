"""Builds the HIP library of the ISD hot path for gfx950 (in-tree, next to this file)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libidlm_isd.so"
SOURCES = ["isd_attention.hip", "isd_attention_shared.hip", "isd_accept.hip", "isd_accept_general.hip", "isd_accept_filtered.hip", "isd_loop.hip", "isd_lora.hip", "idlm_misc.hip"]
# Packed fp32 VALU forms are switched off for all device code (they have produced wrong
# results on the target machines); the host pass does not know the feature and says so.
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]
# Per-file additions.  The attention kernel's score accumulators are read by vector arithmetic right after
# the matrix instructions that produce them: with the results of matrix instructions in ordinary vector
# registers there are no copies out of accumulation registers in its tile loop.
FILE_FLAGS = {"isd_attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
              "isd_attention_shared.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}
NOISE = "is not a recognized feature for this target"


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed (%d): %s" % (res.returncode, " ".join(cmd[-3:])))
    return err


def build(verbose: bool = False, extra=()) -> Path:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    work = Path(tempfile.mkdtemp(prefix="idlm_build_"))
    try:
        objs = [work / (Path(s).stem + ".o") for s in SOURCES]
        cmds = [[hipcc, *FLAGS, *FILE_FLAGS.get(s, []), *extra, "-c", "-o", str(o), str(CSRC / s)]
                for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
            errs = list(pool.map(_run, cmds))
        tmp = LIB.with_suffix(".so.tmp%d" % os.getpid())
        errs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp)] + [str(o) for o in objs]))
        if verbose:
            for e in errs:
                if e.strip():
                    print(e)
        os.replace(tmp, LIB)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
