"""Build libgptstage.so in-tree with hipcc for gfx950.

    python -m paper_2507_19845_amd.build

Compiles every .hip file under csrc/ (in parallel) and links them into
paper_2507_19845_amd/libgptstage.so.  No GPU is needed to build.
"""
from __future__ import annotations

import hashlib
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgptstage.so")
STAMP = LIB + ".srchash"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off on purpose for every device pass
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=fast",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
FLAGS += os.environ.get("GPTS_HIPCC_FLAGS", "").split()   # e.g. -DGPTS_BIG_WAVES=8 for experiments


# gemm_mi16_kernel keeps its 256 accumulators in AGPRs a0..a255 by hand, across separate inline
# assembly statements; the compiler only knows them as clobbered.  That is safe as long as the
# register allocator never needs an AGPR of its own in that kernel, i.e. as long as nothing is
# spilled.  The build checks the compiler's resource report for every instance and fails
# otherwise (a change of compiler or flags must not corrupt results silently).
PINNED_AGPR_KERNEL = "gemm_mi16_kernel"


def _check_pinned_accumulators(src: str, remarks: str) -> None:
    blocks = re.split(r"remark: Function Name: ", remarks)[1:]
    seen = 0
    for b in blocks:
        name = b.split()[0]
        if PINNED_AGPR_KERNEL not in name:
            continue
        seen += 1
        val = {k: int(v) for k, v in re.findall(r"remark:\s+([A-Za-z ]+?)(?: \[bytes/lane\])?: (\d+) \[", b)}
        ok = (val.get("AGPRs") == 256 and val.get("ScratchSize") == 0 and val.get("VGPRs Spill") == 0
              and val.get("SGPRs Spill") == 0 and val.get("VGPRs", 999) < 256)
        if not ok:
            raise RuntimeError(f"{src}: {name} must use exactly the 256 hand-placed AGPRs and spill nothing; "
                               f"the compiler reports {val}")
    if seen == 0:
        raise RuntimeError(f"{src}: no resource report found for {PINNED_AGPR_KERNEL}")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    pinned = os.path.basename(src) == "gemm_mfma.hip"
    extra = ["-Rpass-analysis=kernel-resource-usage"] if pinned else []
    cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if pinned and r.returncode == 0:
        _check_pinned_accumulators(src, r.stderr)
    err = "\n".join(l for l in r.stderr.splitlines()
                    if "packed-fp32-ops" not in l and "kernel-resource-usage" not in l
                    and not (pinned and re.match(r"^\s*\d*\s*\|", l)))   # source excerpts of the remarks
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def source_hash() -> str:
    """Hash of everything the library is built from (kernel sources, their headers, the C header)."""
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".hpp")))
    files.append(os.path.join(os.path.dirname(HERE), "include", "gpt_stage.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def build_library(jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    stamp = source_hash()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, sources()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    # what the library was built from: the binding refuses a library older than its sources
    with open(STAMP, "w") as f:
        f.write(stamp + "\n")
    return LIB


if __name__ == "__main__":
    print(build_library())
