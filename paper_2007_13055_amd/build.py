"""Compile the HIP sources under csrc/ into libbsr_spmm.so (in-tree, gfx950 only)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbsr_spmm.so")
# The checking build: the same sources with -DBSR_PLAIN_LOADS (every hand-placed load becomes an ordinary one
# with compiler-placed waits).  Only tests load it, to hold the two builds' results against each other.
OBJDIR_PLAIN = os.path.join(HERE, "_build_plain")
LIB_PLAIN = os.path.join(HERE, "libbsr_spmm_plain.so")

# -packed-fp32-ops off: the compiler must not form packed fp32 VALU instructions on this target.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Kernels in these files issue loads from inline assembly and place the waits themselves; the compiler
# does not know such a register is still being filled, so a spill of one would store garbage.  The
# build therefore fails if any kernel of these files spills a vector register.
NO_SPILL = ("bsr_mfma_ksplit.hip", "bsr_mfma_tile.hip", "bsr_mfma_small.hip", "bsr_mfma_group.hip")


def _spilling_kernels(remarks: str):
    """Names of kernels whose resource-usage remarks report VGPR spills or scratch memory."""
    bad, name = [], None
    for line in remarks.splitlines():
        if "remark:" not in line:
            continue
        text = line.split("remark:", 1)[1].strip()
        if text.startswith("Function Name:"):
            name = text.split(":", 1)[1].split("[")[0].strip()
        elif text.startswith("VGPRs Spill:") or text.startswith("ScratchSize"):
            if int(text.split(":", 1)[1].split("[")[0].strip()) != 0 and name not in bad:
                bad.append(name)
    return bad


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _compile(src, force, plain=False):
    obj = os.path.join(OBJDIR_PLAIN if plain else OBJDIR, os.path.basename(src) + ".o")
    deps = [src] + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    check = os.path.basename(src) in NO_SPILL and not plain
    extra = ["-Rpass-analysis=kernel-resource-usage"] if check else []
    if plain:
        extra.append("-DBSR_PLAIN_LOADS")
    r = subprocess.run(["hipcc", *HIPCC_FLAGS, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
    if check:
        bad = _spilling_kernels(r.stderr) if r.returncode == 0 else []
        if bad:
            os.remove(obj)
            raise RuntimeError(f"{src}: kernels with hand-placed loads spill registers: {bad}")
        keep, skip = [], 0
        for l in r.stderr.splitlines():          # drop the remarks and the source excerpts printed under them
            if "kernel-resource-usage" in l:
                skip = 2
            elif skip and (l.lstrip().startswith("|") or l.strip()[:1].isdigit()):
                skip -= 1
            else:
                keep.append(l)
        r.stderr = "\n".join(keep)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = True, jobs: int = 4, plain: bool = False) -> str:
    """Compile every .hip file and link the shared library (plain: the checking build); returns its path."""
    os.makedirs(OBJDIR_PLAIN if plain else OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, plain), sources()))
    lib = LIB_PLAIN if plain else LIB
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc",
                        "-Wno-unused-command-line-argument", "-o", lib, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return lib


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
    print(build(force="--incremental" not in sys.argv, plain=True))
