"""Builds the HIP library (libidf.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import glob
import os
import shlex
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libidf.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def extra_flags():
    """Further hipcc flags from the environment (IDF_HIPCC_FLAGS), e.g. -D switches of a timing build."""
    return shlex.split(os.environ.get("IDF_HIPCC_FLAGS", ""))


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))
    return all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every kernel and the host side into paper_1804_10727_amd/libidf.so."""
    if not force and up_to_date():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "build")
    os.makedirs(objdir, exist_ok=True)
    # the host pass does not know the GPU-only feature switch and says so once per use: harmless
    noise = "is not a recognized feature for this target"

    def run(cmd):
        if verbose:
            print(" ".join(cmd))
        proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
        if err.strip():
            print(err)
        if proc.returncode != 0:
            raise RuntimeError(f"hipcc failed with code {proc.returncode}: {' '.join(cmd[-3:])}")

    # one translation unit per kernel file, compiled side by side, then linked
    objs = [os.path.join(objdir, os.path.basename(f)[:-4] + ".o") for f in sources()]
    with ThreadPoolExecutor(max_workers=min(8, len(objs))) as ex:
        list(ex.map(lambda fo: run([hipcc] + HIPCC_FLAGS + extra_flags() + ["-c", "-o", fo[1], fo[0]]), zip(sources(), objs)))
    run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
