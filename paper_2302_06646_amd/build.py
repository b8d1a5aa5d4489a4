"""Compile the HIP library for gfx950: `python -m paper_2302_06646_amd.build`."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblongconv.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # no packed-fp32 instructions (compiler-generated v_pk_*_f32 are not trusted on the test machines)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l)      # host pass does not know the feature: harmless
    if out.strip() and verbose:
        print(out)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)


def build(verbose: bool = True) -> str:
    """Compile every csrc/*.hip (in parallel) and link liblongconv.so next to this file."""
    from concurrent.futures import ThreadPoolExecutor
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    cflags = [f for f in FLAGS if f != "-shared"]
    # -save-temps=obj leaves the device assembly of every source next to its object file, for the hazard check
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        list(ex.map(lambda so: _run([HIPCC, *cflags, "-save-temps=obj", "-c", so[0], "-o", so[1]], verbose),
                    zip(srcs, objs)))
    check_assembly(objdir, srcs, verbose)
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    return LIB


def check_assembly(objdir: str, srcs, verbose: bool = True) -> None:
    """Every kernel's assembly must keep the issue distance between an MFMA and the readers of its result
    (see isa_check.py); a violation is a build error."""
    from . import isa_check
    bad, seen = [], 0
    for s in srcs:
        stem = os.path.basename(s)[:-4]
        for asm in glob.glob(os.path.join(objdir, stem + "-hip-amdgcn-amd-amdhsa-gfx950*.s")):
            seen += 1
            bad += [(stem,) + b for b in isa_check.check_file(asm)]
    if seen == 0:
        raise RuntimeError("no device assembly found in " + objdir + ": the hazard check could not run")
    if bad:
        raise RuntimeError("MFMA result read too early in:\n" + "\n".join(
            f"  {b[0]}: {b[1]}: {b[2]} slots: {b[3]} -> {b[4]}" for b in bad))
    if verbose:
        print(f"assembly hazard check ok ({seen} files)", flush=True)


if __name__ == "__main__":
    build()
    sys.exit(0)
