"""Build ``libmx.so`` (the C-ABI MXInt library) for gfx950 with hipcc, in-tree.

``python -m paper_2307_15517_amd.build`` compiles every ``csrc/*.hip`` translation unit (in
parallel) and links them into ``paper_2307_15517_amd/libmx.so``.  hipcc cross-compiles, so no
GPU is needed to build.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys
from typing import List

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmx.so")
PROBES_SRC = os.path.join(CSRC, "probes", "mx_probes.hip")
PROBES_LIB = os.path.join(HERE, "libmx_probes.so")      # roofline probes of the benchmark, not part of libmx

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    # packed-fp32 VALU forms stay off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def translation_units() -> List[List[str]]:
    """(source, object, extra flags) per unit.  The product kernel is instantiated per block size
    in separate units so that they compile in parallel."""
    units = []
    for name in sorted(os.listdir(CSRC)):
        if not name.endswith(".hip"):
            continue
        stem = name[:-4]
        if stem == "mx_gemm_block":
            for b in (16, 32, 64):
                units.append([os.path.join(CSRC, name), os.path.join(OBJ, "%s_%d.o" % (stem, b)),
                              "-DMX_GEMM_BLOCK=%d" % b])
        else:
            units.append([os.path.join(CSRC, name), os.path.join(OBJ, stem + ".o")])
    return units


def _compile(unit: List[str]) -> str:
    src, obj, extra = unit[0], unit[1], unit[2:]
    cmd = [HIPCC] + FLAGS + extra + ["-c", src, "-o", obj]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "not a recognized feature" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    return out


def build(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    units = translation_units()
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        for unit, out in zip(units, ex.map(_compile, units)):
            if verbose:
                print("compiled", os.path.relpath(unit[1], ROOT), flush=True)
                if out.strip():
                    print(out)
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [u[1] for u in units]
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    if verbose:
        print("linked", os.path.relpath(LIB, ROOT), flush=True)
    tmp = PROBES_LIB + ".tmp.%d" % os.getpid()
    p = subprocess.run([HIPCC] + FLAGS + ["-shared", PROBES_SRC, "-o", tmp], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (PROBES_SRC, p.stdout))
    os.replace(tmp, PROBES_LIB)
    if verbose:
        print("linked", os.path.relpath(PROBES_LIB, ROOT), flush=True)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
