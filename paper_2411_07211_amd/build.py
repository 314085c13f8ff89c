"""Builds libmxblas.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2411_07211_amd.build            # compile what changed, link
    python -m paper_2411_07211_amd.build --force    # recompile everything
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmxblas.so")
SOURCES = ["handle.hip", "level1.hip", "level1_pair.hip", "matvec.hip", "symv_ger.hip", "trisweep.hip", "skinny.hip", "tiny.hip", "trsv.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Wno-unused-parameter",
    # packed fp32 VALU forms are kept off for every kernel in this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _headers():
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    hs.append(os.path.join(os.path.dirname(HERE), "include", "mxblas.h"))
    return hs


# The chained triangular solve is correct only while hipcc keeps its scalar spills low: a build in
# which the compiler had formed every tile row's address ahead of the loops and spilled 300-470
# scalar registers per kernel gave a wrong result in one instance (double precision, lower, not
# transposed), while every build with 13-90 spilled scalars has passed all tests.  The cause was
# never found in the source, so the build checks the compiler's own report and refuses a library
# whose chained kernels spill more scalars than has ever been seen to work.
MAX_CHAIN_SGPR_SPILLS = 128
# The chained kernel is written to fit the 512 registers of a wavefront alone on its SIMD unit.
# An instance that spills vector registers is still right but far slower (14 spilled registers:
# n = 4096 in 105 us instead of 72; 23: n = 16384 in 557 us instead of 313), which no test shows, so
# the build refuses that as well.
MAX_CHAIN_VGPR_SPILLS = 0


def check_chain_spills(report: str) -> dict:
    """Scalar spills per trsv_chain_kernel instance, from hipcc's kernel-resource-usage remarks;
    raises if one exceeds MAX_CHAIN_SGPR_SPILLS, if one spills vector registers, or if no instance
    is reported at all."""
    spills, vector, name = {}, {}, None
    for line in report.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"SGPRs Spill: (\d+)", line)
        if m and name and "trsv_chain_kernel" in name:
            spills[name] = int(m.group(1))
        m = re.search(r"VGPRs Spill: (\d+)", line)
        if m and name and "trsv_chain_kernel" in name:
            vector[name] = int(m.group(1))
    if not spills:
        raise RuntimeError("build: hipcc reported no resource usage for trsv_chain_kernel; cannot check its scalar spills")
    bad = {k: v for k, v in spills.items() if v > MAX_CHAIN_SGPR_SPILLS}
    if bad:
        raise RuntimeError(f"build: trsv_chain_kernel spills more than {MAX_CHAIN_SGPR_SPILLS} scalar registers in {bad}: "
                           "builds like this have given wrong results; change trsv.hip (see load_rows) until the spills are back down")
    slow = {k: v for k, v in vector.items() if v > MAX_CHAIN_VGPR_SPILLS}
    if slow:
        raise RuntimeError(f"build: trsv_chain_kernel spills vector registers in {slow}: "
                           "such instances run up to 1.8 times slower; lower the register pressure in trsv.hip")
    return spills


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    path = os.path.join(CSRC, src)
    deps = [path] + _headers()
    if force or not os.path.exists(obj) or any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps):
        if src == "trsv.hip":
            r = subprocess.run([HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-c", path, "-o", obj], stderr=subprocess.PIPE, text=True)
            if r.returncode != 0:
                sys.stderr.write(r.stderr)
                raise subprocess.CalledProcessError(r.returncode, r.args)
            try:
                check_chain_spills(r.stderr)
            except RuntimeError:
                os.remove(obj)
                raise
        else:
            subprocess.check_call([HIPCC, *FLAGS, "-c", path, "-o", obj])
    return obj


def build(force: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv[1:]))
