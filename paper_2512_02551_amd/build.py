"""Builds libhgemm.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

The MFMA kernel template is instantiated for every configuration in csrc/hgemm_configs.inc;
the instantiations are spread over HGEMM_NUM_CHUNKS translation units that compile in parallel.
"""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(_HERE, "libhgemm.so")
HEADERS = [os.path.join(CSRC, n) for n in ("hgemm_mfma.hpp", "hgemm_aux.hpp", "hgemm_registry.hpp", "hgemm_configs.inc",
                                           "hgemm_skinny.hpp", "dispatch_table.inc", "dispatch_table_tn.inc", "plan_model.inc")] + [os.path.join(os.path.dirname(_HERE), "include", "hgemm.h")]
API_SRC = os.path.join(CSRC, "hgemm_api.hip")
KERNEL_SRC = os.path.join(CSRC, "hgemm_kernels.hip")
SKINNY_SRC = os.path.join(CSRC, "hgemm_skinny.hip")
DEPENDS = HEADERS + [API_SRC, KERNEL_SRC, SKINNY_SRC]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed-fp32 instructions stay off in all device code of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def num_chunks() -> int:
    text = open(os.path.join(CSRC, "hgemm_configs.inc")).read()
    return int(re.search(r"#define HGEMM_NUM_CHUNKS (\d+)", text).group(1))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in DEPENDS)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("command failed: " + " ".join(cmd) + "\n" + out[-6000:])
    if verbose and out.strip():
        print(out)


def build(force: bool = True, verbose: bool = False, jobs: int = 0) -> str:
    """Compile the library.  ``force=False`` skips the compile when the library is newer than its sources."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    n = num_chunks()
    tasks = [[hipcc] + HIPCC_FLAGS + ["-c", API_SRC, "-o", os.path.join(OBJ, "api.o")],
             [hipcc] + HIPCC_FLAGS + ["-c", SKINNY_SRC, "-o", os.path.join(OBJ, "skinny.o")]]
    for k in range(n):
        tasks.append([hipcc] + HIPCC_FLAGS + [f"-DHGEMM_CHUNK={k}", "-c", KERNEL_SRC, "-o", os.path.join(OBJ, f"kernels_{k}.o")])
    jobs = jobs or min(len(tasks), max(1, min(16, os.cpu_count() or 1)))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        for f in [pool.submit(_run, t, verbose) for t in tasks]:
            f.result()
    tmp = LIB + f".tmp{os.getpid()}"
    objs = [os.path.join(OBJ, "api.o"), os.path.join(OBJ, "skinny.o")] + [os.path.join(OBJ, f"kernels_{k}.o") for k in range(n)]
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs, verbose)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
