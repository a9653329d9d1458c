"""Build libsuperkernel.so (HIP, gfx950 only) in-tree next to this file."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsuperkernel.so")
CEILINGS_LIB = os.path.join(HERE, "libsk_ceilings.so")  # measuring aid of bench.py, not part of the ABI
SOURCES = ["superkernel.hip", "planner.cpp", "queue.cpp"]
HEADERS = ["kernels.hip.h", "sk_internal.h", os.path.join(ROOT, "include", "superkernel.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
    # The tile queue's atomic is issued by one thread and its answer is wanted several loop steps
    # later.  The compiler's wave-level atomic combining reads the answer back at once, which
    # makes the wave wait for every load in flight at that point.
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
]


DIAG_LIB = os.path.join(HERE, "libsuperkernel_diag.so")  # -DSK_DIAG_CLOCKS: per-tile phase stamps (tile_phases.py)
DIAG_ALL_LIB = os.path.join(HERE, "libsuperkernel_diag_all.so")  # the same with every workgroup of a launch stamped


def build_diag(verbose: bool = False, all_workgroups: bool = False) -> str:
    """The library once more with -DSK_DIAG_CLOCKS, as libsuperkernel_diag.so (a measuring aid: every tile
    of the first 16 workgroups stamps the device clock at its phase boundaries), or, with `all_workgroups`, as
    libsuperkernel_diag_all.so (512 workgroups, their first 24 tiles).  Not built by build()."""
    if all_workgroups:
        return build(force=True, verbose=verbose, extra=("-DSK_DIAG_CLOCKS", "-DSK_DIAG_WGS_N=512", "-DSK_DIAG_TILES_N=24"),
                     lib=DIAG_ALL_LIB, ceilings=False, tag="diag_all")
    return build(force=True, verbose=verbose, extra=("-DSK_DIAG_CLOCKS",), lib=DIAG_LIB, ceilings=False, tag="diag")


def build(force: bool = True, verbose: bool = False, extra=(), lib: str = LIB, ceilings: bool = True, tag: str = "") -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    if not force and os.path.exists(lib):
        newest = max(os.path.getmtime(p) for p in srcs + [os.path.join(CSRC, h) if not os.path.isabs(h) else h
                                                          for h in HEADERS])
        if os.path.getmtime(lib) >= newest:
            return lib
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    o_hip = os.path.join(obj_dir, f"superkernel{tag}.o")
    o_cpp = os.path.join(obj_dir, "planner.o")
    o_queue = os.path.join(obj_dir, "queue.o")
    steps = [
        [hipcc, *HIPCC_FLAGS, *extra, *inc, "-c", srcs[0], "-o", o_hip],
        ["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", *inc, "-c", srcs[1], "-o", o_cpp],
        # host code that calls the HIP runtime (events): the host compiler with the runtime's headers
        ["g++", "-O2", "-std=c++17", "-fPIC", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include", *inc, "-c", srcs[2],
         "-o", o_queue],
        [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", o_hip, o_cpp, o_queue, "-o", lib],
    ]
    if ceilings:
        steps.append([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
                      "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                      os.path.join(CSRC, "ceilings.hip"), "-o", CEILINGS_LIB])
    for cmd in steps:
        if verbose:
            print(" ".join(cmd))
        res = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass warns that it does not know the packed-fp32 feature: harmless noise
        err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("build step failed: " + " ".join(cmd) + "\n" + err)
        if verbose and err.strip():
            print(err)
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose=True))
