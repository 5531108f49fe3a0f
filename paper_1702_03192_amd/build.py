"""Build libmtnn.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

hipcc cross-compiles without a GPU.  The shared library lands next to this file so that it
travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmtnn.so")

# (the kernel instances first: they take longest, and the pool starts sources in this order)
SOURCES = ["gemm_inst_a.hip", "gemm_inst_b.hip", "gemm_inst_c.hip", "gemm_inst_d.hip", "gemm_inst_e.hip", "gemm_launch.hip", "transpose.hip", "transpose_inplace_rect.hip",
           "fc.hip", "static_scratch.hip", "probe.hip", "api.cpp", "selector.cpp", "gemm_cost.cpp", "device.cpp"]

COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-inline-asm", "-ffp-contract=off",
          "-fvisibility=hidden"]
# packed fp32 VALU forms are switched off for device code: some of their forms have given wrong
# results on this class of machine, and -O3 would otherwise form them from ordinary float code
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    cmd = ["hipcc"] + COMMON + (DEVICE if src.endswith(".hip") else ["-x", "hip", "--offload-arch=gfx950"]) + \
          ["-c", path, "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def _torch_lib_dir():
    import importlib.util
    spec = importlib.util.find_spec("torch")
    if spec is None or not spec.submodule_search_locations:
        return None
    d = os.path.join(list(spec.submodule_search_locations)[0], "lib")
    return d if os.path.exists(os.path.join(d, "libamdhip64.so")) else None


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    sources = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    with ThreadPoolExecutor(max_workers=min(8, len(sources))) as pool:
        objs = list(pool.map(_compile, sources))
    # Link against the HIP runtime PyTorch ships (recorded as NEEDED "libamdhip64.so"), so that a
    # process that has imported torch runs one HIP runtime and torch's stream handles are valid
    # in the library; without torch the system runtime under /opt/rocm/lib is found by RUNPATH.
    tdir = _torch_lib_dir()
    hip_lib_dir = tdir or "/opt/rocm/lib"
    cmd = ["g++", "-shared", "-fPIC", "-o", LIB] + objs + \
          ["-L" + hip_lib_dir, "-l:libamdhip64.so", "-Wl,-rpath,/opt/rocm/lib", "-Wl,--no-undefined"]
    subprocess.run(cmd, check=True)
    if verbose:
        print(LIB)
    return LIB


def build_host_sanitized(out_dir: str, kind: str = "address") -> str:
    """Sanitizer build (g++, host only) of the library's host sources with a driver under
    tests/host_sanitize/; returns the executable.  kind "address": AddressSanitizer + UBSan, with the C
    oracle and driver.cpp; kind "thread": ThreadSanitizer with driver_threads.cpp (several threads on the
    process-wide state; the oracle, which uses OpenMP, is left out).  The kernel launchers are
    replaced by stand-ins that are never reached without a GPU."""
    assert kind in ("address", "thread")
    root = os.path.dirname(HERE)
    drv = os.path.join(root, "tests", "host_sanitize")
    exe = os.path.join(out_dir, "host_sanitize_" + kind)
    san = (["-fsanitize=address,undefined"] if kind == "address" else ["-fsanitize=thread"]) + ["-fno-omit-frame-pointer", "-g", "-O1"]
    cxx = ["g++", "-std=c++17", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-I" + CSRC, "-Wall", "-Wno-unused-parameter",
           "-Wno-deprecated-declarations"] + san
    objs = []
    for src in ["api.cpp", "selector.cpp", "device.cpp", "gemm_cost.cpp"]:
        obj = os.path.join(out_dir, kind + "_" + src + ".o")
        subprocess.run(cxx + ["-c", os.path.join(CSRC, src), "-o", obj], check=True)
        objs.append(obj)
    for src in ["stubs.cpp", "driver.cpp" if kind == "address" else "driver_threads.cpp"]:
        obj = os.path.join(out_dir, kind + "_" + src + ".o")
        subprocess.run(cxx + ["-c", os.path.join(drv, src), "-o", obj], check=True)
        objs.append(obj)
    extra = []
    if kind == "address":
        oobj = os.path.join(out_dir, "oracle.o")
        subprocess.run(["gcc", "-std=c99", "-fopenmp", "-Wall", "-Wextra"] + san + ["-c", os.path.join(root, "oracle", "mtnn_oracle.c"), "-o", oobj],
                       check=True)
        objs.append(oobj)
        extra = ["-fopenmp"]
    hip_lib_dir = _torch_lib_dir() or "/opt/rocm/lib"
    subprocess.run(["g++"] + san + extra + ["-pthread", "-o", exe] + objs + ["-L" + hip_lib_dir, "-l:libamdhip64.so",
                                                                              "-Wl,-rpath," + hip_lib_dir, "-Wl,-rpath,/opt/rocm/lib"], check=True)
    return exe


if __name__ == "__main__":
    build(verbose=True)
