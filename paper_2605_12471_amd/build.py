"""Build libkvfold.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_DIR = os.path.join(_HERE, "_lib")
LIB_PATH = os.path.join(LIB_DIR, "libkvfold.so")
SOURCES = ["kvfold_api.hip", "kvfold_plan.cpp", "append.hip", "attn_bf16.hip", "attn_f32.hip", "combine.hip", "peaks.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the attention kernels unroll a 32-slot software pipeline by pragma; before the per-slot conditions
    # fold, its body is larger than the default size limit for pragma-forced unrolling
    "-mllvm", "-pragma-unroll-threshold=100000",
    # the compiler's per-kernel register / scratch report is kept next to the library
    "-Rpass-analysis=kernel-resource-usage",
]
RESOURCE_REPORT = os.path.join(LIB_DIR, "kernel_resources.txt")
C_CLIENT_PATH = os.path.join(LIB_DIR, "kvfold_c_client")
INCLUDE_DIR = os.path.join(os.path.dirname(_HERE), "include")


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library. Always recompiles."""
    os.makedirs(LIB_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(LIB_DIR, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = [hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    report = []
    for cmd, p in procs:
        out, _ = p.communicate()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode:
            raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), "\n".join(lines)))
        report += [l.split("remark: ", 1)[1].replace(" [-Rpass-analysis=kernel-resource-usage]", "")
                   for l in lines if "remark: " in l and "kernel-resource-usage" in l]
        rest = "\n".join(l for l in lines if "kernel-resource-usage" not in l and "|" not in l[:12])
        if verbose and rest.strip():
            print(rest)
    with open(RESOURCE_REPORT, "w") as f:
        f.write("\n".join(report) + "\n")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    subprocess.run(cmd, check=True)
    return LIB_PATH


def build_c_client() -> str:
    """Compile the plain-C caller of the library (gcc, C11, no HIP compiler): it sees only include/kvfold.h, the HIP
    runtime API and the shared library."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I" + INCLUDE_DIR,
           "-isystem", os.path.join(rocm, "include"), os.path.join(CSRC, "c_client.c"), "-o", C_CLIENT_PATH,
           "-L" + LIB_DIR, "-lkvfold", "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    subprocess.run(cmd, check=True)
    return C_CLIENT_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_c_client())
