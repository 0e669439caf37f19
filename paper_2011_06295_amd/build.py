"""Builds libsparseconv.so (HIP kernels + C ABI) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsparseconv.so")
SOURCES = ["kernels.hip", "probes.hip", "api.cpp", "plan.cpp", "host_csr.cpp"]

# packed fp32 VALU forms are switched off for the device pass (the host pass
# prints a harmless "not a recognized feature" note for the same flag)
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


def build_sanitize(verbose: bool = False) -> str:
    """Host-only build for the sanitizer check: CSR encoder, planner and the C ABI (no kernels; the launch
    functions are stand-ins that report "not supported"), the CPU oracle and tests/sanitize/driver.cpp in one
    executable compiled with -fsanitize=address,undefined.  Returns its path; needs no GPU."""
    root = os.path.dirname(HERE)
    out_dir = os.path.join(root, "_build")
    os.makedirs(out_dir, exist_ok=True)
    exe = os.path.join(out_dir, "sanitize_driver")
    oracle_o = os.path.join(out_dir, "oracle_sanitize.o")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]
    cmds = [
        ["gcc", "-std=c11", "-ffp-contract=off", "-c", *san, "-o", oracle_o, os.path.join(root, "oracle", "sparse_conv_oracle.c")],
        ["g++", "-std=c++17", *san, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", exe,
         os.path.join(root, "tests", "sanitize", "driver.cpp"), oracle_o,
         *[os.path.join(CSRC, f) for f in ("api.cpp", "plan.cpp", "host_csr.cpp", "no_device.cpp")],
         "-L/opt/rocm/lib", "-Wl,-rpath,/opt/rocm/lib", "-lamdhip64", "-lm"],
    ]
    for cmd in cmds:
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("sanitizer build failed:\n" + res.stdout)
    return exe


if __name__ == "__main__":
    if "--sanitize" in sys.argv[1:]:
        print(build_sanitize(verbose=True))
    else:
        print(build(verbose=True))
