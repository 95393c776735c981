"""Build libentro.so in-tree: g++ for the host part, hipcc (gfx950) for the kernels."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(HERE, "libentro.so")
BUILD = os.path.join(HERE, "_build")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -packed-fp32-ops off: the compiler must not form packed fp32 instructions
DEVICE_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature",
                "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def sources():
    return [os.path.join(CSRC, "entro_host.cpp"), os.path.join(CSRC, "entro_device.hip"),
            os.path.join(CSRC, "entro_compress.hip"), os.path.join(INCLUDE, "entro.h")]


def up_to_date() -> bool:
    return os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(s) for s in sources())


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and up_to_date():
        return LIB
    os.makedirs(BUILD, exist_ok=True)
    host_o = os.path.join(BUILD, "entro_host.o")
    dev_o = os.path.join(BUILD, "entro_device.o")
    comp_o = os.path.join(BUILD, "entro_compress.o")
    cmds = [
        ["g++", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Wall", "-Wextra", "-pthread",
         "-I", INCLUDE, "-c", os.path.join(CSRC, "entro_host.cpp"), "-o", host_o],
        [HIPCC, *DEVICE_FLAGS, "-I", INCLUDE, "-c", os.path.join(CSRC, "entro_device.hip"), "-o", dev_o],
        [HIPCC, *DEVICE_FLAGS, "-I", INCLUDE, "-c", os.path.join(CSRC, "entro_compress.hip"), "-o", comp_o],
        [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, host_o, dev_o, comp_o, "-pthread"],
    ]
    for c in cmds:
        if verbose:
            print(" ".join(c), flush=True)
        subprocess.check_call(c)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
