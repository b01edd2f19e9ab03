"""Build tests/native/abi_client: a C++ client of the C ABI with no Python in it (test code; it
links the HIP library and, being a checker, the oracle).  Host compiler only: the client holds no
device code, it calls the HIP runtime for memory and the library for everything else."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
SRC = os.path.join(HERE, "abi_client.cpp")
EXE = os.path.join(HERE, "abi_client")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


def build() -> str:
    sys.path.insert(0, ROOT)
    from oracle import build as oracle_build
    from paper_2106_10796_amd import build as hip_build
    hip_build.ensure_built()
    oracle_build.build(force=False)
    pkg, orc = os.path.join(ROOT, "paper_2106_10796_amd"), os.path.join(ROOT, "oracle")
    tmp = EXE + ".tmp%d" % os.getpid()
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra", "-D__HIP_PLATFORM_AMD__",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROCM, "include"), SRC, "-o", tmp,
           "-L", pkg, "-l:libcdsgd.so", "-L", orc, "-l:liboracle_cdsgd.so",
           "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
           # found relative to the executable, wherever the tree is copied to
           "-Wl,-rpath,$ORIGIN/../../paper_2106_10796_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
           "-Wl,-rpath," + os.path.join(ROCM, "lib")]
    subprocess.run(cmd, check=True)
    os.replace(tmp, EXE)
    return EXE


def ensure_built() -> str:
    """Build if the client is missing or older than its source or the header it is compiled against.
    (It links the two libraries dynamically, so a rebuilt library needs no rebuilt client.)"""
    deps = [SRC, os.path.join(ROOT, "include", "cdsgd.h")]
    if os.path.exists(EXE) and all(os.path.getmtime(EXE) >= os.path.getmtime(d) for d in deps):
        return EXE
    return build()


if __name__ == "__main__":
    print(build())
