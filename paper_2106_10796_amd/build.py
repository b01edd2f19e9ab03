"""Build libcdsgd.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import hashlib
import os
import re
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
SRC = os.path.join(PKG, "csrc", "cdsgd.hip")
SRC_HOST = [os.path.join(PKG, "csrc", "cdsgd_cost_model.cpp")]   # host-only parts of the library
INCLUDE = os.path.join(ROOT, "include")
LIB = os.path.join(PKG, "libcdsgd.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # IEEE as written: no contraction of a*b+c behind our back (the fused
    # multiply-adds of the update rules are spelled out), denormals kept
    "-ffp-contract=off", "-fno-fast-math",
    # no packed-fp32 instructions from the auto-vectoriser
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    p = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(p):
        raise RuntimeError("hipcc not found")
    return p


def source_id(extra_flags=()) -> str:
    """Identity of what a build is made from: the sources, the headers and the flags (16 hex digits).
    It is compiled into the library (cdsgd_build_id) so that a library can be matched to the tree."""
    h = hashlib.sha256()
    headers = sorted(os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h"))
    csrc = os.path.dirname(SRC)                       # cdsgd.hip includes the kernels' .hpp files beside it
    sources = sorted(os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith((".hip", ".hpp", ".cpp")))
    assert SRC in sources and all(p in sources for p in SRC_HOST)
    for path in [*sources, *headers]:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as fh:
            h.update(fh.read())
        h.update(b"\0")
    h.update(" ".join([*HIPCC_FLAGS, *extra_flags]).encode())
    return h.hexdigest()[:16]


def built_id(path=LIB):
    """The source identity a built library carries, or None (no library, or one without an identity)."""
    try:
        with open(path, "rb") as fh:
            m = re.search(rb"CDSGD_BUILD_ID=([0-9a-f]{16})", fh.read())
    except OSError:
        return None
    return m.group(1).decode() if m else None


def build(extra_flags=(), out=LIB, verbose=False) -> str:
    tmp = out + ".tmp%d" % os.getpid()
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, '-DCDSGD_BUILD_ID_HEX="%s"' % source_id(extra_flags),
           "-I", INCLUDE, SRC, *SRC_HOST, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 target feature: harmless
    log = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout)
    if verbose and log:
        print(log, flush=True)
    os.replace(tmp, out)
    return out


def ensure_built() -> str:
    """Build if no library is there or if the one that is there was made from other sources,
    headers or flags than the tree now holds (tests, the smoke check and the benchmark call this;
    the binding itself never builds and never falls back).  The comparison is by content, not by
    file time, so a tree that was copied elsewhere together with its library is not rebuilt."""
    if os.path.exists(LIB) and built_id(LIB) == source_id():
        return LIB
    return build()


if __name__ == "__main__":
    print(build(extra_flags=sys.argv[1:], verbose=True))
