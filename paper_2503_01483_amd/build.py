"""Compile the HIP sources of this package into ``libkurtail.so`` for gfx950."""
import hashlib
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libkurtail.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]


def source_id():
    """16 hex digits over the contents of every file the library is compiled from (csrc/ and the C header).
    The library carries the id it was built from (kt_build_id()), so that the binding can tell a library that no
    longer matches its sources, whatever the files' time stamps say."""
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".h"))]
    files.append(os.path.join(os.path.dirname(_HERE), "include", "kt.h"))
    for f in files:
        h.update(os.path.basename(f).encode())
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def build_library(verbose=False):
    """Always recompiles (cross-compiles without a GPU). Returns the library path."""
    extra = os.environ.get("KT_HIPCC_EXTRA", "").split()  # developer knob: extra hipcc flags
    cmd = ["hipcc", *HIPCC_FLAGS, f'-DKT_BUILD_ID="{source_id()}"', *extra, *sources(), "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
