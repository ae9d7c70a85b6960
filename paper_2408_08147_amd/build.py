"""Builds libkvx.so (HIP, gfx950) in-tree with hipcc."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libkvx.so")
SOURCES = [os.path.join(CSRC, "kvx_api.cpp"), os.path.join(CSRC, "kvx_retriever.cpp"),
           os.path.join(CSRC, "kvx_kernels.hip"), os.path.join(CSRC, "kvx_noalloc.hip")]
ID_TAG = "kvx-sources:"
HEADERS = [os.path.join(CSRC, "kvx_internal.h"), os.path.join(ROOT, "include", "kvx.h")]


def source_id() -> str:
    """Hash of every file the library is built from; the build bakes it in (kvx_build_id)."""
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:32]


def built_id():
    """The id baked into the built library, read without loading it into this process; None if there is
    no library or it carries no id."""
    if not os.path.exists(LIB):
        return None
    with open(LIB, "rb") as fh:
        blob = fh.read()
    at = blob.find(ID_TAG.encode())
    if at < 0:
        return None
    return blob[at + len(ID_TAG):at + len(ID_TAG) + 32].decode("ascii", "replace")


def is_stale() -> bool:
    return built_id() != source_id()


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           "-DKVX_BUILD_ID=\"%s%s\"" % (ID_TAG, source_id()),
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-x", "hip", *SOURCES, "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                    if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
