"""Builds libvnm.so (the C-ABI library with the gfx950 kernels) in-tree with hipcc."""

from __future__ import annotations

import glob
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libvnm.so")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-Wno-unused-value",
    # packed-fp32 VALU forms are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))


HASH_MARKER = "VNM_SOURCE_HASH="


def built_hash(path: str = LIB_PATH) -> str:
    """The source hash a built library carries, read from the file itself (nothing is loaded)."""
    try:
        with open(path, "rb") as f:
            data = f.read()
    except OSError:
        return ""
    i = data.find(HASH_MARKER.encode())
    return data[i + len(HASH_MARKER):i + len(HASH_MARKER) + 64].decode("ascii", "replace") if i >= 0 else ""


def source_hash() -> str:
    """SHA-256 over everything the library is compiled from (kernels, internal and public headers,
    flags), in a fixed order.  The library carries the value it was built with (vnm_source_hash),
    so that a stale binary next to edited sources is noticed when it is loaded."""
    import hashlib
    h = hashlib.sha256()
    files = sources() + sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.h"))) \
        + sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    for path in files:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
        h.update(b"\0")
    h.update(" ".join(HIPCC_FLAGS).encode())
    return h.hexdigest()


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source (one hipcc process per file, in parallel) and link libvnm.so;
    always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="vnm_build_")
    try:
        def compile_one(src):
            obj = os.path.join(tmp, os.path.basename(src) + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-c", src, "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
            return obj
        # the hash of the sources, compiled in as vnm_source_hash()
        stamp = os.path.join(tmp, "vnm_source_hash.hip")
        with open(stamp, "w") as f:
            f.write('static const char stamp[] = "%s%s";\n'
                    'extern "C" const char* vnm_source_hash(void) { return stamp + %d; }\n'
                    % (HASH_MARKER, source_hash(), len(HASH_MARKER)))
        srcs = sources() + [stamp]
        with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
            objs = list(pool.map(compile_one, srcs))
        # linked under a temporary name and moved into place, so that a process that has the old
        # file mapped keeps a valid image
        linked = LIB_PATH + ".tmp%d" % os.getpid()
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", linked]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc (link) failed:\n" + res.stdout + res.stderr)
        os.replace(linked, LIB_PATH)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
