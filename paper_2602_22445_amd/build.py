"""Build libftred.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2602_22445_amd.build [--force]

Objects go to paper_2602_22445_amd/_build/, the library to
paper_2602_22445_amd/libftred.so.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import glob
import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libftred.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _deps():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))


def source_hash() -> str:
    """sha256 over the HIP sources and the headers (csrc/ and include/), in name order.
    The build compiles it into the library (ftred_source_hash), so that a library
    that was built from other sources than those on disk can be told apart."""
    h = hashlib.sha256()
    for p in sorted(_sources() + _deps(), key=os.path.basename):
        h.update(os.path.basename(p).encode())
        h.update(open(p, "rb").read())
    return h.hexdigest()


def built_hash():
    """The source hash the library on disk was built from, or None."""
    if not os.path.exists(LIB):
        return None
    import ctypes
    try:
        L = ctypes.CDLL(LIB)
        L.ftred_source_hash.restype = ctypes.c_char_p
        return L.ftred_source_hash().decode()
    except (OSError, AttributeError):
        return None


def needs_build() -> bool:
    return built_hash() != source_hash()


def build(force: bool = True, jobs: int = 8, verbose: bool = False, incremental: bool = False) -> str:
    """Compile every .hip source and link the shared library.  Returns its path.
    incremental: keep an object that is newer than its source and every header it includes (the file that
    carries the source hash is compiled every time)."""
    if not force and not needs_build():
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    sha = source_hash()
    def up_to_date(obj, dep_file):
        # the object is newer than everything the compiler read for it (its dependency file lists that)
        if not (os.path.exists(obj) and os.path.exists(dep_file)):
            return False
        words = open(dep_file).read().replace("\\\n", " ").split()
        deps = [w for w in words[1:] if not w.endswith(":")]
        t = os.path.getmtime(obj)
        return all(os.path.exists(d) and os.path.getmtime(d) < t for d in deps)

    def compile_one(src):
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        dep_file = obj[:-2] + ".d"
        carries_hash = os.path.basename(src) == "ftred_api.hip"
        if incremental and not carries_hash and up_to_date(obj, dep_file):
            return obj
        cmd = ([HIPCC] + FLAGS + (["-DFTRED_SOURCE_HASH=\"%s\"" % sha] if carries_hash else []) +
               ["-MMD", "-MF", dep_file, "-c", src, "-o", obj])
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, _sources()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True, incremental="--incremental" in sys.argv))
