"""Builds libivit.so (hand-written HIP for gfx950) in-tree with hipcc.

`python -m paper_2207_01405_amd.build` compiles every .hip file under csrc/ to an object in
_build/ (git-ignored) and links them into paper_2207_01405_amd/libivit.so.  hipcc cross-compiles,
so this works on a machine without a GPU.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libivit.so")
SOURCES = ["api.hip", "trace.hip", "rowwise.hip", "gemm_i8.hip", "gemm_rs.hip", "gemm_ks.hip", "gemm_tl.hip", "attention.hip", "host_helpers.hip", "probe.hip"]
# gemm_rs.hip: MFMA results in ordinary vector registers (the epilogue reads them with vector instructions; the
# weights sit in the accumulation registers instead)
_REGST = ["-mllvm", "-amdgpu-mfma-vgpr-form", "-Wno-inline-asm"]
EXTRA_FLAGS = {"gemm_rs.hip": _REGST, "gemm_ks.hip": _REGST, "gemm_tl.hip": ["-Wno-inline-asm"]}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed FP32 instructions are kept out of every code object of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source_id():
    """Digest of everything the library is compiled from (kernel sources, their headers, the C header)."""
    import hashlib
    h = hashlib.sha256()
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".hpp", ".h")))
    files.append(os.path.join(ROOT, "include", "ivit.h"))
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _compile(src):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc(), *FLAGS, *EXTRA_FLAGS.get(src, []), '-DIVIT_BUILD_ID="%s"' % source_id(), "-c", os.path.join(CSRC, src),
           "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    return obj, r.stderr


def build_lib(verbose=False):
    """Compile and link libivit.so; always rebuilds.  Returns the library path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        results = list(ex.map(_compile, SOURCES))
    if verbose:
        for _, err in results:
            if err.strip():
                print(err, file=sys.stderr)
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *[o for o, _ in results]]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True))
