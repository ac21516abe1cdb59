"""Builds libverillm.so (the C-ABI library) for gfx950 with hipcc, in-tree next to this file."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libverillm.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["engine.hip", "kernels_rows.hip", "kernels_gemm_simple.hip", "kernels_gemm_mfma.hip", "kernels_gemm_skinny.hip", "kernels_attn_decode.hip",
           "kernels_attn_rowwise.hip", "kernels_attn_mfma.hip", "kernels_compare.hip", "kernels_merkle.hip"]

FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         # packed-fp32 instructions are kept out of every kernel (the compiler otherwise forms them at -O3)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    errs = [ln for ln in r.stderr.splitlines() if "error" in ln.lower()]
    if errs:
        sys.stderr.write("\n".join(errs) + "\n")
    return obj


def _check_hand_issued_mfma() -> None:
    """The attention kernel issues some matrix instructions as inline assembly; the compiler then inserts none of the
    wait states they need next to vector instructions.  Its device assembly is generated once more as text and checked
    (see check_mfma_asm.py); a violation fails the build instead of giving wrong numbers now and then."""
    if HERE not in sys.path:
        sys.path.insert(0, HERE)
    import check_mfma_asm                                       # sits beside this file; also when run as a script
    asm = os.path.join(OBJ_DIR, "kernels_attn_mfma.s")
    cmd = [hipcc()] + FLAGS + ["-S", "--cuda-device-only", os.path.join(CSRC, "kernels_attn_mfma.hip"), "-o", asm]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc -S failed for kernels_attn_mfma.hip:\n%s\n%s" % (r.stdout, r.stderr))
    bad = check_mfma_asm.check(asm)
    if bad:
        raise RuntimeError("hand-issued MFMA next to a vector instruction on its registers:\n" + "\n".join(bad[:20]))


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        chk = ex.submit(_check_hand_issued_mfma)
        objs = list(ex.map(_compile, SOURCES))
        chk.result()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Wl,-z,defs", "-o", LIB] + objs   # unresolved symbols fail the build, not the load
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
