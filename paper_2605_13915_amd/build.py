"""Build the gfx950 MSD library in-tree: csrc/*.hip -> paper_2605_13915_amd/libmsd.so.

Plain hipcc, one translation unit per kernel family, compiled in parallel; objects go to
_build/ (git-ignored).  The library links only against the HIP runtime.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
OUT = os.path.join(HERE, "libmsd.so")
SOURCES = ["msd_api.hip", "decompose.hip", "gemm_w8.hip", "gemm_w4.hip", "gemm_w4_prefill.hip", "gemm_w4_mid.hip", "attn.hip", "attn_wide.hip", "attn_dequant.hip", "attn_mla.hip", "dequant_gemm.hip",
           "stream_probe.hip"]
# -Wno-inline-asm: the LDS-fill asm statements write m0 and list it as clobbered on purpose
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Per-file additions.  attn_mla.hip, attn_wide.hip: MFMA results feed vector-ALU code directly; let the
# compiler place them in VGPRs instead of accumulation registers that would have to be copied out first.
EXTRA_FLAGS = {"attn_mla.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"], "attn_wide.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
               "attn_dequant.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature and says so: harmless, dropped
    quiet = ("packed-fp32-ops", "warnings generated", "warning generated")
    err = "\n".join(l for l in r.stderr.splitlines() if not any(q in l for q in quiet))
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT,
           "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", OUT)
    return OUT


if __name__ == "__main__":
    build()
