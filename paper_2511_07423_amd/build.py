"""Compiles the HIP sources into the in-tree shared library (gfx950 only)."""
import concurrent.futures
import glob
import os
import shutil
import subprocess

from . import mfma_hazards

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsynera.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["gemm_nf4_high.hip", "gemm_nf4_low.hip", "gemm_nf2.hip", "gemm_k64.hip", "api.hip", "elementwise.hip", "confidence.hip", "attention.hip",
           "importance.hip", "gemm.hip", "gemm_static.hip", "ceilings.hip", "scheduler.cpp"]
# sources whose kernels issue MFMAs from inline assembly: their device assembly is kept and checked
ASM_CHECKED = {"gemm_nf4_high.hip": "proj_kernel", "gemm_nf4_low.hip": "proj_kernel", "gemm_nf2.hip": "proj_kernel", "gemm_k64.hip": "proj_kernel",
               "ceilings.hip": "ceiling_mfma_f16"}
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# The attention kernel's builtin MFMAs take their accumulators in VGPRs: in AGPRs (the compiler's default choice)
# all 36 of them were read out at the top of every tile iteration and written back at its end.
EXTRA_FLAGS = {"attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _quiet(stderr):
    # hipcc's host pass does not know the packed-fp32 target feature and says so; harmless.
    err = "\n".join(l for l in stderr.splitlines() if "packed-fp32-ops" not in l)
    return err[:3000] + "\n...\n" + err[-3000:] if len(err) > 6000 else err


def _compile(src):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
    if src in ASM_CHECKED:
        cmd.append("-save-temps=obj")
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=OBJ_DIR)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n" + _quiet(res.stderr))
    return obj, _quiet(res.stderr)


def build_library(verbose=False):
    """hipcc -> paper_2511_07423_amd/libsynera.so.  Always recompiles every source (in parallel), checks the
    generated assembly of the inline-MFMA kernels for unsettled accumulator reads, then links."""
    shutil.rmtree(OBJ_DIR, ignore_errors=True)
    os.makedirs(OBJ_DIR)
    with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as pool:
        done = list(pool.map(_compile, SOURCES))
    for src, name_filter in ASM_CHECKED.items():
        stem = src.replace(".hip", "")
        asm = glob.glob(os.path.join(OBJ_DIR, stem + "-hip-amdgcn-amd-amdhsa-gfx950*.s"))
        if len(asm) != 1:
            raise RuntimeError(f"expected one device assembly file for {src}, found {asm}")
        n_kernels, n_mfma, hazards = mfma_hazards.check_file(asm[0], name_filter)
        if n_kernels == 0 or n_mfma == 0:
            raise RuntimeError(f"{src}: no '{name_filter}' kernels with MFMAs in {asm[0]}: the check saw nothing")
        if hazards:
            raise RuntimeError(f"{src}: {len(hazards)} accumulator reads behind an unsettled MFMA:\n" + "\n".join(hazards[:20]))
        if verbose:
            print(f"{src}: {n_kernels} kernels, {n_mfma} inline MFMAs, no unsettled accumulator access")
    res = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *[o for o, _ in done], "-o", LIB],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + _quiet(res.stderr))
    for f in os.listdir(OBJ_DIR):              # keep only the checked assembly (tests re-read it)
        if not f.endswith("gfx950.s"):
            os.remove(os.path.join(OBJ_DIR, f))
    if verbose:
        for _, err in done:
            if err.strip():
                print(err)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
