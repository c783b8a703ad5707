"""Compiles csrc/*.hip into libtvmattn.so for gfx950 with hipcc (in-tree, beside this file)."""
import glob
import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libtvmattn.so")
PEAKS_LIB = os.path.join(HERE, "libtvmpeaks.so")  # bench.py's microbenchmarks of the card's ceilings, not part of the product

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",  # the LDS-DMA asm names m0 on purpose
]
# MFMA results straight into VGPRs (the score tiles are consumed by the VALU).  Not used for the translation
# units that hold only d > 96 instantiations (bwd_mfma_wide.hip, bwd_mfma_onesided2.hip), whose register
# pressure sends the compiler's AGPR rewrite pass astray (more spills, 2 % slower).
PER_FILE = {
    "fwd_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "fwd_mfma_qnorm.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    "bwd_mfma_onesided1.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
    # hand-ordered instruction stream: source order must survive to the ISA
    "bwd_row_pipe.hip": ["-mllvm", "-enable-misched=false"],
    "bwd_col_pipe.hip": ["-mllvm", "-enable-misched=false"],
    "bwd_row_pipe_tangent.hip": ["-mllvm", "-enable-misched=false"],
    "bwd_col_pipe_tangent.hip": ["-mllvm", "-enable-misched=false"],
    "bwd_row_pipe_qknorm.hip": ["-mllvm", "-enable-misched=false"],
    "bwd_col_pipe_qknorm.hip": ["-mllvm", "-enable-misched=false"],
    # (its unrolled phases exceed the default size limit of "#pragma unroll": a loop left rolled would index
    # register arrays at run time)
    "bwd_pass.hip": ["-mllvm", "-enable-misched=false", "-mllvm", "-pragma-unroll-threshold=262144"],
}


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build(verbose=False, extra=(), jobs=None):
    srcs = sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))
    jobs = jobs or min(8, os.cpu_count() or 1, len(srcs))
    with tempfile.TemporaryDirectory() as tmp:
        def compile_one(src):
            name = os.path.basename(src)
            obj = os.path.join(tmp, name + ".o")
            _run(["hipcc", *COMMON, *PER_FILE.get(name, []), *extra, "-c", src, "-o", obj], verbose)
            return obj

        with ThreadPoolExecutor(max_workers=jobs) as pool:  # one hipcc process per translation unit
            objs = list(pool.map(compile_one, srcs))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], verbose)
    _run(["hipcc", *COMMON, "-shared", os.path.join(HERE, "peaks", "peaks.hip"), "-o", PEAKS_LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
