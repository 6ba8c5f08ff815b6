"""Compile libtrdq.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtrdq.so")

SOURCES = ["api.cpp", "rotate_quant.hip", "rotate_quant_wide.hip", "rotate_quant_rpr.hip", "calibrate.hip", "greedy_rotation.hip", "rotate_quant_dense.hip", "attention_share.hip", "prepare_weights.hip", "qgemm.hip", "qgemm_dma.hip", "qgemm_wide.hip", "qgemm_tiled.hip", "fused.hip", "peaks.hip"]

# packed-FP32 instructions are switched off for every device compile
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-inline-asm", "-I", CSRC, "-I", INCLUDE]


# per-source extra flags: keep the matrix-instruction accumulators of the pipelined product kernel
# in ordinary VGPRs (no accumulator-register copies around the loop)
SOURCE_FLAGS = {"qgemm_dma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
                "qgemm_tiled.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
                # ... and have the first kernel arguments delivered in registers at wave launch instead
                # of fetched by the kernel's first instructions (a fraction of a microsecond per launch)
                "rotate_quant.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-mllvm", "-amdgpu-kernarg-preload-count=16"],
                "rotate_quant_rpr.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"],
                "calibrate.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile(src, extra, obj_dir):
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *FLAGS, *SOURCE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    return obj, out


def build(verbose=False, extra=(), lib=None, obj_dir=None):
    """Compiles every source and links the library; lib / obj_dir name another output (a build with
    extra preprocessor switches, e.g. the phase probe) beside the default one."""
    lib = lib or LIB
    obj_dir = obj_dir or OBJ_DIR
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(lambda s: _compile(s, list(extra), obj_dir), SOURCES))
    if verbose:
        for _, out in results:
            if out:
                print(out)
    objs = [o for o, _ in results]
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib, *objs]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
