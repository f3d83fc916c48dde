"""Compile libq4kv.so (hand-written HIP for gfx950 + the C ABI) in-tree with hipcc."""
import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libq4kv.so")
SOURCES = ["api.hip", "codec.hip", "decode_attention.hip", "chunk_attention.hip", "mla_decode.hip", "read_probe.hip", "persist.hip", "block_pool.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# No fast-math anywhere: the quantizer needs IEEE binary32 division and rounding.
# packed-fp32 instruction selection is switched off (its forms have been unreliable on the test machines).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-gpu-sanitize"]
# The chunk kernel reads most of its matrix results with vector instructions (scales, softmax), so its matrix
# instructions write vector registers directly instead of accumulator registers that must be copied out first.
FILE_FLAGS = {"chunk_attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def build(verbose=False):
    with tempfile.TemporaryDirectory(prefix="q4kv_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            cmd = [HIPCC] + FLAGS + FILE_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd))
            subprocess.check_call(cmd)
            return obj
        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-sanitize", "-o", LIB] + objs
        if verbose:
            print(" ".join(cmd))
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv))
