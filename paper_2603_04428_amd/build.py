"""Compile libq4kv.so (hand-written HIP for gfx950 + the C ABI) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libq4kv.so")
SOURCES = ["api.hip", "codec.hip", "decode_attention.hip", "chunk_attention.hip", "mla_decode.hip", "read_probe.hip", "persist.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# No fast-math anywhere: the quantizer needs IEEE binary32 division and rounding.
# packed-fp32 instruction selection is switched off (its forms have been unreliable on the test machines).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-gpu-sanitize"]


def build(verbose=False):
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = [HIPCC] + FLAGS + ["-o", LIB] + srcs
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose="-v" in sys.argv))
