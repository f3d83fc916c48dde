"""The quantize kernels take scale = fl((max - min) / 15) (Sec. 3.2) without a division: a multiply by fl(1/15)
and two fused multiply-adds.  This host test checks, value by value in C, that the sequence equals the IEEE
binary32 division on the whole range the kernels can meet: max - min of two finite binary16 numbers, rounded
to binary32, is 0 or lies in [2^-24, 2^17]."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def _has_fma():
    try:
        return " fma " in open("/proc/cpuinfo").read()
    except OSError:
        return False


def test_multiply_and_two_fmas_equal_division_by_15(tmp_path):
    exe = str(tmp_path / "div15_check")
    flags = ["-O2", "-ffp-contract=off"] + (["-mfma"] if _has_fma() else [])
    subprocess.run(["gcc", *flags, "-o", exe, os.path.join(HERE, "host_c", "div15_check.c"), "-lm"], check=True)
    # with hardware FMA the whole range takes about a second; the software fmaf is slow, so three binades then
    # (the sequence is invariant under scaling by 2 away from overflow and underflow)
    ranges = [("-24", "17")] if _has_fma() else [("-24", "-23"), ("0", "1"), ("16", "17")]
    for lo, hi in ranges:
        out = subprocess.run([exe, lo, hi], capture_output=True, text=True)
        assert out.returncode == 0, out.stdout
        words = out.stdout.split()
        assert int(words[words.index("mismatches") + 1]) == 0
        # the plain product fl(r * fl(1/15)) alone is wrong for most r: the two corrections are what is tested
        assert int(words[words.index("plain_multiply_mismatches") + 1]) > int(words[words.index("checked") + 1]) // 4


def test_small_quotients_by_reciprocal_multiplication():
    """The append kernel finds a lane's row and head with floor((n + 0.5) * fl(1 / d)) in binary32 instead of an
    integer division (n: a few groups or chunk tokens past the wave's start, d: groups per row or chunk length).
    That equals n // d for every n below 2^21, the range the library admits (chunk_len <= 2^20)."""
    import numpy as np
    n = np.arange(0, 1 << 21, dtype=np.int64)
    nf = n.astype(np.float32) + np.float32(0.5)
    for d in [1, 2, 3, 4, 5, 7, 8, 9, 10, 16, 63, 64, 65, 100, 511, 512, 513, 1000, 4095, 4096, 65535, 65536,
              (1 << 20) - 1, 1 << 20]:
        inv = np.float32(1.0) / np.float32(d)
        got = np.floor(nf * inv).astype(np.int64)
        assert np.array_equal(got, n // d), d
