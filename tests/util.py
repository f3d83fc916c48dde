"""Small helpers shared by the tests (no method arithmetic from either side)."""
import numpy as np


def read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            k, v = line.split()
            out[k] = float(v) if "." in v else int(v)
    return out


def unpack_codes(words):
    """uint32 [..., W] -> uint8 [..., 8W]; element d = word d//8, bits 4*(d%8).. (low nibble first)."""
    w = np.asarray(words, np.uint32)
    shifts = (4 * np.arange(8, dtype=np.uint32))
    c = (w[..., None] >> shifts) & np.uint32(0xF)
    return c.reshape(w.shape[:-1] + (w.shape[-1] * 8,)).astype(np.uint8)


def within_tol(got, want, atol=2e-3, rtol=2e-3):
    """|got - want| <= atol + rtol*|want| element-wise (the stated fp16 attention tolerance)."""
    g = np.asarray(got, np.float64)
    w = np.asarray(want, np.float64)
    err = np.abs(g - w)
    lim = atol + rtol * np.abs(w)
    return bool(np.all(err <= lim)), float(np.max(err - lim)), float(np.max(err))
