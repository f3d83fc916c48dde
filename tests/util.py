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


def tie_adjacent_rows(seed=7):
    """float16 [rows][64]: groups whose quotients (x - min) / scale sit on, just below and just above k + 0.5 for
    every code k and many scales (normal and subnormal binary16, mostly not powers of two).  Input construction
    only: which code each element gets is for the quantizer under test to say."""
    F16 = np.float16
    rng = np.random.default_rng(seed)
    rows = []
    scales = np.concatenate([rng.uniform(0.01, 4.0, 300), 2.0 ** rng.integers(-20, 3, 60).astype(np.float64),
                             rng.uniform(1, 60, 60) * 2.0 ** -24])
    for sc in scales:
        s16 = float(F16(sc))
        if s16 == 0.0:
            continue
        base = float(F16(rng.uniform(-3, 3))) if sc > 1e-4 else 0.0
        g = np.empty(64)
        g[0], g[1] = base, base + 15 * s16
        k = rng.integers(0, 15, 62) + 0.5
        g[2:] = base + k * s16
        x16 = g.astype(F16)
        # neighbours in binary16 of the tie points, in both directions
        nb = x16.copy().view(np.uint16)
        step = rng.integers(-2, 3, 64).astype(np.int32)
        step[:2] = 0
        nb = (nb.astype(np.int32) + step).clip(0, 0xFBFF).astype(np.uint16)
        rows.append(x16)
        rows.append(nb.view(F16))
    x = np.stack(rows)
    return x[np.isfinite(x.astype(np.float32)).all(axis=1)]


def tie_adjacent_rows_bf16(seed=8):
    """The same construction with scales and group minima that bfloat16 holds exactly (rounded with torch's
    bfloat16, a library type), for the parameter format that stores both as bfloat16."""
    import torch
    F16 = np.float16
    rng = np.random.default_rng(seed)
    bf = lambda v: float(torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).to(torch.float32))
    rows = []
    for _ in range(400):
        s = bf(rng.uniform(0.01, 4.0))
        base = bf(rng.uniform(-3, 3))
        g = np.empty(64)
        g[0], g[1] = base, base + 15 * s
        g[2:] = base + (rng.integers(0, 15, 62) + 0.5) * s
        x16 = g.astype(F16)
        nb = x16.copy().view(np.uint16).astype(np.int32)
        step = rng.integers(-2, 3, 64)
        step[:2] = 0
        rows.append(x16)
        rows.append((nb + step).clip(0, 0xFBFF).astype(np.uint16).view(F16))
    x = np.stack(rows)
    return x[np.isfinite(x.astype(np.float32)).all(axis=1)]
