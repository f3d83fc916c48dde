"""CPU oracle for the Q4 KV-cache hot path -- TEST INFRASTRUCTURE ONLY.

Thin numpy/ctypes access to oracle/q4kv_oracle.c.  Only tests, the smoke check and
the benchmark's cpu_baseline leg may import this package; the GPU library never does.
All arrays are host numpy arrays; binary16 data travels as uint16 bit patterns or
as numpy float16 (viewed, never converted by this wrapper).
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build as _build_oracle

GROUP = 64

_lib = None


class Spec(C.Structure):
    """Mirror of oracle_spec (the ModelCacheSpec of Sec. 3.1/3.6)."""
    _fields_ = [("num_layers", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("k_dim", C.c_int32), ("v_dim", C.c_int32), ("v_aliases_k", C.c_int32),
                ("block_tokens", C.c_int32), ("group_size", C.c_int32), ("param_format", C.c_int32)]


class _Pool(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scale", C.c_void_p), ("bias", C.c_void_p), ("num_blocks", C.c_int32)]


def lib():
    global _lib
    if _lib is None:
        _build_oracle(force=False)
        _lib = C.CDLL(LIB)
        _lib.oracle_h2f.restype = C.c_float
        _lib.oracle_h2f.argtypes = [C.c_uint16]
        _lib.oracle_d2h.restype = C.c_uint16
        _lib.oracle_d2h.argtypes = [C.c_double]
        _lib.oracle_f2h.restype = C.c_uint16
        _lib.oracle_f2h.argtypes = [C.c_float]
        for f in (_lib.oracle_fp16_layer_bytes, _lib.oracle_q4_layer_bytes):
            f.restype = C.c_int64
            f.argtypes = [C.c_int64] * 4
        _lib.oracle_bf2f.restype = C.c_float
        _lib.oracle_bf2f.argtypes = [C.c_uint16]
        _lib.oracle_f2bf.restype = C.c_uint16
        _lib.oracle_f2bf.argtypes = [C.c_float]
        _lib.oracle_q4_quantize_fmt.argtypes = [C.c_void_p, C.c_int64, C.c_int, C.c_int, C.c_void_p, C.c_void_p,
                                                C.c_void_p]
        _lib.oracle_q4_dequantize_fmt.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int,
                                                  C.c_void_p]
        _lib.oracle_append.argtypes = [C.POINTER(Spec), C.POINTER(_Pool), C.POINTER(_Pool), C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]
        _lib.oracle_attention.argtypes = [C.POINTER(Spec), C.POINTER(_Pool), C.POINTER(_Pool), C.c_void_p,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_int,
                                          C.c_int, C.c_float, C.c_int, C.c_void_p, C.c_int, C.c_int,
                                          C.POINTER(C.c_int)]
        _lib.oracle_attention_probs.argtypes = [C.POINTER(Spec), C.POINTER(_Pool), C.POINTER(_Pool), C.c_int,
                                                C.c_void_p, C.c_int, C.c_void_p, C.c_int, C.c_int, C.c_float,
                                                C.c_void_p, C.c_void_p]
        _lib.oracle_max_threads.restype = C.c_int
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _bits(x):
    """float16 or uint16 array -> contiguous uint16 view."""
    x = np.ascontiguousarray(x)
    if x.dtype == np.float16:
        return x.view(np.uint16)
    assert x.dtype == np.uint16, x.dtype
    return x


F16_PARAMS, BF16_PARAMS = 0, 1   # type of the stored scale and bias (Sec. 3.1, appendix "safetensors Q4 Format")


def make_spec(num_layers, num_q_heads, num_kv_heads, k_dim, v_dim=None, v_aliases_k=False, block_tokens=256,
              param_format=F16_PARAMS):
    return Spec(num_layers, num_q_heads, num_kv_heads, k_dim, k_dim if v_dim is None else v_dim,
                1 if v_aliases_k else 0, block_tokens, GROUP, param_format)


class Pool:
    """One paged Q4 pool on the host: [layers][blocks][kv_heads][block_tokens][dim/8 | dim/64]."""

    def __init__(self, spec, dim, num_blocks, fill=None):
        shp = (spec.num_layers, num_blocks, spec.num_kv_heads, spec.block_tokens)
        self.dim = dim
        self.num_blocks = num_blocks
        self.codes = np.zeros(shp + (dim // 8,), np.uint32)
        self.scale = np.zeros(shp + (dim // GROUP,), np.uint16)
        self.bias = np.zeros(shp + (dim // GROUP,), np.uint16)
        if fill is not None:           # poison: every slot decodes to NaN until overwritten
            self.codes[...] = 0xFFFFFFFF
            self.scale[...] = fill
            self.bias[...] = fill

    def c(self):
        return _Pool(_ptr(self.codes), _ptr(self.scale), _ptr(self.bias), self.num_blocks)


def h2f(bits):
    return float(lib().oracle_h2f(int(bits)))


def d2h(x):
    return int(lib().oracle_d2h(float(x)))


def f2h(x):
    return int(lib().oracle_f2h(float(np.float32(x))))


def bf2f(bits):
    return float(lib().oracle_bf2f(int(bits)))


def f2bf(x):
    return int(lib().oracle_f2bf(float(np.float32(x))))


def fp16_layer_bytes(kv_heads, k_dim, v_dim, tokens):
    return int(lib().oracle_fp16_layer_bytes(kv_heads, k_dim, v_dim, tokens))


def q4_layer_bytes(kv_heads, k_dim, v_dim, tokens):
    return int(lib().oracle_q4_layer_bytes(kv_heads, k_dim, v_dim, tokens))


def quantize(x, param_format=F16_PARAMS):
    """x: [..., dim] float16/uint16 -> (codes uint32 [..., dim/8], scale uint16 [..., dim/64], bias same).
    scale / bias are bit patterns of binary16 or, with param_format=BF16_PARAMS, of bfloat16."""
    xb = _bits(x)
    dim = xb.shape[-1]
    rows = xb.size // dim if dim else 0
    lead = xb.shape[:-1]
    codes = np.empty(lead + (dim // 8,), np.uint32)
    scale = np.empty(lead + (dim // GROUP,), np.uint16)
    bias = np.empty(lead + (dim // GROUP,), np.uint16)
    rc = lib().oracle_q4_quantize_fmt(_ptr(xb), rows, dim, int(param_format), _ptr(codes), _ptr(scale), _ptr(bias))
    if rc:
        raise ValueError(f"oracle_q4_quantize_fmt rc={rc}")
    return codes, scale, bias


def dequantize(codes, scale, bias, param_format=F16_PARAMS):
    """Inverse layout of quantize(); returns float16 [..., dim]."""
    codes = np.ascontiguousarray(codes, np.uint32)
    scale, bias = _bits(scale), _bits(bias)
    dim = codes.shape[-1] * 8
    rows = codes.size // codes.shape[-1] if codes.shape[-1] else 0
    out = np.empty(codes.shape[:-1] + (dim,), np.uint16)
    rc = lib().oracle_q4_dequantize_fmt(_ptr(codes), _ptr(scale), _ptr(bias), rows, dim, int(param_format), _ptr(out))
    if rc:
        raise ValueError(f"oracle_q4_dequantize_fmt rc={rc}")
    return out.view(np.float16)


def append(spec, kpool, vpool, k_new, v_new, block_table, seq_len_before, layer_begin=0, layer_end=None):
    """k_new/v_new: [layers_in_call][A][C][kv_heads][dim] float16.  Writes into the pools in place."""
    layer_end = spec.num_layers if layer_end is None else layer_end
    kb = _bits(k_new)
    vb = None if spec.v_aliases_k else _bits(v_new)
    bt = np.ascontiguousarray(block_table, np.int32)
    sl = np.ascontiguousarray(seq_len_before, np.int32)
    A, C_ = kb.shape[1], kb.shape[2]
    kp = kpool.c()
    vp = kp if spec.v_aliases_k else vpool.c()
    rc = lib().oracle_append(C.byref(spec), C.byref(kp), C.byref(vp), _ptr(kb), _ptr(vb), _ptr(bt), bt.shape[1],
                             _ptr(sl), A, C_, layer_begin, layer_end)
    if rc:
        raise ValueError(f"oracle_append rc={rc}")


def attention(spec, kpool, vpool, q, block_table, seq_len, sm_scale, window=0, window_per_layer=None,
              layer_begin=0, layer_end=None, return_f64=False, return_threads=False):
    """q: [layers_in_call][A][q_len][q_heads][k_dim] float16 -> float16 of the same leading shape, v_dim wide."""
    layer_end = spec.num_layers if layer_end is None else layer_end
    qb = _bits(q)
    Lr, A, q_len, Hq, _ = qb.shape
    assert Lr == layer_end - layer_begin and Hq == spec.num_q_heads
    bt = np.ascontiguousarray(block_table, np.int32)
    sl = np.ascontiguousarray(seq_len, np.int32)
    out = np.zeros((Lr, A, q_len, Hq, spec.v_dim), np.uint16)
    out_d = np.zeros(out.shape, np.float64) if return_f64 else None
    wpl = None if window_per_layer is None else np.ascontiguousarray(window_per_layer, np.int32)
    kp = kpool.c()
    vp = kp if spec.v_aliases_k else vpool.c()
    used = C.c_int(0)
    rc = lib().oracle_attention(C.byref(spec), C.byref(kp), C.byref(vp), _ptr(qb), _ptr(out), _ptr(out_d), _ptr(bt),
                                bt.shape[1], _ptr(sl), A, q_len, float(sm_scale), int(window), _ptr(wpl),
                                layer_begin, layer_end, C.byref(used))
    if rc:
        raise ValueError(f"oracle_attention rc={rc}")
    res = [out.view(np.float16)]
    if return_f64:
        res.append(out_d)
    if return_threads:
        res.append(used.value)
    return res[0] if len(res) == 1 else tuple(res)


def attention_probs(spec, kpool, vpool, layer, table_row, kv_head, q_row, vis, sm_scale, window=0):
    """Softmax weights p[0..vis) and the binary64 output of one (layer, agent, row, head) unit."""
    tr = np.ascontiguousarray(table_row, np.int32)
    qb = _bits(q_row)
    p = np.zeros(max(vis, 1), np.float64)
    o = np.zeros(spec.v_dim, np.float64)
    kp = kpool.c()
    vp = kp if spec.v_aliases_k else vpool.c()
    rc = lib().oracle_attention_probs(C.byref(spec), C.byref(kp), C.byref(vp), layer, _ptr(tr), kv_head, _ptr(qb),
                                      vis, int(window), float(sm_scale), _ptr(p), _ptr(o))
    if rc:
        raise ValueError(f"oracle_attention_probs rc={rc}")
    return p[:vis], o


def max_threads():
    return int(lib().oracle_max_threads())
