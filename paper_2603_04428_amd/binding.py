"""ctypes binding of libq4kv.so: the same entry points as include/q4kv.h, taking torch tensors.

Argument marshalling only -- pointers, sizes and the current HIP stream are handed to the C ABI;
every step of the path runs in the library's kernels.  There is no fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libq4kv.so")

EXPORTS = ["q4kv_quantize", "q4kv_dequantize", "q4kv_quantize_fmt", "q4kv_dequantize_fmt", "q4kv_append", "q4kv_batched_attention",
           "q4kv_batched_attention_windows", "q4kv_batched_attention_static", "q4kv_decode_plan",
           "q4kv_batched_attention_planned", "q4kv_attention_workspace_bytes", "q4kv_default_split_tokens", "q4kv_cache_bytes", "q4kv_block_image_bytes", "q4kv_export_blocks", "q4kv_import_blocks", "q4kv_read_probe",
           "q4kv_block_pool_create", "q4kv_block_pool_destroy", "q4kv_block_pool_reserve", "q4kv_block_pool_release",
           "q4kv_block_pool_blocks", "q4kv_block_pool_table_row", "q4kv_block_pool_touch", "q4kv_block_pool_pin",
           "q4kv_block_pool_lru_victim", "q4kv_block_pool_free_blocks", "q4kv_block_pool_owner",
           "q4kv_last_error",
           "q4kv_version"]


class Q4KVError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libq4kv error {code}: {msg}")
        self.code = code


class Spec(C.Structure):
    """q4kv_spec"""
    _fields_ = [("num_layers", C.c_int32), ("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32),
                ("k_dim", C.c_int32), ("v_dim", C.c_int32), ("v_aliases_k", C.c_int32),
                ("block_tokens", C.c_int32), ("group_size", C.c_int32), ("param_format", C.c_int32)]


PARAMS_F16, PARAMS_BF16 = 0, 1   # q4kv_param_format: type of the stored scale and bias


class _CPool(C.Structure):
    """q4kv_pool"""
    _fields_ = [("codes", C.c_void_p), ("scale", C.c_void_p), ("bias", C.c_void_p), ("num_blocks", C.c_int32)]


_lib = None


def lib():
    """Load libq4kv.so (built in-tree by paper_2603_04428_amd/build.py); raise if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(there is no fallback path)")
        l = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        l.q4kv_quantize.argtypes = [vp, i64, i32, vp, vp, vp, vp]
        l.q4kv_dequantize.argtypes = [vp, vp, vp, i64, i32, vp, vp]
        l.q4kv_quantize_fmt.argtypes = [vp, i64, i32, i32, vp, vp, vp, vp]
        l.q4kv_dequantize_fmt.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp]
        l.q4kv_append.argtypes = [C.POINTER(Spec), C.POINTER(_CPool), C.POINTER(_CPool), vp, vp, vp, i32, vp, i32, i32,
                                  i32, i32, vp]
        l.q4kv_batched_attention.argtypes = [C.POINTER(Spec), C.POINTER(_CPool), C.POINTER(_CPool), vp, vp, vp, i32, vp,
                                             i32, i32, i32, C.c_float, i32, i32, i32, i32, vp, C.c_size_t, vp]
        l.q4kv_batched_attention_windows.argtypes = [C.POINTER(Spec), C.POINTER(_CPool), C.POINTER(_CPool), vp, vp, vp,
                                                     i32, vp, i32, i32, i32, C.c_float, C.POINTER(i32), i32, i32, i32,
                                                     vp, C.c_size_t, vp]
        l.q4kv_batched_attention_static.argtypes = [C.POINTER(Spec), C.POINTER(_CPool), C.POINTER(_CPool), vp, vp, vp, i32,
                                                    vp, i32, i32, i32, C.c_float, i32, i32, i32, i32, vp]
        l.q4kv_decode_plan.argtypes = [C.POINTER(Spec), vp, i32, i32, i32, i32, i32, vp, C.c_size_t, vp]
        l.q4kv_batched_attention_planned.argtypes = [C.POINTER(Spec), C.POINTER(_CPool), C.POINTER(_CPool), vp, vp, vp, i32,
                                                     i32, i32, C.c_float, i32, i32, i32, i32, vp, C.c_size_t, vp]
        l.q4kv_attention_workspace_bytes.restype = C.c_size_t
        l.q4kv_attention_workspace_bytes.argtypes = [C.POINTER(Spec), i32, i32, i32, i32, i32]
        l.q4kv_default_split_tokens.restype = i32
        l.q4kv_default_split_tokens.argtypes = [C.POINTER(Spec), i32, i32, i32, i32]
        l.q4kv_cache_bytes.restype = i64
        l.q4kv_cache_bytes.argtypes = [C.POINTER(Spec), i64]
        l.q4kv_read_probe.argtypes = [vp, C.c_size_t, vp, vp]
        l.q4kv_block_image_bytes.restype = C.c_size_t
        l.q4kv_block_image_bytes.argtypes = [C.POINTER(Spec), i32]
        for f in (l.q4kv_export_blocks, l.q4kv_import_blocks):
            f.argtypes = [C.POINTER(Spec), C.POINTER(_CPool), C.POINTER(_CPool), vp, i32, vp, C.c_size_t, vp]
        l.q4kv_block_pool_create.restype = vp
        l.q4kv_block_pool_create.argtypes = [i32]
        l.q4kv_block_pool_destroy.restype = None
        l.q4kv_block_pool_destroy.argtypes = [vp]
        l.q4kv_block_pool_reserve.argtypes = [vp, i64, i64]
        l.q4kv_block_pool_release.argtypes = [vp, i64]
        l.q4kv_block_pool_blocks.argtypes = [vp, i64, C.POINTER(i32), i32]
        l.q4kv_block_pool_table_row.argtypes = [vp, i64, C.POINTER(i32), i32, i32]
        l.q4kv_block_pool_touch.argtypes = [vp, i64]
        l.q4kv_block_pool_pin.argtypes = [vp, i64, i32]
        l.q4kv_block_pool_lru_victim.restype = i64
        l.q4kv_block_pool_lru_victim.argtypes = [vp]
        l.q4kv_block_pool_free_blocks.argtypes = [vp]
        l.q4kv_block_pool_owner.restype = i64
        l.q4kv_block_pool_owner.argtypes = [vp, i32]
        l.q4kv_last_error.restype = C.c_char_p
        l.q4kv_version.restype = C.c_int
        _lib = l
    return _lib


def _check(rc):
    if rc != 0:
        raise Q4KVError(rc, lib().q4kv_last_error().decode())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    if t is None:
        return None
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU, got {t.dtype} on {t.device}")
    return C.c_void_p(t.data_ptr())


def make_spec(num_layers, num_q_heads, num_kv_heads, k_dim, v_dim=None, v_aliases_k=False, block_tokens=256,
              param_format=PARAMS_F16):
    return Spec(num_layers, num_q_heads, num_kv_heads, k_dim, k_dim if v_dim is None else v_dim,
                1 if v_aliases_k else 0, block_tokens, 64, param_format)


class Pool:
    """Device arrays of one paged Q4 pool: [layers][blocks][kv_heads][256][dim/8 | dim/64]."""

    def __init__(self, spec, dim, num_blocks, device="cuda", poison=False):
        shp = (spec.num_layers, num_blocks, spec.num_kv_heads, spec.block_tokens)
        self.dim, self.num_blocks = dim, num_blocks
        # torch has no uint32/uint16 arithmetic, and none is needed: int32 / int16 storage of the same bits
        self.codes = torch.zeros(shp + (dim // 8,), dtype=torch.int32, device=device)
        self.scale = torch.zeros(shp + (dim // 64,), dtype=torch.int16, device=device)
        self.bias = torch.zeros(shp + (dim // 64,), dtype=torch.int16, device=device)
        if poison:                      # every slot decodes to NaN until it is written
            nan_bits = 0x7FC0 if spec.param_format == PARAMS_BF16 else 0x7E00
            self.codes.fill_(-1)
            self.scale.fill_(nan_bits)
            self.bias.fill_(nan_bits)

    def c(self):
        return _CPool(self.codes.data_ptr(), self.scale.data_ptr(), self.bias.data_ptr(), self.num_blocks)


class BlockPool:
    """q4kv_block_pool: host-side bookkeeping of block ownership (Sec. 3.1).  Marshalling only."""
    ENOSPACE = -6

    def __init__(self, num_blocks):
        self._h = lib().q4kv_block_pool_create(num_blocks)
        if not self._h:
            raise ValueError("q4kv_block_pool_create failed")

    def close(self):
        if self._h:
            lib().q4kv_block_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    @staticmethod
    def _ok(rc):
        if rc < 0:
            raise Q4KVError(rc, "block pool: " + {-1: "bad argument or unknown agent", -3: "more blocks than the row holds",
                                                  -6: "not enough free blocks"}.get(rc, "error"))
        return rc

    def reserve(self, agent_id, tokens):
        return self._ok(lib().q4kv_block_pool_reserve(self._h, agent_id, tokens))

    def release(self, agent_id):
        return self._ok(lib().q4kv_block_pool_release(self._h, agent_id))

    def blocks(self, agent_id):
        n = self._ok(lib().q4kv_block_pool_blocks(self._h, agent_id, None, 0))
        ids = (C.c_int32 * max(n, 1))()
        self._ok(lib().q4kv_block_pool_blocks(self._h, agent_id, ids, n))
        return list(ids[:n])

    def table_row(self, agent_id, max_blocks, fill=-1):
        row = (C.c_int32 * max_blocks)()
        self._ok(lib().q4kv_block_pool_table_row(self._h, agent_id, row, max_blocks, fill))
        return list(row)

    def touch(self, agent_id):
        self._ok(lib().q4kv_block_pool_touch(self._h, agent_id))

    def pin(self, agent_id, pinned=True):
        self._ok(lib().q4kv_block_pool_pin(self._h, agent_id, 1 if pinned else 0))

    def lru_victim(self):
        return lib().q4kv_block_pool_lru_victim(self._h)

    def free_blocks(self):
        return lib().q4kv_block_pool_free_blocks(self._h)

    def owner(self, block_id):
        return lib().q4kv_block_pool_owner(self._h, block_id)


def q4kv_version():
    return lib().q4kv_version()


def q4kv_cache_bytes(spec, tokens):
    r = lib().q4kv_cache_bytes(C.byref(spec), tokens)
    if r < 0:
        _check(-1)
    return r


def q4kv_block_image_bytes(spec, num_blocks):
    return lib().q4kv_block_image_bytes(C.byref(spec), num_blocks)


def _image_call(fn, spec, kpool, vpool, block_ids, image):
    """block_ids: int32 tensor on the GPU; image: uint8 tensor on the GPU or in pinned host memory."""
    if not (image.dtype == torch.uint8 and image.is_contiguous() and (image.is_cuda or image.is_pinned())):
        raise ValueError("image: contiguous uint8 tensor on the GPU or in pinned host memory")
    kp = kpool.c()
    vp = None if spec.v_aliases_k else vpool.c()
    _check(fn(C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp), _dev(block_ids, torch.int32, "block_ids"),
              block_ids.numel(), C.c_void_p(image.data_ptr()), image.numel(), _stream()))


def q4kv_export_blocks(spec, kpool, vpool, block_ids, image=None):
    """Gather the listed blocks of every layer into a block image (see include/q4kv.h); returns the image."""
    if image is None:
        image = torch.empty(q4kv_block_image_bytes(spec, block_ids.numel()), dtype=torch.uint8, device=block_ids.device)
    _image_call(lib().q4kv_export_blocks, spec, kpool, vpool, block_ids, image)
    return image


def q4kv_import_blocks(spec, kpool, vpool, block_ids, image):
    """Scatter a block image into the listed blocks of every layer."""
    _image_call(lib().q4kv_import_blocks, spec, kpool, vpool, block_ids, image)


def q4kv_read_probe(buf, sink):
    """Measurement helper: read the contiguous GPU tensor `buf` once (nothing is written); sink: int32 [1] on the GPU."""
    if not (buf.is_cuda and buf.is_contiguous() and sink.is_cuda and sink.numel() >= 1 and sink.element_size() == 4):
        raise ValueError("q4kv_read_probe: contiguous GPU tensors, sink of at least one 4-byte element")
    _check(lib().q4kv_read_probe(C.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(), C.c_void_p(sink.data_ptr()),
                                 _stream()))


def q4kv_quantize(x, codes=None, scale=None, bias=None, param_format=None):
    """x: fp16 [..., dim] on the GPU -> (codes int32 [..., dim/8], scale int16 [..., dim/64], bias same).
    param_format None: q4kv_quantize; PARAMS_F16 / PARAMS_BF16: q4kv_quantize_fmt."""
    dim = x.shape[-1]
    rows = x.numel() // dim if dim else 0
    lead = tuple(x.shape[:-1])
    if codes is None:
        codes = torch.empty(lead + (dim // 8,), dtype=torch.int32, device=x.device)
        scale = torch.empty(lead + (dim // 64,), dtype=torch.int16, device=x.device)
        bias = torch.empty(lead + (dim // 64,), dtype=torch.int16, device=x.device)
    outs = (_dev(codes, torch.int32, "codes"), _dev(scale, torch.int16, "scale"), _dev(bias, torch.int16, "bias"))
    if param_format is None:
        _check(lib().q4kv_quantize(_dev(x, torch.float16, "x"), rows, dim, *outs, _stream()))
    else:
        _check(lib().q4kv_quantize_fmt(_dev(x, torch.float16, "x"), rows, dim, int(param_format), *outs, _stream()))
    return codes, scale, bias


def q4kv_dequantize(codes, scale, bias, out=None, param_format=None):
    dim = codes.shape[-1] * 8
    rows = codes.numel() // codes.shape[-1] if codes.shape[-1] else 0
    if out is None:
        out = torch.empty(tuple(codes.shape[:-1]) + (dim,), dtype=torch.float16, device=codes.device)
    ins = (_dev(codes, torch.int32, "codes"), _dev(scale, torch.int16, "scale"), _dev(bias, torch.int16, "bias"))
    if param_format is None:
        _check(lib().q4kv_dequantize(*ins, rows, dim, _dev(out, torch.float16, "out"), _stream()))
    else:
        _check(lib().q4kv_dequantize_fmt(*ins, rows, dim, int(param_format), _dev(out, torch.float16, "out"), _stream()))
    return out


def q4kv_append(spec, kpool, vpool, k_new, v_new, block_table, seq_len_before, layer_begin=0, layer_end=None):
    """k_new / v_new: fp16 [layers_in_call][A][C][kv_heads][dim]; block_table int32 [A][max_blocks] (device)."""
    layer_end = spec.num_layers if layer_end is None else layer_end
    A, Cn = k_new.shape[1], k_new.shape[2]
    kp = kpool.c()
    vp = None if spec.v_aliases_k else vpool.c()
    _check(lib().q4kv_append(C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp),
                             _dev(k_new, torch.float16, "k_new"), _dev(v_new, torch.float16, "v_new"),
                             _dev(block_table, torch.int32, "block_table"), block_table.shape[1],
                             _dev(seq_len_before, torch.int32, "seq_len_before"), A, Cn, layer_begin, layer_end,
                             _stream()))


def q4kv_default_split_tokens(spec, num_agents, q_len, max_seq_len, layers_in_call):
    return lib().q4kv_default_split_tokens(C.byref(spec), num_agents, q_len, max_seq_len, layers_in_call)


def q4kv_attention_workspace_bytes(spec, num_agents, q_len, max_seq_len, split_tokens, layers_in_call):
    return lib().q4kv_attention_workspace_bytes(C.byref(spec), num_agents, q_len, max_seq_len, split_tokens,
                                                layers_in_call)


def q4kv_batched_attention(spec, kpool, vpool, q, block_table, seq_len, max_seq_len, sm_scale, window=0,
                           split_tokens=0, layer_begin=0, layer_end=None, out=None, workspace=None):
    """q: fp16 [layers_in_call][A][q_len][q_heads][k_dim] -> fp16 out of the same leading shape, v_dim wide.
    window: one int for all layers, or a sequence with one window per layer of the call (q4kv_batched_attention_windows)."""
    layer_end = spec.num_layers if layer_end is None else layer_end
    Lr, A, q_len = q.shape[0], q.shape[1], q.shape[2]
    if out is None:
        out = torch.empty((Lr, A, q_len, spec.num_q_heads, spec.v_dim), dtype=torch.float16, device=q.device)
    need = q4kv_attention_workspace_bytes(spec, max(A, 1), q_len, max_seq_len, split_tokens, max(Lr, 1))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    kp = kpool.c()
    vp = None if spec.v_aliases_k else vpool.c()
    common = (C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp),
              _dev(q, torch.float16, "q"), _dev(out, torch.float16, "out"),
              _dev(block_table, torch.int32, "block_table"), block_table.shape[1],
              _dev(seq_len, torch.int32, "seq_len"), A, q_len, max_seq_len, float(sm_scale))
    tail = (int(split_tokens), layer_begin, layer_end, C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream())
    if isinstance(window, (list, tuple)) or hasattr(window, "__len__"):      # one window per layer of the call (host)
        if len(window) != layer_end - layer_begin:
            raise ValueError(f"{len(window)} windows for {layer_end - layer_begin} layers")
        windows = (C.c_int32 * len(window))(*[int(x) for x in window])
        _check(lib().q4kv_batched_attention_windows(*common, windows, *tail))
    else:
        _check(lib().q4kv_batched_attention(*common, int(window), *tail))
    return out


STATIC_SCRATCH_BYTES = 16 << 20   # Q4KV_STATIC_SCRATCH_BYTES


def q4kv_batched_attention_static(spec, kpool, vpool, q, out, block_table, seq_len, max_seq_len, sm_scale, window=0,
                                  split_tokens=0, layer_begin=0, layer_end=None):
    """q4kv_batched_attention_static: the decode path's workspace comes from the library's fixed per-GPU array.
    Allocates no tensor: `out` (fp16 [layers_in_call][A][q_len][q_heads][v_dim]) is the caller's."""
    layer_end = spec.num_layers if layer_end is None else layer_end
    kp = kpool.c()
    vp = None if spec.v_aliases_k else vpool.c()
    _check(lib().q4kv_batched_attention_static(
        C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp), _dev(q, torch.float16, "q"),
        _dev(out, torch.float16, "out"), _dev(block_table, torch.int32, "block_table"), block_table.shape[1],
        _dev(seq_len, torch.int32, "seq_len"), q.shape[1], q.shape[2], max_seq_len, float(sm_scale), int(window),
        int(split_tokens), layer_begin, layer_end, _stream()))
    return out


def q4kv_decode_plan(spec, seq_len, max_seq_len, workspace, window=0, split_tokens=0, layers_in_call=1):
    """q4kv_decode_plan: prepare `workspace` (uint8 tensor on the GPU) for q4kv_batched_attention_planned calls."""
    _check(lib().q4kv_decode_plan(C.byref(spec), _dev(seq_len, torch.int32, "seq_len"), seq_len.numel(), max_seq_len,
                                  int(window), int(split_tokens), layers_in_call, C.c_void_p(workspace.data_ptr()),
                                  workspace.numel(), _stream()))


def q4kv_batched_attention_planned(spec, kpool, vpool, q, out, block_table, max_seq_len, sm_scale, workspace, window=0,
                                   split_tokens=0, layer_begin=0, layer_end=None):
    """q4kv_batched_attention_planned: decode attention (q_len 1) on a workspace prepared by q4kv_decode_plan."""
    layer_end = spec.num_layers if layer_end is None else layer_end
    kp = kpool.c()
    vp = None if spec.v_aliases_k else vpool.c()
    _check(lib().q4kv_batched_attention_planned(
        C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp), _dev(q, torch.float16, "q"),
        _dev(out, torch.float16, "out"), _dev(block_table, torch.int32, "block_table"), block_table.shape[1], q.shape[1],
        max_seq_len, float(sm_scale), int(window), int(split_tokens), layer_begin, layer_end,
        C.c_void_p(workspace.data_ptr()), workspace.numel(), _stream()))
    return out
