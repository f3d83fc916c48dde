"""Host-side checks of libq4kv that need no GPU: the library loads, exports everything the header
declares, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

from paper_2603_04428_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "q4kv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(q4kv_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_symbols()
    assert set(names) == set(b.EXPORTS)
    l = b.lib()
    for n in names:
        assert getattr(l, n) is not None


def test_version_and_cache_bytes_closed_form():
    assert b.q4kv_version() >= 100
    gemma = b.make_spec(48, 16, 8, 256)
    assert b.q4kv_cache_bytes(gemma, 4096) == 432 * 2 ** 20           # App. FP16 vs Q4: 9.0 MB * 48 layers
    assert b.q4kv_cache_bytes(gemma, 1) == 48 * 8 * 256 * (64 + 8) // 64
    llama = b.make_spec(32, 32, 8, 128)
    assert b.q4kv_cache_bytes(llama, 4096) == 144 * 2 ** 20
    mla = b.make_spec(27, 16, 1, 576, 512, True)
    assert b.q4kv_cache_bytes(mla, 1) == 27 * 324


def _err():
    return b.lib().q4kv_last_error().decode()


def test_codec_argument_errors():
    l = b.lib()
    assert l.q4kv_quantize(None, 5, 100, None, None, None, None) == -2 and "64" in _err()
    assert l.q4kv_quantize(None, -1, 64, None, None, None, None) == -1
    assert l.q4kv_quantize(None, 5, 64, None, None, None, None) == -1 and "NULL" in _err()
    assert l.q4kv_quantize(8, 5, 64, 16, 16, 16, None) == -1 and "aligned" in _err()
    assert l.q4kv_quantize(None, 0, 64, None, None, None, None) == 0          # empty input is a no-op
    assert l.q4kv_dequantize(None, None, None, 3, 96, None, None) == -2
    assert l.q4kv_dequantize(None, None, None, 0, 128, None, None) == 0


def test_parameter_format_argument_errors():
    l = b.lib()
    assert l.q4kv_quantize_fmt(None, 5, 64, 2, None, None, None, None) == -1 and "param_format" in _err()
    assert l.q4kv_dequantize_fmt(None, None, None, 5, 64, -1, None, None) == -1 and "param_format" in _err()
    assert l.q4kv_quantize_fmt(None, 0, 64, b.PARAMS_BF16, None, None, None, None) == 0
    assert l.q4kv_quantize_fmt(None, 5, 100, b.PARAMS_BF16, None, None, None, None) == -2
    bad = b.make_spec(2, 4, 2, 128, param_format=7)
    assert b.lib().q4kv_cache_bytes(C.byref(bad), 10) == -1 and "param_format" in _err()
    assert b.lib().q4kv_block_image_bytes(C.byref(bad), 1) == 0
    good = b.make_spec(48, 16, 8, 256, param_format=b.PARAMS_BF16)
    assert b.q4kv_cache_bytes(good, 4096) == 432 * 2 ** 20        # both parameter types are 16 bits wide


def _pool(nb=4):
    return b._CPool(0x1000, 0x2000, 0x3000, nb)


def test_attention_argument_errors():
    l = b.lib()
    spec = b.make_spec(2, 4, 2, 128)
    kp, vp = _pool(), _pool()
    args = dict(q=0x4000, out=0x5000, bt=0x6000, mb=4, sl=0x7000, A=2, q_len=1, msl=1024, sm=0.1, win=0, st=0, lb=0,
                le=2, ws=0x8000, wsb=1 << 30)

    def call(spec=spec, kp=kp, vp=vp, **kw):
        a = dict(args, **kw)
        return l.q4kv_batched_attention(C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp), a["q"],
                                        a["out"], a["bt"], a["mb"], a["sl"], a["A"], a["q_len"], a["msl"], a["sm"],
                                        a["win"], a["st"], a["lb"], a["le"], a["ws"], a["wsb"], None)

    assert call(msl=1025) == -3 and "max_blocks" in _err()                     # beyond the block table
    assert call(le=3) == -1 and call(lb=2, le=1) == -1
    assert call(st=100) == -1
    assert call(q=None) == -1
    assert call(wsb=16) == -4 and "workspace" in _err()
    assert call(ws=None) == -4
    assert call(kp=b._CPool(0x1000, 0, 0x3000, 4)) == -1
    assert call(kp=b._CPool(0x1004, 0x2000, 0x3000, 4)) == -1                  # misaligned
    assert call(vp=_pool(5)) == -1
    assert call(spec=b.make_spec(2, 5, 2, 128)) == -2
    assert call(spec=b.make_spec(2, 4, 2, 100)) == -2
    assert call(spec=b.make_spec(2, 4, 2, 128, block_tokens=128)) == -2
    bad_group = b.make_spec(2, 4, 2, 128)
    bad_group.group_size = 32
    assert call(spec=bad_group) == -2
    assert call(spec=b.make_spec(2, 4, 2, 512)) == -2 and "no decode kernel" in _err()
    assert call(A=0) == 0 and call(lb=1, le=1) == 0                             # nothing to do


def test_append_argument_errors():
    l = b.lib()
    spec = b.make_spec(2, 4, 2, 128)
    kp, vp = _pool(), _pool()

    def call(spec=spec, kp=kp, vp=vp, kn=0x4000, vn=0x5000, bt=0x6000, mb=4, sl=0x7000, A=2, Cn=8, lb=0, le=2):
        return l.q4kv_append(C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp), kn, vn, bt, mb, sl, A,
                             Cn, lb, le, None)

    assert call(le=5) == -1
    assert call(kn=None) == -1
    assert call(vp=None) == -1
    assert call(Cn=0) == 0
    assert call(Cn=(1 << 20) + 1) == -3 and "chunk_len" in _err()
    mla = b.make_spec(2, 4, 1, 576, 512, True)
    assert call(spec=mla, vp=vp) == -1 and "NULL" in _err()                     # aliased V takes no V pool


def test_window_array_and_block_image_argument_errors():
    """The later entry points find their argument errors on the host, before anything is launched (fake pointers)."""
    l = b.lib()
    spec = b.make_spec(2, 4, 2, 128)
    kp, vp = _pool(), _pool()
    windows = (C.c_int32 * 2)(0, 16)

    def attend(win=windows, spec=spec, lb=0, le=2):
        return l.q4kv_batched_attention_windows(C.byref(spec), C.byref(kp), C.byref(vp), 0x4000, 0x5000, 0x6000, 4,
                                                0x7000, 2, 1, 1024, 0.1, win, 0, lb, le, 0x8000, 1 << 30, None)

    assert attend(win=None) == -1 and "window" in _err()
    big = b.make_spec(200, 4, 2, 128)
    assert attend(win=(C.c_int32 * 200)(), spec=big, le=200) == -1 and "128" in _err()      # one window per layer: 128 at most
    assert attend(lb=1, le=1) == 0                                                         # nothing to do

    def image(fn=l.q4kv_export_blocks, spec=spec, kp=kp, vp=vp, ids=0x4000, n=3, img=0x9000, nbytes=1 << 30):
        return fn(C.byref(spec), C.byref(kp), None if vp is None else C.byref(vp), ids, n, img, nbytes, None)

    need = l.q4kv_block_image_bytes(C.byref(spec), 3)
    rows = 2 * 256                                            # per (layer, block): K and V codes, scales, biases
    assert need == 2 * 3 * 2 * (rows * 16 * 4 + 2 * rows * 2 * 2)
    assert l.q4kv_block_image_bytes(C.byref(spec), -1) == 0
    for fn in (l.q4kv_export_blocks, l.q4kv_import_blocks):
        assert image(fn, nbytes=need - 1) == -4 and "image" in _err()
        assert image(fn, ids=None) == -1 and image(fn, img=None) == -1
        assert image(fn, img=0x9004) == -1                                                 # misaligned image
        assert image(fn, n=-1) == -1
        assert image(fn, vp=None) == -1                                                    # V pool missing
        assert image(fn, vp=_pool(5)) == -1                                                # pools of different sizes
        assert image(fn, n=0, ids=None, img=None) == 0                                     # nothing to do
    mla = b.make_spec(2, 16, 1, 576, 512, True)
    assert image(spec=mla, vp=vp) == -1                                                    # aliased V takes no V pool
    assert l.q4kv_block_image_bytes(C.byref(mla), 1) == 2 * (256 * 72 * 4 + 2 * 256 * 9 * 2)
    assert l.q4kv_read_probe(None, 1 << 20, 0x4000, None) == -1
    assert l.q4kv_read_probe(0x4000, 1 << 20, None, None) == -1
    assert l.q4kv_read_probe(0x4004, 1 << 20, 0x4000, None) == -1
    assert l.q4kv_read_probe(None, 100, None, None) == 0                                   # below one step: nothing to read


def test_workspace_and_split_queries():
    gemma = b.make_spec(48, 16, 8, 256)
    st = b.q4kv_default_split_tokens(gemma, 10, 1, 8192, 48)
    assert st % 256 == 0 and 256 <= st <= 512
    assert b.q4kv_default_split_tokens(gemma, 10, 1, 8192, 1) == 512            # one layer's call: twice an even share
    assert b.q4kv_default_split_tokens(gemma, 1, 1, 1024, 1) == 256             # small job: finest share
    n = b.q4kv_attention_workspace_bytes(gemma, 10, 1, 8192, 1024, 48)
    slots = (8192 // 64 + 15) // 16 + 1            # a unit of 128 tiles can meet at most 9 shares of >= 16 tiles
    # plan: six-word header, per-layer prefix and class, L class blocks, lengths, agents without tokens
    A, L = 10, 48
    plan = ((6 + 2 * L + 1 + L * (2 * A + 2) + 2 * A) * 4 + 255) // 256 * 256
    arrivals = (L * 8 * A * 4 + 255) // 256 * 256  # one counter per (layer, KV head, agent)
    assert n == plan + arrivals + 48 * 10 * 16 * slots * (256 + 2) * 4
    assert b.q4kv_attention_workspace_bytes(gemma, 10, 1, 8192, 100, 48) == 0   # not a multiple of 256


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/libq4kv.so")
    with pytest.raises(ImportError):
        b.lib()
