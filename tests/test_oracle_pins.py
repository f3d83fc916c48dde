"""Pins for the CPU oracle: each part of oracle/q4kv_oracle.c is checked against something other than
itself -- numbers the paper prints, closed forms, invariants, a library routine it must reduce to, or
brute force on tiny inputs.  Runs without a GPU."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import synth
from tests.util import read_golden, unpack_codes

F16 = np.float16


# ----------------------------------------------------------------------------- binary16 conversions

def test_h2f_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(F16).astype(np.float32)
    got = np.array([oracle.h2f(b) for b in bits], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f2h_rounding_matches_numpy():
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 5, 20000),
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25,
                  2.0 ** -14, 2.0 ** -14 - 2.0 ** -25, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -12],
                 np.float32)])
    # every tie between neighbouring binary16 values in a few binades
    h = np.arange(0x3C00, 0x3C40, dtype=np.uint16).view(F16).astype(np.float32)
    ties = (h[:-1] + h[1:]) / np.float32(2)
    sub = np.arange(0, 40, dtype=np.uint16).view(F16).astype(np.float32)
    vals = np.concatenate([vals, ties, -ties, (sub[:-1] + sub[1:]) / np.float32(2)]).astype(np.float32)
    with np.errstate(over="ignore"):
        want = vals.astype(F16).view(np.uint16)
    got = np.array([oracle.f2h(v) for v in vals], np.uint16)
    assert np.array_equal(got, want)


def test_d2h_from_double_is_single_rounding():
    # 1 + 2^-11 + 2^-30 lies just above a tie: direct rounding goes up, double rounding via binary32 would not
    x = 1.0 + 2.0 ** -11 + 2.0 ** -30
    assert oracle.d2h(x) == 0x3C01
    rng = np.random.default_rng(2)
    vals = rng.standard_normal(5000) * 10.0 ** rng.integers(-6, 4, 5000)
    want = vals.astype(F16).view(np.uint16)
    got = np.array([oracle.d2h(v) for v in vals], np.uint16)
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------- P1 byte accounting

def test_byte_counts_match_paper(golden_dir):
    g = read_golden(os.path.join(golden_dir, "paper_capacity.txt"))
    MiB = 1 << 20
    assert oracle.fp16_layer_bytes(8, 256, 256, 4096) == g["gemma_fp16_layer_bytes_4k"]
    assert oracle.fp16_layer_bytes(8, 256, 256, 4096) * 48 == g["gemma_fp16_agent_mib_4k"] * MiB
    q4 = oracle.q4_layer_bytes(8, 256, 256, 4096)
    assert q4 == g["gemma_q4_layer_bytes_4k"]
    assert q4 == g["gemma_q4_packed_bytes_4k"] + g["gemma_q4_scale_bias_bytes_4k"]
    assert q4 * 48 == g["gemma_q4_agent_mib_4k"] * MiB
    assert round(q4 / oracle.fp16_layer_bytes(8, 256, 256, 4096), 3) == g["q4_over_fp16_ratio"]
    assert oracle.fp16_layer_bytes(8, 128, 128, 4096) == g["llama_fp16_layer_bytes_4k"]
    assert oracle.fp16_layer_bytes(8, 128, 128, 4096) * 32 == g["llama_fp16_agent_mib_4k"] * MiB
    assert oracle.q4_layer_bytes(8, 128, 128, 4096) * 32 == g["llama_q4_agent_mib_4k"] * MiB
    assert oracle.fp16_layer_bytes(8, 128, 128, 1) * 32 == g["llama_fp16_kib_per_token"] * 1024
    assert oracle.fp16_layer_bytes(16, 192, 0, 4096) == g["deepseek_fp16_k_bytes_4k"]
    assert oracle.fp16_layer_bytes(16, 0, 128, 4096) == g["deepseek_fp16_v_bytes_4k"]
    assert oracle.fp16_layer_bytes(16, 192, 128, 4096) * 27 == g["deepseek_fp16_agent_mib_4k"] * MiB
    assert round(oracle.q4_layer_bytes(16, 192, 128, 4096) * 27 / MiB) == g["deepseek_q4_agent_mib_4k"]
    # h*d*n*(1 + 8/g) for symmetric heads, any size
    for h, d, n in [(8, 256, 4096), (8, 128, 777), (1, 64, 1), (16, 512, 12345)]:
        assert oracle.q4_layer_bytes(h, d, d, n) == h * d * n * (64 + 8) // 64


def test_array_sizes_agree_with_byte_formula():
    x = np.zeros((7, 256), F16)
    codes, scale, bias = oracle.quantize(x)
    assert codes.nbytes + scale.nbytes + bias.nbytes == 7 * (256 // 2 + 4 * (256 // 64))
    assert 2 * (codes.nbytes + scale.nbytes + bias.nbytes) == oracle.q4_layer_bytes(1, 256, 256, 7)


# ----------------------------------------------------------------------------- P2-P5 quantizer closed forms

def ramp_group():
    return np.tile(np.arange(16, dtype=F16), 4)          # 64 values 0..15 repeated


def test_unit_ramp_is_identity():
    x = ramp_group()[None, :]
    codes, scale, bias = oracle.quantize(x)
    assert scale.tolist() == [[0x3C00]] and bias.tolist() == [[0x0000]]       # scale 1.0, bias 0
    assert np.array_equal(unpack_codes(codes)[0], x[0].astype(np.uint8))
    assert np.array_equal(oracle.dequantize(codes, scale, bias), x)


def test_nibble_order_low_nibble_first():
    codes, _, _ = oracle.quantize(ramp_group()[None, :])
    assert codes[0].tolist() == [0x76543210, 0xFEDCBA98] * 4


def test_group_axis_is_head_dim_and_groups_are_independent():
    # second group = 2*ramp - 3: scale 2, bias -3; first group untouched
    x = np.concatenate([ramp_group(), 2 * ramp_group() - 3]).astype(F16)[None, :]
    codes, scale, bias = oracle.quantize(x)
    assert scale.view(F16).tolist() == [[1.0, 2.0]] and bias.view(F16).tolist() == [[0.0, -3.0]]
    assert codes[0].tolist() == [0x76543210, 0xFEDCBA98] * 8
    assert np.array_equal(oracle.dequantize(codes, scale, bias), x)
    # two rows are independent too
    x2 = np.stack([x[0], x[0][::-1]])
    c2, s2, b2 = oracle.quantize(x2)
    assert np.array_equal(c2[0], codes[0]) and not np.array_equal(c2[1], codes[0])


def test_ties_round_to_even():
    x = np.zeros(64, F16)
    x[1] = 15.0
    x[2:10] = [0.5, 1.5, 2.5, 3.5, 13.5, 14.5, 7.5, 8.5]
    c = unpack_codes(oracle.quantize(x[None])[0])[0]
    assert c[:10].tolist() == [0, 15, 0, 2, 2, 4, 14, 14, 8, 8]


def test_affine_grid_is_exact():
    # x = b + k*s with s a power of two: codes are k, round trip exact
    rng = np.random.default_rng(3)
    for s, b in [(0.5, -3.0), (0.125, 1.25), (4.0, -30.0), (2.0 ** -10, 0.0)]:
        k = rng.integers(0, 16, 64)
        k[5], k[17] = 0, 15
        x = (b + k * s).astype(F16)[None]
        codes, scale, bias = oracle.quantize(x)
        assert scale.view(F16)[0, 0] == F16(s) and bias.view(F16)[0, 0] == F16(b)
        assert np.array_equal(unpack_codes(codes)[0], k)
        assert np.array_equal(oracle.dequantize(codes, scale, bias), x)


def test_dequantize_formula_on_hand_built_codes():
    # codes 0..15 in every nibble position, scale 0.25, bias -1: x_hat = -1 + 0.25*c
    words = np.array([[0x76543210, 0xFEDCBA98] * 4], np.uint32)
    scale = np.array([[0.25]], F16)
    bias = np.array([[-1.0]], F16)
    got = oracle.dequantize(words, scale, bias)
    want = (-1.0 + 0.25 * np.tile(np.arange(16), 4)).astype(F16)[None]
    assert np.array_equal(got, want)
    # rounding of the sum to binary16: 15*0.1(fp16) + 1000 is not representable
    s16, b16 = F16(0.1), F16(1000.0)
    got = oracle.dequantize(np.array([[0xFFFFFFFF] * 8], np.uint32), np.array([[s16]]), np.array([[b16]]))
    want = F16(np.float32(15.0) * np.float32(s16) + np.float32(b16))
    assert got[0, 0] == want


def test_degenerate_groups():
    x = np.full((1, 64), 3.25, F16)
    codes, scale, bias = oracle.quantize(x)
    assert scale[0, 0] == 0 and bias.view(F16)[0, 0] == F16(3.25) and not codes.any()
    assert np.array_equal(oracle.dequantize(codes, scale, bias), x)
    # range so small that (max-min)/15 rounds to binary16 zero: 7 subnormal steps
    x = np.zeros((1, 64), np.uint16)
    x[0, 3] = 7                                   # 7 * 2^-24
    codes, scale, bias = oracle.quantize(x.view(F16))
    assert (7 * 2.0 ** -24) / 15 < 2.0 ** -25     # below half the smallest subnormal
    assert scale[0, 0] == 0 and not codes.any() and bias[0, 0] == 0
    # 8 steps: scale32 = 8/15 * 2^-24 rounds to 2^-24 (bits 0x0001); codes = rint(k/1)
    x[0, 3] = 8
    codes, scale, bias = oracle.quantize(x.view(F16))
    assert scale[0, 0] == 1 and unpack_codes(codes)[0, 3] == 8


def test_negative_zero_bias_bits_follow_first_minimum():
    x = np.zeros((1, 64), F16)
    x[0, 0] = -0.0
    x[0, 1] = 1.0
    _, _, bias = oracle.quantize(x)
    assert bias[0, 0] == 0x8000
    x[0, 0], x[0, 5] = 0.0, -0.0
    _, _, bias = oracle.quantize(x)
    assert bias[0, 0] == 0x0000


# ----------------------------------------------------------------------------- P6 round-trip bound

def _roundtrip_check(x):
    codes, scale, bias = oracle.quantize(x)
    c = unpack_codes(codes).astype(np.float64)
    s = np.repeat(scale.view(F16).astype(np.float64), 64, axis=-1)
    b = np.repeat(bias.view(F16).astype(np.float64), 64, axis=-1)
    xf = x.astype(np.float64)
    assert c.min() >= 0 and c.max() <= 15
    xg = xf.reshape(-1, 64)
    cg = c.reshape(-1, 64)
    sg = s.reshape(-1, 64)[:, 0]
    mn, mx = xg.min(1), xg.max(1)
    assert np.array_equal(b.reshape(-1, 64)[:, 0], mn)                        # bias is the group minimum, exactly
    rel = np.abs(sg - (mx - mn) / 15) <= 2.0 ** -11 * (mx - mn) / 15 + 2.0 ** -25   # stored scale = fp16((max-min)/15)
    assert rel.all()
    live = sg > 0
    assert np.all(cg[live][np.arange(live.sum()), xg[live].argmin(1)] == 0)   # min -> code 0
    normal = sg >= 2.0 ** -14                                                 # stored scale is a normal binary16
    assert np.all(cg[normal][np.arange(normal.sum()), xg[normal].argmax(1)] == 15)  # max -> code 15
    # unrounded reconstruction within scale/2 (tiny slack for the binary32 division).  A subnormal stored scale
    # carries an absolute rounding error of up to 2^-25, which the top code multiplies by 15; a group whose
    # scale rounds to zero reconstructs as its minimum, so its error is at most its range.
    err = np.abs(xf - (c * s + b)).reshape(-1, 64)
    bound = np.where(normal, sg / 2 * (1 + 2.0 ** -20), np.where(live, sg / 2 + 15 * 2.0 ** -25, mx - mn))
    assert np.all(err <= bound[:, None])
    # the fp16 output of dequantize is the binary32 sum rounded once more
    xh = oracle.dequantize(codes, scale, bias)
    x32 = (c.astype(np.float32) * s.astype(np.float32) + b.astype(np.float32)).astype(F16)
    assert np.array_equal(xh, x32)


def test_roundtrip_bound_random_and_adversarial():
    rng = np.random.default_rng(4)
    _roundtrip_check(rng.standard_normal((200, 256)).astype(F16))
    _roundtrip_check((rng.standard_normal((100, 128)) * 100).astype(F16))
    _roundtrip_check((rng.standard_normal((100, 64)) * 1e-3).astype(F16))
    _roundtrip_check((rng.standard_normal((50, 64)) * 3e-6).astype(F16))          # subnormal inputs
    x = rng.standard_normal((50, 128))
    x[:, ::7] *= 8                                                                # outlier channels
    _roundtrip_check(x.astype(F16))
    big = rng.uniform(-60000, 60000, (20, 64)).astype(F16)                        # near the binary16 range limit
    _roundtrip_check(big)
    # values sitting on code boundaries k + 1/2
    k = rng.integers(0, 15, (30, 64)) + 0.5
    k[:, 0], k[:, 1] = 0, 15
    _roundtrip_check(k.astype(F16))


def test_synthetic_workload_rows_roundtrip():
    w = synth.config(0)
    k = w.k_rows(0, 0, 0, 40).numpy().reshape(-1, 128)
    _roundtrip_check(k)


# ----------------------------------------------------------------------------- helpers for attention pins

def build_cache(w, poison=None, extra_blocks=0, table=None, param_format=oracle.F16_PARAMS):
    """Fill host pools for workload w through oracle.append (tokens 0..final_len-1 of every agent)."""
    spec = oracle.make_spec(w.num_layers, w.num_q_heads, w.num_kv_heads, w.k_dim, w.v_dim, w.v_aliases_k,
                            param_format=param_format)
    if table is None:
        table, nblocks = w.block_table()
    else:
        nblocks = int(table.max()) + 1
    nblocks += extra_blocks
    kpool = oracle.Pool(spec, w.k_dim, nblocks, fill=poison)
    vpool = None if w.v_aliases_k else oracle.Pool(spec, w.v_dim, nblocks, fill=poison)
    for a, n in enumerate(w.final_lens()):
        if n == 0:
            continue
        k_new = np.stack([w.k_rows(l, a, 0, n).numpy() for l in range(w.num_layers)])[:, None]
        v_new = None if w.v_aliases_k else np.stack([w.v_rows(l, a, 0, n).numpy() for l in range(w.num_layers)])[:, None]
        oracle.append(spec, kpool, vpool, k_new, v_new, table[a:a + 1], np.zeros(1, np.int32))
    return spec, kpool, vpool, table


def param_values(bits, param_format=oracle.F16_PARAMS):
    """Stored scale / bias bit patterns -> float64, decoded by numpy (binary16) or torch (bfloat16)."""
    bits = np.ascontiguousarray(bits, np.uint16)
    if param_format == oracle.BF16_PARAMS:
        return torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).double().numpy()
    return bits.view(F16).astype(np.float64)


def dense_rows(w, spec, pool, table, layer, agent, n, dim):
    """Explicitly dequantized [n][kv_heads][dim] float64 of one agent/layer, decoded here with numpy."""
    out = np.zeros((n, spec.num_kv_heads, dim))
    fmt = spec.param_format
    for t in range(n):
        blk = table[agent, t // w.block_tokens]
        slot = t % w.block_tokens
        c = unpack_codes(pool.codes[layer, blk, :, slot]).astype(np.float64)
        s = np.repeat(param_values(pool.scale[layer, blk, :, slot], fmt), 64, axis=-1)
        b = np.repeat(param_values(pool.bias[layer, blk, :, slot], fmt), 64, axis=-1)
        out[t] = c * s + b
    return out


def library_attention(q, k, v, n_rep, sm_scale, vis_per_row, window=0):
    """softmax(sm * q k^T) v with torch float64.  q [R][Hq][Dk], k [n][Hkv][Dk], v [n][Hkv][Dv]."""
    sm_scale = float(np.float32(sm_scale))            # the interface carries the softmax scale as binary32
    q = torch.as_tensor(q, dtype=torch.float64)
    k = torch.as_tensor(k, dtype=torch.float64).repeat_interleave(n_rep, dim=1)
    v = torch.as_tensor(v, dtype=torch.float64).repeat_interleave(n_rep, dim=1)
    out = torch.zeros(q.shape[0], q.shape[1], v.shape[2], dtype=torch.float64)
    for r in range(q.shape[0]):
        vis = vis_per_row[r]
        lo = max(0, vis - window) if window > 0 else 0
        if vis <= lo:
            continue
        z = torch.einsum("hd,thd->ht", q[r], k[lo:vis]) * sm_scale
        p = torch.softmax(z, dim=-1)
        out[r] = torch.einsum("ht,thd->hd", p, v[lo:vis])
    return out.numpy()


SHAPES = [
    # layers, Hq, Hkv, Dk, Dv, alias, seq_lens, q_len
    (2, 4, 2, 64, 64, False, (37, 5, 300), 1),
    (1, 8, 2, 128, 128, False, (260,), 1),
    (1, 2, 2, 128, 64, False, (33, 70), 1),          # asymmetric K/V widths, n_rep 1
    (1, 4, 1, 192, 128, True, (41, 257), 1),         # shared latent: V = first 128 dims of K row
    (1, 4, 2, 64, 64, False, (20, 3), 6),            # chunk of 6 queries
]


@pytest.mark.parametrize("shape", SHAPES)
def test_attention_equals_library_softmax_attention(shape):
    L, Hq, Hkv, Dk, Dv, alias, lens, q_len = shape
    w = synth.small(11, L, Hq, Hkv, Dk, Dv, alias, lens, q_len)
    spec, kpool, vpool, table = build_cache(w, poison=0x7E00, extra_blocks=2)
    q = w.q_all().numpy()
    out16, out64 = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, return_f64=True)
    for l in range(L):
        for a, n in enumerate(w.final_lens()):
            kd = dense_rows(w, spec, kpool, table, l, a, n, Dk)
            vd = kd[:, :, :Dv] if alias else dense_rows(w, spec, vpool, table, l, a, n, Dv)
            vis = [n - (q_len - 1 - r) for r in range(q_len)]
            want = library_attention(q[l, a].astype(np.float64), kd, vd, w.n_rep, w.sm_scale, vis)
            assert np.allclose(out64[l, a], want, rtol=1e-11, atol=1e-12)
            assert np.array_equal(out16[l, a], want.astype(F16)) or \
                np.max(np.abs(out16[l, a].astype(np.float64) - want)) <= np.max(np.abs(want)) * 2.0 ** -10
    assert not np.isnan(out64).any()


def test_attention_brute_force_python_loops():
    # smallest case written with bare loops, no vector library
    import math
    w = synth.small(5, 1, 2, 1, 64, 64, False, (9,), 1)
    spec, kpool, vpool, table = build_cache(w)
    q = w.q_all().numpy()
    _, out64 = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), 0.25, return_f64=True)
    kd = dense_rows(w, spec, kpool, table, 0, 0, 9, 64)
    vd = dense_rows(w, spec, vpool, table, 0, 0, 9, 64)
    for h in range(2):
        z = [0.25 * sum(float(q[0, 0, 0, h, d]) * kd[t, 0, d] for d in range(64)) for t in range(9)]
        m = max(z)
        e = [math.exp(v - m) for v in z]
        tot = sum(e)
        for d in range(64):
            o = sum(e[t] / tot * vd[t, 0, d] for t in range(9))
            assert abs(o - out64[0, 0, 0, h, d]) < 1e-13


# ----------------------------------------------------------------------------- P8 softmax sanity

def test_softmax_rows_sum_to_one_and_special_cases():
    w = synth.small(6, 1, 4, 2, 64, 64, False, (150,), 1)
    spec, kpool, vpool, table = build_cache(w)
    q = w.q_all().numpy()
    for h in range(4):
        p, o = oracle.attention_probs(spec, kpool, vpool, 0, table[0], h // 2, q[0, 0, 0, h], 150, w.sm_scale)
        assert abs(p.sum() - 1.0) < 1e-12 and (p >= 0).all()
        vd = dense_rows(w, spec, vpool, table, 0, 0, 150, 64)[:, h // 2]
        assert np.allclose(o, p @ vd, rtol=1e-12, atol=1e-13)
    # one key: the output is that V row exactly
    out64 = oracle.attention(spec, kpool, vpool, q, table, [1], w.sm_scale, return_f64=True)[1]
    v0 = dense_rows(w, spec, vpool, table, 0, 0, 1, 64)[0]
    assert np.array_equal(out64[0, 0, 0], np.repeat(v0, 2, axis=0))
    # zero query: uniform weights, output = mean of V rows
    out64 = oracle.attention(spec, kpool, vpool, np.zeros_like(q), table, [150], w.sm_scale, return_f64=True)[1]
    vd = dense_rows(w, spec, vpool, table, 0, 0, 150, 64)
    assert np.allclose(out64[0, 0, 0], np.repeat(vd.mean(0), 2, axis=0), rtol=1e-12, atol=1e-13)
    # zero keys visible: zeros, not NaN
    out16 = oracle.attention(spec, kpool, vpool, q, table, [0], w.sm_scale)
    assert not out16.view(np.uint16).any()


def test_dominant_key_selects_its_value_row():
    w = synth.small(7, 1, 1, 1, 64, 64, False, (50,), 1)
    spec, kpool, vpool, table = build_cache(w)
    # make token 17's key huge along the query direction: hand-built row, code 15 everywhere, scale 4
    q = np.ones((1, 1, 1, 1, 64), F16)
    blk = table[0, 0]
    kpool.codes[0, blk, 0, 17] = 0xFFFFFFFF
    kpool.scale[0, blk, 0, 17] = np.array(4.0, F16).view(np.uint16)
    kpool.bias[0, blk, 0, 17] = 0
    out64 = oracle.attention(spec, kpool, vpool, q, table, [50], 1.0, return_f64=True)[1]
    v17 = dense_rows(w, spec, vpool, table, 0, 0, 50, 64)[17, 0]
    assert np.allclose(out64[0, 0, 0, 0], v17, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- P9 chunk == decode

def test_chunk_rows_equal_decode_steps():
    w = synth.small(8, 1, 4, 2, 64, 64, False, (70, 10), 5)
    spec, kpool, vpool, table = build_cache(w)
    q = w.q_all().numpy()
    full = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, return_f64=True)[1]
    for r in range(5):
        lens = [n + r + 1 for n in w.seq_lens]
        one = oracle.attention(spec, kpool, vpool, q[:, :, r:r + 1], table, lens, w.sm_scale, return_f64=True)[1]
        assert np.array_equal(one[:, :, 0], full[:, :, r])


# ----------------------------------------------------------------------------- P10 paging / batching / isolation

def test_block_permutation_batching_and_poison():
    w = synth.small(9, 2, 4, 2, 64, 64, False, (300, 513, 40), 1)
    spec, kpool, vpool, table = build_cache(w, poison=0x7E00, extra_blocks=3)
    q = w.q_all().numpy()
    ref16, ref64 = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, return_f64=True)
    assert not np.isnan(ref64).any()                    # poisoned tail slots and spare blocks never read
    # another physical placement of the same logical cache
    rng = np.random.default_rng(0)
    nb = kpool.num_blocks
    perm = rng.permutation(nb).astype(np.int32)
    table2 = np.where(table >= 0, perm[np.clip(table, 0, nb - 1)], -1).astype(np.int32)
    spec2, kpool2, vpool2, _ = build_cache(w, poison=0x7E00, extra_blocks=0, table=np.where(table2 >= 0, table2, 0))
    kpool2b = oracle.Pool(spec, 64, nb, fill=0x7E00)
    vpool2b = oracle.Pool(spec, 64, nb, fill=0x7E00)
    for src, dst in ((kpool, kpool2b), (vpool, vpool2b)):
        for arr in ("codes", "scale", "bias"):
            getattr(dst, arr)[:, perm] = getattr(src, arr)
    out = oracle.attention(spec, kpool2b, vpool2b, q, table2, w.final_lens(), w.sm_scale, return_f64=True)[1]
    assert np.array_equal(out, ref64)
    # batch of A agents == A single-agent calls
    for a in range(3):
        one = oracle.attention(spec, kpool, vpool, q[:, a:a + 1], table[a:a + 1], w.final_lens()[a:a + 1],
                               w.sm_scale, return_f64=True)[1]
        assert np.array_equal(one[:, 0], ref64[:, a])
    # layer range: layers [1,2) alone
    one = oracle.attention(spec, kpool, vpool, q[1:2], table, w.final_lens(), w.sm_scale, layer_begin=1, layer_end=2,
                           return_f64=True)[1]
    assert np.array_equal(one[0], ref64[1])


def test_token_order_does_not_matter_for_decode():
    w = synth.small(10, 1, 2, 1, 64, 64, False, (100,), 1)
    spec, kpool, vpool, table = build_cache(w)
    q = w.q_all().numpy()
    ref = oracle.attention(spec, kpool, vpool, q, table, [100], w.sm_scale, return_f64=True)[1]
    perm = np.random.default_rng(1).permutation(100)
    blk = table[0, 0]
    for p in (kpool, vpool):
        for arr in ("codes", "scale", "bias"):
            getattr(p, arr)[0, blk, 0, :100] = getattr(p, arr)[0, blk, 0, perm]
    out = oracle.attention(spec, kpool, vpool, q, table, [100], w.sm_scale, return_f64=True)[1]
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-14)


# ----------------------------------------------------------------------------- P11 GQA / shared latent mapping

def test_gqa_grouping_is_contiguous():
    w = synth.small(12, 1, 6, 2, 64, 64, False, (90,), 1)
    spec, kpool, vpool, table = build_cache(w)
    q = w.q_all().numpy()
    q[0, 0, 0, 1] = q[0, 0, 0, 0]          # heads 0,1,2 share kv head 0
    q[0, 0, 0, 3] = q[0, 0, 0, 0]          # head 3 reads kv head 1
    out = oracle.attention(spec, kpool, vpool, q, table, [90], w.sm_scale, return_f64=True)[1][0, 0, 0]
    assert np.array_equal(out[0], out[1]) and not np.allclose(out[0], out[3])
    # against single-kv-head problems built from each kv head alone
    for kvh in range(2):
        w1 = synth.small(12, 1, 3, 1, 64, 64, False, (90,), 1)
        spec1 = oracle.make_spec(1, 3, 1, 64, 64)
        k1 = oracle.Pool(spec1, 64, kpool.num_blocks)
        v1 = oracle.Pool(spec1, 64, kpool.num_blocks)
        for src, dst in ((kpool, k1), (vpool, v1)):
            for arr in ("codes", "scale", "bias"):
                getattr(dst, arr)[:, :, 0] = getattr(src, arr)[:, :, kvh]
        o1 = oracle.attention(spec1, k1, v1, q[:, :, :, 3 * kvh:3 * kvh + 3], table, [90], w.sm_scale,
                              return_f64=True)[1][0, 0, 0]
        assert np.array_equal(o1, out[3 * kvh:3 * kvh + 3])
        del w1


def test_shared_latent_equals_separate_v_copy():
    w = synth.small(13, 1, 4, 1, 192, 128, True, (75,), 1)
    spec, kpool, _, table = build_cache(w)
    q = w.q_all().numpy()
    out = oracle.attention(spec, kpool, None, q, table, [75], w.sm_scale, return_f64=True)[1]
    spec2 = oracle.make_spec(1, 4, 1, 192, 128, False)
    vpool = oracle.Pool(spec2, 128, kpool.num_blocks)
    vpool.codes[...] = kpool.codes[..., :16]
    vpool.scale[...] = kpool.scale[..., :2]
    vpool.bias[...] = kpool.bias[..., :2]
    out2 = oracle.attention(spec2, kpool, vpool, q, table, [75], w.sm_scale, return_f64=True)[1]
    assert np.array_equal(out, out2)


# ----------------------------------------------------------------------------- sliding window

def test_sliding_window_against_library_mask():
    w = synth.small(14, 2, 4, 2, 64, 64, False, (120, 30), 4)
    spec, kpool, vpool, table = build_cache(w)
    q = w.q_all().numpy()
    glob = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, return_f64=True)[1]
    assert np.array_equal(oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, window=1000,
                                           return_f64=True)[1], glob)
    win = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, window=16, return_f64=True)[1]
    per_layer = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale,
                                 window_per_layer=[0, 16], return_f64=True)[1]
    assert np.array_equal(per_layer[0], glob[0]) and np.array_equal(per_layer[1], win[1])
    for a, n in enumerate(w.final_lens()):
        kd = dense_rows(w, spec, kpool, table, 1, a, n, 64)
        vd = dense_rows(w, spec, vpool, table, 1, a, n, 64)
        vis = [n - (4 - 1 - r) for r in range(4)]
        want = library_attention(q[1, a].astype(np.float64), kd, vd, 2, w.sm_scale, vis, window=16)
        assert np.allclose(win[1, a], want, rtol=1e-11, atol=1e-12)
    # window 1: each row sees only its own position
    w1 = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, window=1, return_f64=True)[1]
    vd = dense_rows(w, spec, vpool, table, 0, 0, 124, 64)
    assert np.array_equal(w1[0, 0, 3, 0], vd[123, 0]) and np.array_equal(w1[0, 0, 0, 3], vd[120, 1])


# ----------------------------------------------------------------------------- append

def test_append_places_flat_quantizer_output_and_touches_nothing_else():
    w = synth.small(15, 2, 2, 2, 128, 64, False, (250, 7), 1)
    spec = oracle.make_spec(2, 2, 2, 128, 64)
    table, nb = w.block_table()
    table = np.concatenate([table, [[nb], [nb + 1]]], axis=1).astype(np.int32)     # room for the chunk
    kpool = oracle.Pool(spec, 128, nb + 2, fill=0x7E00)
    vpool = oracle.Pool(spec, 64, nb + 2, fill=0x7E00)
    before = [kpool.codes.copy(), vpool.scale.copy()]
    C_ = 10
    k_new = np.stack([np.stack([w.k_rows(l, a, 1000, 1000 + C_).numpy() for a in range(2)]) for l in range(2)])
    v_new = np.stack([np.stack([w.v_rows(l, a, 1000, 1000 + C_).numpy() for a in range(2)]) for l in range(2)])
    oracle.append(spec, kpool, vpool, k_new[1:], v_new[1:], table, w.seq_lens, layer_begin=1, layer_end=2)
    kc, ks, kb = oracle.quantize(k_new)
    vc, vs, vb = oracle.quantize(v_new)
    touched = np.zeros(kpool.codes.shape[:4], bool)
    for a, n in enumerate(w.seq_lens):
        for c in range(C_):
            t = n + c
            blk, slot = table[a, t // 256], t % 256
            assert np.array_equal(kpool.codes[1, blk, :, slot], kc[1, a, c])
            assert np.array_equal(kpool.scale[1, blk, :, slot], ks[1, a, c])
            assert np.array_equal(kpool.bias[1, blk, :, slot], kb[1, a, c])
            assert np.array_equal(vpool.codes[1, blk, :, slot], vc[1, a, c])
            assert np.array_equal(vpool.scale[1, blk, :, slot], vs[1, a, c])
            assert np.array_equal(vpool.bias[1, blk, :, slot], vb[1, a, c])
            touched[1, blk, :, slot] = True
    assert np.array_equal(kpool.codes[~touched], before[0][~touched])
    assert np.array_equal(vpool.scale[~touched], before[1][~touched])
    # agent 0's chunk crosses from block 0 (slots 250..255) into its second block
    assert touched[1, table[0, 0], 0, 255] and touched[1, table[0, 1], 0, 3]


def test_bad_arguments_are_rejected():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 100), F16))
    w = synth.small(16, 1, 2, 1, 64, 64, False, (10,), 1)
    spec, kpool, vpool, table = build_cache(w)
    with pytest.raises(ValueError):
        oracle.attention(spec, kpool, vpool, w.q_all().numpy(), table, [10_000], w.sm_scale)
