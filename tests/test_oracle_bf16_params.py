"""Pins for the oracle's bfloat16 parameter format (scale and bias stored as bfloat16, Sec. 3.1 / 3.2 and the
appendix "safetensors Q4 Format"): conversions against torch's bfloat16, hand-worked groups, the round-trip bound
that follows from the reading, agreement with the binary16 format wherever both store the same values, and
attention against a library softmax over explicitly decoded rows.  Runs without a GPU."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import synth
from tests.test_oracle_pins import build_cache, dense_rows, library_attention, param_values, ramp_group
from tests.util import unpack_codes

F16 = np.float16
BF = oracle.BF16_PARAMS


def torch_bf16_bits(x32):
    """binary32 array -> bfloat16 bit patterns by torch's conversion (round to nearest even)."""
    t = torch.from_numpy(np.ascontiguousarray(x32, np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


# ----------------------------------------------------------------------------- conversions

def test_bf2f_all_patterns_match_torch():
    bits = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    got = np.array([oracle.bf2f(b) for b in bits], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_f2bf_rounding_matches_torch():
    rng = np.random.default_rng(21)
    vals = rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 20000)
    # every tie between neighbouring bfloat16 values of two binades, and values one binary32 step beside them
    b = torch.arange(0x3F80, 0x4080, dtype=torch.int16).view(torch.bfloat16).float().numpy()
    ties = (b[:-1] + b[1:]) / np.float32(2)
    beside = np.concatenate([np.nextafter(ties, np.float32(0)), np.nextafter(ties, np.float32(10))])
    special = np.array([0.0, -0.0, 1.0, 3.3895314e38, 3.4e38, 1e-40, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -134,
                        2.0 ** -126, 65504.0, 1.00390625, 1.01171875], np.float32)
    vals = np.concatenate([vals, ties, -ties, beside, special]).astype(np.float32)
    want = torch_bf16_bits(vals)
    got = np.array([oracle.f2bf(v) for v in vals], np.uint16)
    assert np.array_equal(got, want)


# ----------------------------------------------------------------------------- hand-worked groups

def test_unit_ramp_is_identity_with_bfloat16_parameters():
    x = ramp_group()[None, :]
    codes, scale, bias = oracle.quantize(x, BF)
    assert scale.tolist() == [[0x3F80]] and bias.tolist() == [[0x0000]]       # bfloat16 1.0 and 0
    assert codes[0].tolist() == [0x76543210, 0xFEDCBA98] * 4
    assert np.array_equal(oracle.dequantize(codes, scale, bias, BF), x)


def test_bias_that_rounds_down_shifts_the_codes_up():
    # min 1000.5 is a binary16 value but bfloat16 has steps of 4 there: stored bias 1000.  The range 7.5 gives
    # scale 0.5 exactly.  Codes are taken against the stored bias: (1000.5 + k/2 - 1000) / 0.5 = k + 1, and the
    # top element (k = 15) clamps at 15.
    k = np.tile(np.arange(16), 4)
    x = (1000.5 + 0.5 * k).astype(F16)[None]
    assert np.array_equal(x.astype(np.float64)[0], 1000.5 + 0.5 * k)          # all representable
    codes, scale, bias = oracle.quantize(x, BF)
    assert scale.tolist() == [[0x3F00]] and bias.tolist() == [[0x447A]]       # 0.5 and 1000 = 1.953125 * 2^9
    assert np.array_equal(unpack_codes(codes)[0], np.minimum(k + 1, 15))
    back = oracle.dequantize(codes, scale, bias, BF).astype(np.float64)[0]
    assert np.array_equal(back, 1000.0 + 0.5 * np.minimum(k + 1, 15))


def test_bias_that_rounds_up_clamps_at_zero():
    # min 1 + 6/1024 rounds to the bfloat16 value 1 + 1/128 above it; the minimum's quotient is negative and
    # becomes code 0, every other element sits 1/512 below its grid point and rounds to it
    k = np.tile(np.arange(16), 4)
    x = (1.005859375 + 0.125 * k).astype(F16)[None]
    assert np.array_equal(x.astype(np.float64)[0], 1.005859375 + 0.125 * k)
    codes, scale, bias = oracle.quantize(x, BF)
    assert scale.tolist() == [[0x3E00]] and bias.tolist() == [[0x3F81]]       # 0.125 and 1.0078125
    assert np.array_equal(unpack_codes(codes)[0], k)
    assert oracle.dequantize(codes, scale, bias, BF)[0, 0] == F16(1.0078125)


def test_tie_of_the_bias_goes_to_the_even_neighbour():
    x = np.full((1, 64), 1.00390625, F16)          # halfway between bfloat16 1.0 (even) and 1.0078125
    x[0, 1] = 2.0
    _, _, bias = oracle.quantize(x, BF)
    assert bias[0, 0] == 0x3F80
    x[0, :] = 1.01171875                           # halfway between 1.0078125 (odd) and 1.015625 (even)
    x[0, 1] = 2.0
    _, _, bias = oracle.quantize(x, BF)
    assert bias[0, 0] == 0x3F82


def test_dequantize_formula_on_hand_built_codes_bfloat16():
    words = np.array([[0x76543210, 0xFEDCBA98] * 4], np.uint32)
    scale = np.array([[0x3E80]], np.uint16)        # 0.25
    bias = np.array([[0xBF80]], np.uint16)         # -1
    got = oracle.dequantize(words, scale, bias, BF)
    assert np.array_equal(got, (-1.0 + 0.25 * np.tile(np.arange(16), 4)).astype(F16)[None])
    # the same bit patterns mean something else as binary16: the format argument is honoured
    assert not np.array_equal(oracle.dequantize(words, scale, bias), got)
    # a sum that binary16 cannot hold is rounded once: 15 * 0.099609375 + 1000
    got = oracle.dequantize(np.array([[0xFFFFFFFF] * 8], np.uint32), np.array([[0x3DCC]], np.uint16),
                            np.array([[0x447A]], np.uint16), BF)
    assert got[0, 0] == F16(np.float32(15.0) * np.float32(0.099609375) + np.float32(1000.0))


def test_constant_group_and_tiny_range():
    x = np.full((1, 64), 3.25, F16)
    codes, scale, bias = oracle.quantize(x, BF)
    assert scale[0, 0] == 0 and bias[0, 0] == 0x4050 and not codes.any()
    assert np.array_equal(oracle.dequantize(codes, scale, bias, BF), x)
    # one binary16 subnormal step of range: binary16 would store scale 0, bfloat16 holds 2^-24 / 15
    xb = np.zeros((1, 64), np.uint16)
    xb[0, 3] = 1
    codes, scale, bias = oracle.quantize(xb.view(F16), BF)
    assert scale[0, 0] == torch_bf16_bits(np.array([np.float32(2.0 ** -24) / np.float32(15)]))[0]
    assert unpack_codes(codes)[0, 3] == 15 and bias[0, 0] == 0


# ----------------------------------------------------------------------------- the bound the reading implies

def _roundtrip_check(x):
    codes, scale, bias = oracle.quantize(x, BF)
    c = unpack_codes(codes).astype(np.float64).reshape(-1, 64)
    xg = x.astype(np.float64).reshape(-1, 64)
    s = param_values(scale, BF).reshape(-1)
    b = param_values(bias, BF).reshape(-1)
    mn, mx = xg.min(1), xg.max(1)
    # stored parameters are the bfloat16 roundings (torch's) of the minimum and of the binary32 quotient
    assert np.array_equal(bias.reshape(-1), torch_bf16_bits(mn.astype(np.float32)))
    s32 = (mx.astype(np.float32) - mn.astype(np.float32)) / np.float32(15)
    assert np.array_equal(scale.reshape(-1), torch_bf16_bits(s32))
    assert c.min() >= 0 and c.max() <= 15
    # inside the code range the error is half a step; below the stored bias it is the bias's rounding error,
    # above the top code the scale's (times 15) plus the bias's
    err = np.abs(xg - (c * s[:, None] + b[:, None]))
    bound = s / 2 * (1 + 2.0 ** -20) + np.abs(b - mn) + 15 * np.abs(s - s32.astype(np.float64))
    assert np.all(err <= bound[:, None])
    # and where the quotient lands strictly inside [0, 15] the half-step bound alone holds
    u = (xg - b[:, None]) / np.where(s > 0, s, 1)[:, None]
    inside = (u >= 0) & (u <= 15) & (s > 0)[:, None]
    assert np.all(err[inside] <= (np.broadcast_to(s[:, None], err.shape)[inside]) / 2 * (1 + 2.0 ** -20))
    # codes are the rounded quotient against the stored parameters wherever no tie is near
    frac = np.abs(u - np.floor(u) - 0.5)
    clear = (frac > 1e-4) & (s > 0)[:, None]
    assert np.array_equal(c[clear], np.clip(np.rint(u), 0, 15)[clear])
    # dequantize = binary32 sum rounded to binary16
    xh = oracle.dequantize(codes, scale, bias, BF).reshape(-1, 64)
    x32 = (c.astype(np.float32) * s.astype(np.float32)[:, None] + b.astype(np.float32)[:, None]).astype(F16)
    assert np.array_equal(xh, x32)


def test_roundtrip_bound_random_and_adversarial_bfloat16():
    rng = np.random.default_rng(24)
    _roundtrip_check(rng.standard_normal((200, 256)).astype(F16))
    _roundtrip_check((rng.standard_normal((100, 128)) * 100).astype(F16))
    _roundtrip_check((rng.standard_normal((100, 64)) * 1e-3).astype(F16))
    _roundtrip_check((rng.standard_normal((50, 64)) * 3e-6).astype(F16))          # subnormal inputs
    _roundtrip_check((1000 + rng.standard_normal((50, 64))).astype(F16))          # bias error >> scale
    _roundtrip_check((-700 + 0.1 * rng.standard_normal((50, 64))).astype(F16))
    x = rng.standard_normal((50, 128))
    x[:, ::7] *= 8
    _roundtrip_check(x.astype(F16))
    _roundtrip_check(rng.uniform(-30000, 30000, (20, 64)).astype(F16))
    w = synth.config(0)
    _roundtrip_check(w.k_rows(0, 0, 0, 40).numpy().reshape(-1, 128))


# ----------------------------------------------------------------------------- ties to the binary16 format

def test_formats_agree_when_both_store_the_same_parameters():
    # power-of-two scale and a bias of few significant bits are exact in both formats: same codes, same values
    rng = np.random.default_rng(25)
    for s, b in [(0.5, -3.0), (0.125, 1.25), (4.0, -30.0), (2.0 ** -10, 0.0)]:
        k = rng.integers(0, 16, 64)
        k[5], k[17] = 0, 15
        x = (b + k * s).astype(F16)[None]
        c16, s16, b16 = oracle.quantize(x)
        cbf, sbf, bbf = oracle.quantize(x, BF)
        assert np.array_equal(c16, cbf) and np.array_equal(unpack_codes(cbf)[0], k)
        assert param_values(sbf, BF)[0, 0] == s16.view(F16)[0, 0] == s
        assert param_values(bbf, BF)[0, 0] == b16.view(F16)[0, 0] == b
        assert np.array_equal(oracle.dequantize(cbf, sbf, bbf, BF), x)


def test_attention_agrees_with_binary16_format_on_exactly_representable_caches():
    # rows on a grid with power-of-two steps and small integer offsets: both formats hold the same cache, so the
    # attention outputs must be identical
    w = synth.small(26, 1, 4, 2, 64, 64, False, (70, 9), 1)
    rng = np.random.default_rng(26)

    def grid_rows(shape):
        k = rng.integers(0, 16, shape + (64,))
        k[..., 0], k[..., 1] = 0, 15
        off = rng.integers(-4, 5, shape + (1,))
        return (off + 0.25 * k).astype(F16)

    outs = []
    for fmt in (oracle.F16_PARAMS, BF):
        rng = np.random.default_rng(26)
        spec = oracle.make_spec(1, 4, 2, 64, 64, param_format=fmt)
        table, nb = w.block_table()
        kpool, vpool = oracle.Pool(spec, 64, nb), oracle.Pool(spec, 64, nb)
        for a, n in enumerate(w.seq_lens):
            oracle.append(spec, kpool, vpool, grid_rows((1, 1, n, 2)), grid_rows((1, 1, n, 2)), table[a:a + 1],
                          np.zeros(1, np.int32))
        outs.append(oracle.attention(spec, kpool, vpool, w.q_all().numpy(), table, w.seq_lens, w.sm_scale,
                                     return_f64=True)[1])
    assert np.array_equal(outs[0], outs[1]) and np.abs(outs[0]).max() > 0


# ----------------------------------------------------------------------------- attention and append

SHAPES = [
    (2, 4, 2, 64, 64, False, (37, 5, 300), 1),
    (1, 2, 2, 128, 64, False, (33, 70), 1),
    (1, 4, 1, 192, 128, True, (41, 257), 1),
    (1, 4, 2, 64, 64, False, (20, 3), 6),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_attention_equals_library_softmax_attention_bfloat16(shape):
    L, Hq, Hkv, Dk, Dv, alias, lens, q_len = shape
    w = synth.small(27, L, Hq, Hkv, Dk, Dv, alias, lens, q_len)
    spec, kpool, vpool, table = build_cache(w, poison=0x7FC0, extra_blocks=2, param_format=BF)
    q = w.q_all().numpy()
    out16, out64 = oracle.attention(spec, kpool, vpool, q, table, w.final_lens(), w.sm_scale, return_f64=True)
    for l in range(L):
        for a, n in enumerate(w.final_lens()):
            kd = dense_rows(w, spec, kpool, table, l, a, n, Dk)
            vd = kd[:, :, :Dv] if alias else dense_rows(w, spec, vpool, table, l, a, n, Dv)
            vis = [n - (q_len - 1 - r) for r in range(q_len)]
            want = library_attention(q[l, a].astype(np.float64), kd, vd, w.n_rep, w.sm_scale, vis)
            assert np.allclose(out64[l, a], want, rtol=1e-11, atol=1e-12)
    assert not np.isnan(out64).any()
    # the pools really hold bfloat16 parameters: read as binary16 the same bits give another answer
    spec16 = oracle.make_spec(L, Hq, Hkv, Dk, Dv, alias)
    other = oracle.attention(spec16, kpool, vpool, q, table, w.final_lens(), w.sm_scale, return_f64=True)[1]
    assert not np.allclose(other, out64, rtol=1e-3, atol=1e-3, equal_nan=True)


def test_append_places_the_bfloat16_quantizer_output():
    w = synth.small(28, 2, 2, 2, 128, 64, False, (250, 7), 1)
    spec = oracle.make_spec(2, 2, 2, 128, 64, param_format=BF)
    table, nb = w.block_table()
    table = np.concatenate([table, [[nb], [nb + 1]]], axis=1).astype(np.int32)
    kpool, vpool = oracle.Pool(spec, 128, nb + 2, fill=0x7FC0), oracle.Pool(spec, 64, nb + 2, fill=0x7FC0)
    C_ = 10
    k_new = np.stack([np.stack([w.k_rows(l, a, 1000, 1000 + C_).numpy() for a in range(2)]) for l in range(2)])
    v_new = np.stack([np.stack([w.v_rows(l, a, 1000, 1000 + C_).numpy() for a in range(2)]) for l in range(2)])
    oracle.append(spec, kpool, vpool, k_new, v_new, table, w.seq_lens)
    kc, ks, kb = oracle.quantize(k_new, BF)
    vc, vs, vb = oracle.quantize(v_new, BF)
    assert not np.array_equal(ks, oracle.quantize(k_new)[1])
    for l in range(2):
        for a, n in enumerate(w.seq_lens):
            for c in range(C_):
                blk, slot = table[a, (n + c) // 256], (n + c) % 256
                assert np.array_equal(kpool.codes[l, blk, :, slot], kc[l, a, c])
                assert np.array_equal(kpool.scale[l, blk, :, slot], ks[l, a, c])
                assert np.array_equal(kpool.bias[l, blk, :, slot], kb[l, a, c])
                assert np.array_equal(vpool.codes[l, blk, :, slot], vc[l, a, c])
                assert np.array_equal(vpool.scale[l, blk, :, slot], vs[l, a, c])
                assert np.array_equal(vpool.bias[l, blk, :, slot], vb[l, a, c])


def test_unknown_format_is_rejected():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((1, 64), F16), param_format=2)
    with pytest.raises(ValueError):
        oracle.dequantize(np.zeros((1, 8), np.uint32), np.zeros((1, 1), np.uint16), np.zeros((1, 1), np.uint16), 7)
