"""GPU parity with the CPU oracle when scale and bias are stored as bfloat16 (Sec. 3.1, Sec. 3.2 and the appendix
"safetensors Q4 Format" name both bfloat16 and binary16): the codec bit-exact, every attention kernel within
|gpu - oracle| <= 2e-3 + 2e-3*|oracle| on the binary16 outputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import binding as b
from paper_2603_04428_amd import synth
from tests.gpu_util import DEV, bits, gpu_cache, host_cache, oracle_unit
from tests.util import tie_adjacent_rows_bf16
from tests.test_gpu_chunk import append_chunk_and_attend
from tests.test_gpu_decode import assert_close, run_gpu

pytestmark = pytest.mark.gpu
F16 = np.float16
BF = b.PARAMS_BF16
assert BF == oracle.BF16_PARAMS


def check_quantize(x_np):
    x = torch.from_numpy(x_np).to(DEV)
    codes, scale, bias = b.q4kv_quantize(x, param_format=BF)
    oc, os_, ob = oracle.quantize(x_np, BF)
    assert np.array_equal(bits(scale), os_), "scale bits"
    assert np.array_equal(bits(bias), ob), "bias bits"
    assert np.array_equal(bits(codes), oc), "codes"
    xh = b.q4kv_dequantize(codes, scale, bias, param_format=BF)
    assert np.array_equal(bits(xh), oracle.dequantize(oc, os_, ob, BF).view(np.uint16)), "dequantized"


@pytest.mark.parametrize("dim", [64, 256, 576])
def test_quantize_random_rows_bit_exact(dim):
    rng = np.random.default_rng(dim + 1)
    check_quantize(rng.standard_normal((1000 + 7, dim)).astype(F16))
    x = rng.standard_normal((333, dim))
    x[:, ::11] *= 8
    check_quantize(x.astype(F16))
    # the binary16 entry point and format 0 of the new one are the same thing
    xt = torch.from_numpy(x.astype(F16)).to(DEV)
    for u, v in zip(b.q4kv_quantize(xt), b.q4kv_quantize(xt, param_format=b.PARAMS_F16)):
        assert torch.equal(u, v)


def test_quantize_special_groups_bit_exact():
    rng = np.random.default_rng(0)
    rows = []
    ramp = np.tile(np.arange(16), 4).astype(np.float64)
    rows.append(ramp)
    rows.append(1000.5 + 0.5 * ramp)                              # bias rounds down by a whole code step, top clamps
    rows.append(1.005859375 + 0.125 * ramp)                       # bias rounds up past the minimum
    rows.append(np.full(64, 3.25))                                # constant group
    z = np.zeros(64); z[3] = 2.0 ** -24; rows.append(z)           # one subnormal step of range: scale 2^-24 / 15
    z = np.zeros(64); z[3] = 7 * 2.0 ** -24; rows.append(z)
    t = np.zeros(64); t[1] = 15; t[2:10] = [0.5, 1.5, 2.5, 3.5, 13.5, 14.5, 7.5, 8.5]; rows.append(t)   # ties
    nz = np.zeros(64); nz[0] = -0.0; nz[1] = 1.0; rows.append(nz)  # -0 is the first minimum
    pz = np.zeros(64); pz[5] = -0.0; pz[9] = 2.0; rows.append(pz)  # +0 first, -0 later
    tie = np.full(64, 1.00390625); tie[1] = 2.0; rows.append(tie)  # bias on a bfloat16 tie (to even: down)
    tie = np.full(64, 1.01171875); tie[1] = 2.0; rows.append(tie)  # (to even: up)
    check_quantize(np.stack(rows).astype(F16))
    check_quantize((rng.standard_normal((200, 64)) * 3e-6).astype(F16))          # subnormal inputs
    check_quantize((rng.standard_normal((200, 128)) * 1e-3).astype(F16))
    check_quantize((1000 + rng.standard_normal((300, 64))).astype(F16))          # bias error >> scale: heavy clamping
    check_quantize((-700 + 0.1 * rng.standard_normal((300, 64))).astype(F16))
    check_quantize(rng.uniform(-30000, 30000, (200, 64)).astype(F16))
    k = rng.integers(0, 15, (300, 64)) + 0.5                                     # values on code boundaries
    k[:, 0], k[:, 1] = 0, 15
    check_quantize(k.astype(F16))
    check_quantize((k * 0.37 - 2.0).astype(F16))
    allbits = np.arange(0, 0x7800, dtype=np.uint16)               # every finite binary16 magnitude below 32,768
    allbits = np.concatenate([allbits, allbits | 0x8000])
    rng.shuffle(allbits)
    check_quantize(allbits[: (len(allbits) // 64) * 64].view(F16).reshape(-1, 64))


def test_quantize_quotients_next_to_rounding_ties_bit_exact():
    """Quotients (x - bias_stored) / scale_stored on, just below and just above k + 0.5 for bfloat16-representable
    scales and biases: an approximate division flips some of these codes."""
    check_quantize(tie_adjacent_rows_bf16(8))


def test_dequantize_arbitrary_codes_bit_exact():
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 2 ** 32, (777, 32), dtype=np.uint64).astype(np.uint32)
    to_bf = lambda a: np.array([oracle.f2bf(v) for v in a.ravel()], np.uint16).reshape(a.shape)
    scale = to_bf(rng.standard_normal((777, 4)) * 0.3)
    bias = to_bf(rng.standard_normal((777, 4)) * 2)
    scale[5] = 0
    scale[6] = oracle.f2bf(2.0 ** -30)
    bias[7] = oracle.f2bf(60000.0)
    got = b.q4kv_dequantize(torch.from_numpy(codes.view(np.int32)).to(DEV), torch.from_numpy(scale.view(np.int16)).to(DEV),
                            torch.from_numpy(bias.view(np.int16)).to(DEV), param_format=BF)
    assert np.array_equal(bits(got), oracle.dequantize(codes, scale, bias, BF).view(np.uint16))


def test_unknown_format_is_an_argument_error():
    x = torch.zeros((4, 64), dtype=torch.float16, device=DEV)
    with pytest.raises(b.Q4KVError) as e:
        b.q4kv_quantize(x, param_format=2)
    assert e.value.code == -1
    spec = b.make_spec(1, 2, 2, 64, param_format=5)
    with pytest.raises(b.Q4KVError):
        b.q4kv_cache_bytes(spec, 10)


@pytest.mark.parametrize("alias", [False, True])
def test_append_bit_exact(alias):
    if alias:
        w = synth.small(23, 2, 16, 1, 576, 512, True, (250, 7, 600), 1)
    else:
        w = synth.small(23, 3, 4, 2, 128, 64, False, (250, 7, 600), 1)
    spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=BF)
    ospec, okp, ovp, otable = host_cache(w, param_format=BF)
    for a, n in enumerate(w.seq_lens):
        for i in range((n + 255) // 256):
            blk, m = table[a, i], min(n - 256 * i, 256)
            for gp, op in ((kpool, okp), (vpool, ovp)):
                if gp is None:
                    continue
                assert np.array_equal(bits(gp.codes[:, blk, :, :m]), op.codes[:, blk, :, :m])
                assert np.array_equal(bits(gp.scale[:, blk, :, :m]), op.scale[:, blk, :, :m])
                assert np.array_equal(bits(gp.bias[:, blk, :, :m]), op.bias[:, blk, :, :m])
    # the pools differ from what the binary16 format stores for the same rows
    _, k16, _, table16, _ = gpu_cache(w)
    assert not np.array_equal(bits(kpool.scale[:, table[0, 0], :, :7]), bits(k16.scale[:, table16[0, 0], :, :7]))


DECODE = [
    (2, 4, 2, 64, (37, 5, 300, 1)),
    (1, 8, 2, 128, (260, 700)),
    (1, 16, 8, 256, (513, 130)),
    (1, 4, 1, 128, (1500, 20)),
    (2, 16, 16, (192, 128), (37, 300, 1, 64)),
]


@pytest.mark.parametrize("shape", DECODE)
@pytest.mark.parametrize("split_tokens", [0, 256])
def test_decode_matches_oracle_small(shape, split_tokens):
    L, Hq, Hkv, D, lens = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    w = synth.small(33, L, Hq, Hkv, Dk, Dv, False, lens)
    spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=BF)          # poisoned: NaN parameters outside
    ospec, okp, ovp, otable = host_cache(w, param_format=BF)
    got = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
    assert_close(got, want, f"{shape} split {split_tokens}")
    # windows and a layer range go through the same kernel
    got = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens, window=48)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale, window=48)
    assert_close(got, want, f"{shape} window 48")


@pytest.mark.parametrize("shape", [(1, (37,)), (2, (1, 64, 65, 300)), (1, (1500, 20)), (1, (4200,))])
def test_latent_decode_matches_oracle_small(shape):
    L, lens = shape
    w = synth.small(43, L, 16, 1, 576, 512, True, lens)
    spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=BF)
    ospec, okp, ovp, otable = host_cache(w, param_format=BF)
    got = run_gpu(w, spec, kpool, vpool, table_d, list(lens))
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
    assert_close(got, want, f"{shape}")


CHUNK = [
    (2, 4, 2, 128, (300, 0, 70), 70),
    (1, 2, 2, 256, (513, 64), 129),
    (1, 16, 8, 256, (100,), 64),
    (1, 8, 1, 64, (1000, 40), 33),
    (1, 4, 4, (192, 128), (300, 0), 130),
]


@pytest.mark.parametrize("shape", CHUNK)
def test_chunk_matches_oracle_small(shape):
    L, Hq, Hkv, D, lens, C = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    w = synth.small(41, L, Hq, Hkv, Dk, Dv, False, lens, q_len=C)
    got, _ = append_chunk_and_attend(w, param_format=BF)
    ospec, okp, ovp, otable = host_cache(w, param_format=BF)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, w.final_lens(), w.sm_scale)
    assert_close(got, want, f"{shape}")


def test_headline_config_sampled_units():
    """Config 2 (Gemma-shaped, 10 ragged agents, 48 layers) at full size with bfloat16 parameters, in the launch
    configuration the benchmark times; the oracle recomputes a seeded sample of units from the generator alone."""
    w = synth.config(2)
    spec, kpool, vpool, table, table_d = gpu_cache(w, poison=False, extra_blocks=0, param_format=BF)
    got = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens)
    assert not np.isnan(got.astype(np.float32)).any()
    rng = np.random.default_rng(12)
    shortest, longest = int(np.argmin(w.seq_lens)), int(np.argmax(w.seq_lens))
    units = {(0, shortest, 0), (w.num_layers - 1, longest, w.num_kv_heads - 1)}
    while len(units) < 6:
        units.add((int(rng.integers(w.num_layers)), int(rng.integers(w.num_agents)), int(rng.integers(w.num_kv_heads))))
    R = w.n_rep
    for (l, a, h) in sorted(units):
        want = oracle_unit(w, l, a, h, w.seq_lens[a], param_format=BF)
        assert_close(got[l, a, :, h * R:(h + 1) * R], want, f"unit layer {l} agent {a} kv head {h}")
