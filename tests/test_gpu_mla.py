"""GPU parity of q4kv_batched_attention (decode) on the shared-latent spec of Sec. 3.6: one 576-wide Q4 row per
token is K in full and V in its first 512 elements, 16 query heads read it (DeepSeek-V2-Lite-shaped).

Tolerance as for the other attention tests: |gpu - oracle| <= 2e-3 + 2e-3*|oracle| element-wise, the oracle's
binary64 result rounded to binary16 last."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import binding as b
from paper_2603_04428_amd import synth
from tests.gpu_util import DEV, bits, gpu_cache, host_cache, oracle_unit
from tests.test_gpu_decode import assert_close, run_gpu

pytestmark = pytest.mark.gpu

SMALL = [
    # layers, seq_lens  (tiles with ragged tails, block boundaries, several agents per wave and waves per agent)
    (1, (37,)),
    (2, (1, 64, 65, 300)),
    (1, (255, 256, 257, 5)),
    (1, (1500, 20)),
    (1, (4200,)),
]


def mla(seed, layers, lens):
    return synth.small(seed, layers, 16, 1, 576, 512, True, lens)


@pytest.mark.parametrize("shape", SMALL)
@pytest.mark.parametrize("split_tokens", [0, 256, 1024])
def test_latent_decode_matches_oracle_small(shape, split_tokens):
    L, lens = shape
    w = mla(41, L, lens)
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    assert vpool is None
    ospec, okp, ovp, otable = host_cache(w)
    for a, n in enumerate(lens):
        blk, m = table[a, 0], min(n, 256)
        assert np.array_equal(bits(kpool.codes[:, blk, :, :m]), okp.codes[:, blk, :, :m])
    got = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
    assert_close(got, want, f"{shape} split {split_tokens}")


def test_latent_edge_cases_zero_length_poison_window_layer_range_and_bad_blocks():
    w = mla(42, 3, (300, 0, 77, 600))
    spec, kpool, vpool, table, table_d = gpu_cache(w, poison=True, extra_blocks=2)
    ospec, okp, ovp, otable = host_cache(w)
    lens = list(w.seq_lens)
    q = w.q_all().numpy()
    got = run_gpu(w, spec, kpool, vpool, table_d, lens)
    want = oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale)
    assert_close(got, want, "ragged with an empty agent")
    assert not got[:, 1].view(np.uint16).any()                       # zero cached tokens -> zeros
    again = run_gpu(w, spec, kpool, vpool, table_d, lens)
    assert np.array_equal(got.view(np.uint16), again.view(np.uint16)), "run-to-run identical"
    short = [100, 0, 1, 300]
    assert_close(run_gpu(w, spec, kpool, vpool, table_d, short),
                 oracle.attention(ospec, okp, ovp, q, otable, short, w.sm_scale), "shortened")
    for win in (1, 50, 256, 500):
        assert_close(run_gpu(w, spec, kpool, vpool, table_d, lens, split_tokens=256, window=win),
                     oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale, window=win), f"window {win}")
    g = run_gpu(w, spec, kpool, vpool, table_d, lens, layer_begin=1, layer_end=3)
    assert_close(g, want[1:3], "layers 1..2")
    # a block id outside the pool hides its 256 tokens: agent 3 keeps blocks 0 and 2 (256 + 88 tokens)
    bad = table_d.clone()
    bad[3, 1] = 10_000
    got_bad = run_gpu(w, spec, kpool, vpool, bad, lens)
    spec1 = oracle.make_spec(3, 16, 1, 576, 512, True)
    kp = oracle.Pool(spec1, 576, 2)
    for name in ("codes", "scale", "bias"):
        getattr(kp, name)[:, 0] = getattr(okp, name)[:, otable[3, 0]]
        getattr(kp, name)[:, 1] = getattr(okp, name)[:, otable[3, 2]]
    want_bad = oracle.attention(spec1, kp, None, q[:, 3:4], np.array([[0, 1]], np.int32), [344], w.sm_scale)
    assert_close(got_bad[:, 3:4], want_bad, "masked block")
    assert_close(got_bad[:, :3], want[:, :3], "agents beside the masked block")


@pytest.mark.parametrize("param_format", [0, 1])
def test_latent_tolerance_does_not_depend_on_the_draw(param_format):
    """Agents of a handful of tokens, twenty draws: here one or two products p * s make up an output, and their
    rounding decides the margin (the kernel carries p * s in two binary16 terms for this case)."""
    lens = (5, 3, 9, 20)
    for seed in range(100, 120):
        w = mla(seed, 1, lens)
        spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=param_format)
        ospec, okp, ovp, otable = host_cache(w, param_format=param_format)
        got = run_gpu(w, spec, kpool, vpool, table_d, list(lens))
        want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
        assert_close(got, want, f"seed {seed} format {param_format}")


def test_latent_per_layer_windows_match_oracle():
    w = mla(44, 4, (700, 90, 0, 1300))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    lens = list(w.seq_lens)
    q = w.q_all().numpy()
    for windows in ([0, 128, 0, 1000], [1, 64, 65, 5000]):
        got = run_gpu(w, spec, kpool, vpool, table_d, lens, split_tokens=256, window=windows)
        want = oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale, window_per_layer=windows)
        assert_close(got, want, f"windows {windows}")


def test_latent_outliers_and_large_scores():
    """Sharp softmax (scores far apart, running maximum moving late) and large-magnitude channels."""
    w = mla(43, 1, (900, 130))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    q = w.q_all()
    for scale in (0.25, 1.0):
        got = b.q4kv_batched_attention(spec, kpool, vpool, q.to(DEV), table_d,
                                       torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV), max(w.seq_lens),
                                       scale, 0, 0, 0, None)
        torch.cuda.synchronize()
        want = oracle.attention(ospec, okp, ovp, q.numpy(), otable, w.seq_lens, scale)
        assert_close(got.cpu().numpy(), want, f"sm_scale {scale}")


def test_config3_full_size_sampled_units():
    """Config 3 (5 agents x 32,768 tokens x 27 layers, 576/512 latent, 16 heads) at full size, all layers in one
    call with the default split, as the benchmark launches it; the oracle recomputes a seeded sample of
    (layer, agent) units from the generator alone."""
    w = synth.config(3)
    spec, kpool, vpool, table, table_d = gpu_cache(w, poison=False, extra_blocks=0)
    got = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens)
    assert not np.isnan(got.astype(np.float32)).any()
    rng = np.random.default_rng(3)
    units = {(0, 0), (w.num_layers - 1, w.num_agents - 1)}
    while len(units) < 5:
        units.add((int(rng.integers(w.num_layers)), int(rng.integers(w.num_agents))))
    for (l, a) in sorted(units):
        want = oracle_unit(w, l, a, 0, w.seq_lens[a])
        assert_close(got[l, a], want, f"config 3 unit layer {l} agent {a}")
    # outputs are convex combinations of latent rows, whose outlier channels reach 8 x the N(0,1) table's range
    assert float(np.abs(got.astype(np.float32)).max()) < 8 * 4.5
