"""q4kv_batched_attention_static (the entry point for callers that cannot allocate): its output against
q4kv_batched_attention's on the same arguments, bit for bit (the same kernels run, the workspace alone differs),
and against the CPU oracle within |gpu - oracle| <= 2e-3 + 2e-3*|oracle|; two calls in a row, the second smaller,
so that the second call finds the first call's contents in the library's fixed array."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import binding as b
from paper_2603_04428_amd import synth
from tests.gpu_util import DEV, gpu_cache, host_cache
from tests.util import within_tol

pytestmark = pytest.mark.gpu


def both_entry_points(w, spec, kpool, vpool, table_d, lens, layer_begin, layer_end, split_tokens=0, window=0):
    q = w.q_all(DEV, layer_begin, layer_end)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    msl = max(max(lens), 1)
    shape = (layer_end - layer_begin, len(lens), 1, spec.num_q_heads, spec.v_dim)
    out_static = torch.full(shape, float("nan"), dtype=torch.float16, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    b.q4kv_batched_attention_static(spec, kpool, vpool, q, out_static, table_d, sl, msl, w.sm_scale, window,
                                    split_tokens, layer_begin, layer_end)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # nothing came from torch's allocator either
    out_ws = b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, sl, msl, w.sm_scale, window, split_tokens,
                                      layer_begin, layer_end)
    torch.cuda.synchronize()
    return out_static.cpu().numpy(), out_ws.cpu().numpy(), q.cpu().numpy()


def check(w, spec, kpool, vpool, table_d, ospec, okp, ovp, otable, lens, layer_begin, layer_end, **kw):
    got, ref, q = both_entry_points(w, spec, kpool, vpool, table_d, lens, layer_begin, layer_end, **kw)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16)), "static-scratch call differs from the workspace call"
    want = oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale, window=kw.get("window", 0),
                            layer_begin=layer_begin, layer_end=layer_end)
    ok, over, worst = within_tol(got, want)
    assert ok, f"exceeds 2e-3 abs/rel by {over:.3e} (max abs err {worst:.3e})"


def test_two_calls_in_a_row_the_second_smaller():
    w = synth.small(71, 3, 8, 2, 128, 128, False, (700, 130, 2000, 0, 65))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    args = (w, spec, kpool, vpool, table_d, ospec, okp, ovp, otable)
    check(*args, list(w.seq_lens), 0, 3)                               # all layers, every agent at full length
    check(*args, [90, 5, 300, 0, 1], 1, 2)                             # one layer, shorter lengths: a smaller plan
    check(*args, list(w.seq_lens), 0, 3, split_tokens=256, window=100)  # and a larger one again


def test_shared_latent_shape_and_a_second_smaller_call():
    w = synth.small(72, 2, 16, 1, 576, 512, True, (900, 130, 37))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    args = (w, spec, kpool, vpool, table_d, ospec, okp, ovp, otable)
    check(*args, list(w.seq_lens), 0, 2)
    check(*args, [64, 3, 0], 0, 1)


def test_a_call_that_does_not_fit_is_refused_and_launches_nothing():
    w = synth.small(73, 1, 8, 2, 128, 128, False, (300,))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    big = b.make_spec(64, 16, 8, 256, 256)                 # 64 layers x 64 agents at 32K tokens: far beyond 16 MiB
    assert b.q4kv_attention_workspace_bytes(big, 64, 1, 32768, 0, 64) > b.STATIC_SCRATCH_BYTES
    q = torch.zeros((64, 64, 1, 16, 256), dtype=torch.float16, device=DEV)
    out = torch.full((64, 64, 1, 16, 256), 7.0, dtype=torch.float16, device=DEV)
    with pytest.raises(b.Q4KVError) as e:
        b.q4kv_batched_attention_static(big, kpool, vpool, q, out, table_d.expand(64, -1).contiguous(),
                                        torch.zeros(64, dtype=torch.int32, device=DEV), 32768, 1.0)
    assert e.value.code == -4 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    # the entry point still works afterwards
    ospec, okp, ovp, otable = host_cache(w)
    check(w, spec, kpool, vpool, table_d, ospec, okp, ovp, otable, [300], 0, 1)
