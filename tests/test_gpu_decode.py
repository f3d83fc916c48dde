"""GPU parity of q4kv_batched_attention (decode, q_len = 1) with the CPU oracle.

Tolerance (stated by the project brief for binary16 attention outputs): |gpu - oracle| <= 2e-3 + 2e-3*|oracle|
element-wise, the oracle's binary64 result rounded to binary16 last."""
import numpy as np
import pytest
import torch

import oracle
from paper_2603_04428_amd import binding as b
from paper_2603_04428_amd import synth
from tests.gpu_util import DEV, bits, gpu_cache, host_cache, oracle_unit
from tests.util import within_tol

pytestmark = pytest.mark.gpu


def run_gpu(w, spec, kpool, vpool, table_d, lens, split_tokens=0, window=0, q=None, layer_begin=0, layer_end=None):
    q = w.q_all(DEV, layer_begin, layer_end) if q is None else q
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    msl = max(max(lens), 1)
    out = b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, sl, msl, w.sm_scale, window, split_tokens,
                                   layer_begin, layer_end)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def assert_close(got, want, what=""):
    ok, over, worst = within_tol(got, want)
    assert ok, f"{what}: exceeds 2e-3 abs/rel by {over:.3e} (max abs err {worst:.3e})"
    assert not np.isnan(got.astype(np.float32)).any()


SMALL = [
    # layers, Hq, Hkv, D, seq_lens  (several 64-token tiles, ragged tails, several blocks)
    (2, 4, 2, 64, (37, 5, 300, 1)),
    (1, 8, 2, 128, (260, 700)),
    (2, 2, 2, 128, (1, 64, 65, 255, 256, 257)),
    (1, 16, 8, 256, (513, 130)),
    (1, 4, 4, 256, (90,)),
    (1, 8, 2, 64, (1000,)),
    (1, 4, 1, 128, (1500, 20)),
    # eight query heads per KV head: two passes of four heads on the value side
    (1, 8, 1, 64, (200, 70)),
    (1, 16, 2, 128, (300, 5)),
    (1, 8, 1, 256, (150, 65)),
]


PER_HEAD_MLA = [
    # the decompressed per-head cache of Sec. 3.6: keys 192 wide (128 + 64 rotary), values 128 wide, one KV head
    # per query head (K and V pools of different row widths, three K groups per row)
    (2, 16, 16, (192, 128), (37, 300, 1, 64)),
    (1, 4, 4, (192, 128), (700, 257)),
    (1, 8, 4, (192, 128), (513,)),
    (1, 8, 1, (192, 128), (130, 3)),
]


# split_tokens 4,096 makes a workgroup's range long enough (64 tiles) for the kernel's other way of sharing it out: a
# contiguous quarter per wave instead of tiles in turn
@pytest.mark.parametrize("shape", SMALL + PER_HEAD_MLA)
@pytest.mark.parametrize("split_tokens", [0, 256, 512, 4096])
def test_decode_matches_oracle_small(shape, split_tokens):
    L, Hq, Hkv, D, lens = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    w = synth.small(31, L, Hq, Hkv, Dk, Dv, False, lens)
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    # the two quantizers must agree before attention is compared (same Q4 cache on both sides)
    for a, n in enumerate(lens):
        blk = table[a, 0]
        m = min(n, 256)
        assert np.array_equal(bits(kpool.codes[:, blk, :, :m]), okp.codes[:, blk, :, :m])
    got = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
    assert_close(got, want, f"{shape} split {split_tokens}")


def test_config0_full_tensor():
    """Llama-3.1-8B-shaped, 1 agent, 1 layer, 1,024 cached tokens, every output element."""
    w = synth.config(0)
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    got = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, w.seq_lens, w.sm_scale)
    assert_close(got, want, "config 0")


def test_edge_cases_zero_length_poison_window_and_layer_range():
    w = synth.small(33, 3, 4, 2, 128, 128, False, (300, 0, 77, 512))
    spec, kpool, vpool, table, table_d = gpu_cache(w, poison=True, extra_blocks=2)
    ospec, okp, ovp, otable = host_cache(w)
    lens = list(w.seq_lens)
    q = w.q_all().numpy()
    got = run_gpu(w, spec, kpool, vpool, table_d, lens)
    want = oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale)
    assert_close(got, want, "ragged with an empty agent")
    assert not got[:, 1].view(np.uint16).any()                       # zero cached tokens -> zeros
    # shorter visible lengths than what is cached: slots past seq_len are never read
    short = [100, 0, 1, 300]
    assert_close(run_gpu(w, spec, kpool, vpool, table_d, short),
                 oracle.attention(ospec, okp, ovp, q, otable, short, w.sm_scale), "shortened")
    # sliding window, also one that hides whole splits
    for win in (1, 50, 256, 1000):
        assert_close(run_gpu(w, spec, kpool, vpool, table_d, lens, split_tokens=256, window=win),
                     oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale, window=win), f"window {win}")
    # a layer sub-range
    g = run_gpu(w, spec, kpool, vpool, table_d, lens, layer_begin=1, layer_end=3)
    assert_close(g, want[1:3], "layers 1..2")


def test_per_layer_windows_match_oracle():
    """Global and sliding-window layers interleaved (Sec. 3.6), several distinct windows, also a layer sub-range
    and windows that hide whole shares of the tile stream."""
    w = synth.small(37, 6, 8, 2, 128, 128, False, (1500, 0, 300, 77, 2100))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    lens = list(w.seq_lens)
    q = w.q_all().numpy()
    for windows in ([0, 256, 256, 0, 1, 1000], [64] * 6, [0] * 6, [5000, 100, 0, 100, 5000, 300]):
        for st in (0, 256):
            got = run_gpu(w, spec, kpool, vpool, table_d, lens, split_tokens=st, window=windows)
            want = oracle.attention(ospec, okp, ovp, q, otable, lens, w.sm_scale, window_per_layer=windows)
            assert_close(got, want, f"windows {windows} split {st}")
    same = run_gpu(w, spec, kpool, vpool, table_d, lens, window=[64] * 6)
    one = run_gpu(w, spec, kpool, vpool, table_d, lens, window=64)
    assert np.array_equal(same.view(np.uint16), one.view(np.uint16)), "equal windows = the single-window call"
    windows = [0, 256, 256, 0, 1, 1000]
    part = run_gpu(w, spec, kpool, vpool, table_d, lens, window=windows[2:5], layer_begin=2, layer_end=5)
    want = oracle.attention(ospec, okp, ovp, q[2:5], otable, lens, w.sm_scale, window_per_layer=windows,
                            layer_begin=2, layer_end=5)
    assert_close(part, want, "layers 2..4 with their windows")
    with pytest.raises(ValueError):
        b.q4kv_batched_attention(spec, kpool, vpool, w.q_all(DEV), table_d,
                                 torch.tensor(lens, dtype=torch.int32, device=DEV), max(lens), w.sm_scale,
                                 [0] * 5)                                  # 5 windows for 6 layers


def test_split_invariance_and_determinism():
    w = synth.small(34, 1, 8, 2, 128, 128, False, (2000, 900))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, w.seq_lens, w.sm_scale)
    outs = {}
    for st in (256, 512, 1024, 2048):
        outs[st] = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens, st)
        assert_close(outs[st], want, f"split {st}")
        again = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens, st)
        assert np.array_equal(outs[st].view(np.uint16), again.view(np.uint16)), "run-to-run identical"


def test_batch_equals_single_agent_calls_and_block_placement():
    w = synth.small(35, 1, 4, 2, 64, 64, False, (300, 513, 40))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    full = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens, 256)
    q = w.q_all(DEV)
    for a in range(3):
        one = run_gpu(w, spec, kpool, vpool, table_d[a:a + 1].contiguous(), w.seq_lens[a:a + 1], 256,
                      q=q[:, a:a + 1].contiguous())
        # the token ranges handed to wavefronts depend on the whole batch, so the summation order (not the
        # result beyond rounding) differs between a batched and a single-agent call
        assert_close(one[:, 0], full[:, a].astype(np.float64), f"agent {a} alone vs in the batch")
        ok, _, worst = within_tol(one[:, 0], full[:, a], atol=2e-4, rtol=1e-3)
        assert ok, worst
    # move every block to another physical slot: identical bits
    nb = kpool.num_blocks
    perm = torch.randperm(nb, generator=torch.Generator().manual_seed(0)).to(DEV)
    k2, v2 = b.Pool(spec, 64, nb, DEV, True), b.Pool(spec, 64, nb, DEV, True)
    for src, dst in ((kpool, k2), (vpool, v2)):
        for name in ("codes", "scale", "bias"):
            getattr(dst, name)[:, perm] = getattr(src, name)
    table2 = perm[table_d.long()].to(torch.int32).contiguous()
    moved = run_gpu(w, spec, k2, v2, table2, w.seq_lens, 256)
    assert np.array_equal(moved.view(np.uint16), full.view(np.uint16))


def test_block_ids_outside_the_pool_are_masked():
    w = synth.small(36, 1, 2, 1, 64, 64, False, (600,))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    bad = table_d.clone()
    bad[0, 1] = 10_000                                               # tokens 256..511 unreachable
    got = run_gpu(w, spec, kpool, vpool, bad, [600])
    # oracle on the reachable tokens: a two-block cache made of the agent's first and third block
    q = w.q_all().numpy()
    spec1 = oracle.make_spec(1, 2, 1, 64, 64)
    kp, vp = oracle.Pool(spec1, 64, 2), oracle.Pool(spec1, 64, 2)
    for src, dst in ((okp, kp), (ovp, vp)):
        for name in ("codes", "scale", "bias"):
            getattr(dst, name)[0, 0] = getattr(src, name)[0, otable[0, 0]]
            getattr(dst, name)[0, 1] = getattr(src, name)[0, otable[0, 2]]
    want = oracle.attention(spec1, kp, vp, q, np.array([[0, 1]], np.int32), [344], w.sm_scale)
    assert_close(got, want, "masked block")


@pytest.mark.parametrize("cfg,split_tokens", [(1, 0), (2, 0), (2, 256), (2, 2048)])
def test_full_size_configs_sampled_units(cfg, split_tokens):
    """Configs 1 (Llama-shaped, 5 x 4,096, 32 layers) and 2 (Gemma-shaped, 10 ragged agents, 48 layers) at full
    size, in the launch configuration the benchmark times (all layers in one call, default split), and config 2
    also with the smallest and a larger chunk (waves then fetch many / a few chunks from the queues).  The oracle
    recomputes a seeded sample of (layer, agent, kv head) units from the generator alone."""
    w = synth.config(cfg)
    spec, kpool, vpool, table, table_d = gpu_cache(w, poison=False, extra_blocks=0)
    got = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens, split_tokens)
    assert not np.isnan(got.astype(np.float32)).any()
    # which wave computes which chunk varies from run to run; the result does not
    again = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens, split_tokens)
    assert np.array_equal(got.view(np.uint16), again.view(np.uint16)), "run-to-run identical"
    rng = np.random.default_rng(cfg)
    shortest, longest = int(np.argmin(w.seq_lens)), int(np.argmax(w.seq_lens))
    units = {(0, shortest, 0), (w.num_layers - 1, longest, w.num_kv_heads - 1), (0, longest, 3),
             (w.num_layers - 1, shortest, 5)}
    while len(units) < 10:
        units.add((int(rng.integers(w.num_layers)), int(rng.integers(w.num_agents)), int(rng.integers(w.num_kv_heads))))
    R = w.n_rep
    for (l, a, h) in sorted(units):
        want = oracle_unit(w, l, a, h, w.seq_lens[a])
        assert_close(got[l, a, :, h * R:(h + 1) * R], want, f"config {cfg} unit layer {l} agent {a} kv head {h}")
    # property at any size: outputs are convex combinations of V rows, so bounded by the cache's value range
    assert float(np.abs(got.astype(np.float32)).max()) < 6.0


def test_per_head_mla_full_size_sampled_units():
    """The decompressed per-head MLA cache (keys 192, values 128, 16 KV heads, 27 layers, 5 agents x 8,192 tokens) in
    the launch configuration the benchmark times; the oracle recomputes a seeded sample of units from the generator."""
    w = synth.per_head_mla_config()
    spec, kpool, vpool, table, table_d = gpu_cache(w, poison=False, extra_blocks=0)
    got = run_gpu(w, spec, kpool, vpool, table_d, w.seq_lens)
    assert not np.isnan(got.astype(np.float32)).any()
    rng = np.random.default_rng(5)
    units = {(0, 0, 0), (w.num_layers - 1, w.num_agents - 1, w.num_kv_heads - 1)}
    while len(units) < 8:
        units.add((int(rng.integers(w.num_layers)), int(rng.integers(w.num_agents)), int(rng.integers(w.num_kv_heads))))
    for (l, a, h) in sorted(units):
        want = oracle_unit(w, l, a, h, w.seq_lens[a])
        assert_close(got[l, a, :, h:h + 1], want, f"per-head MLA unit layer {l} agent {a} kv head {h}")
    assert float(np.abs(got.astype(np.float32)).max()) < 6.0


def test_decode_call_replays_from_a_graph():
    """The library only enqueues kernels (no allocation, no memset, no synchronisation), so a call can be recorded
    into a graph; every replay, with eager work between the replays, gives the eager call's bits."""
    w = synth.small(37, 3, 8, 2, 128, 128, False, (700, 90, 257))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    q = w.q_all(DEV)
    sl = torch.tensor(w.seq_lens, dtype=torch.int32, device=DEV)
    msl = max(w.seq_lens)
    ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, w.num_agents, 1, msl, 256, w.num_layers), dtype=torch.uint8,
                     device=DEV)
    out = torch.empty((w.num_layers, w.num_agents, 1, w.num_q_heads, w.v_dim), dtype=torch.float16, device=DEV)

    def call():
        b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, sl, msl, w.sm_scale, [0, 64, 0], 256, 0, None, out, ws)

    call()
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for i in range(4):
        out.zero_()
        ws.fill_(0xFF)                        # eager work between replays; the call must not depend on old workspace bits
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {i}"
    # new lengths are picked up by a replay: the plan is rebuilt on the device from seq_len every time
    sl.copy_(torch.tensor([300, 90, 1], dtype=torch.int32))
    graph.replay()
    torch.cuda.synchronize()
    replayed = out.clone()
    call()
    torch.cuda.synchronize()
    assert torch.equal(out, replayed)


def test_host_threads_on_their_own_streams():
    """Calls that overlap in time from several host threads, each on a stream of its own with its own output and
    workspace, give bit for bit what the same calls give one after the other (the boundary promises this)."""
    import threading
    w = synth.small(51, 2, 8, 2, 128, 128, False, (700, 90, 1300, 5))
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    lens = list(w.seq_lens)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    q = w.q_all(DEV)
    x = torch.randn((4096, 128), generator=torch.Generator().manual_seed(5)).to(torch.float16).to(DEV)
    variants = [dict(window=0, split_tokens=0), dict(window=100, split_tokens=256), dict(window=0, split_tokens=512),
                dict(window=[0, 64], split_tokens=0)]

    def work(i):
        out = b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, sl, max(lens), w.sm_scale, **variants[i % 4])
        codes, scale, bias = b.q4kv_quantize(x[i * 512:(i + 2) * 512])
        return out, codes, scale, bias

    serial = [work(i) for i in range(6)]
    torch.cuda.synchronize()
    results, errors = [None] * 6, []

    def worker(i):
        try:
            st = torch.cuda.Stream()
            with torch.cuda.stream(st):
                for _ in range(20):
                    r = work(i)
                st.synchronize()
            results[i] = r
        except Exception as e:      # noqa: BLE001 - reported below
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(6)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i in range(6):
        for got, want in zip(results[i], serial[i]):
            assert torch.equal(got, want), f"thread {i}"


WIDE_V = [
    # Hq, Hkv, (Dk, Dv): every kernel template (64 / 128 / 256 / 192-128 wide) x 1, 2, 4, 8 query heads per KV head
    (1, 1, 64), (4, 2, 64), (4, 1, 64), (8, 1, 64),
    (2, 2, 128), (4, 2, 128), (8, 2, 128), (8, 1, 128),
    (1, 1, 256), (4, 2, 256), (4, 1, 256), (8, 1, 256),
    (2, 2, (192, 128)), (2, 1, (192, 128)), (4, 1, (192, 128)), (8, 1, (192, 128)),
]


@pytest.mark.parametrize("param_format", [0, 1], ids=["f16_params", "bf16_params"])
@pytest.mark.parametrize("shape", WIDE_V)
def test_decode_tolerance_with_wide_value_groups(shape, param_format):
    """Value groups spanning 20 to 45 (a quarter of the V channels multiplied by 8) and contexts of 3 to 20 tokens,
    twenty draws: an output is then a handful of products p * s * c with c * s up to the group's range, and nothing
    averages their rounding out.  With p * s in one binary16 term the error reaches 2^-12 of the range (1e-2 here);
    the kernel carries it in two terms."""
    Hq, Hkv, D = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    lens = (5, 3, 9, 20)
    for seed in range(200, 220):
        w = synth.small(seed, 1, Hq, Hkv, Dk, Dv, False, lens, wide_v=True)
        spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=param_format)
        ospec, okp, ovp, otable = host_cache(w, param_format=param_format)
        got = run_gpu(w, spec, kpool, vpool, table_d, list(lens))
        want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
        assert_close(got, want, f"{shape} seed {seed} format {param_format}")
    # and a longer context with the same values (several tiles, two waves meeting in a unit)
    w = synth.small(221, 1, Hq, Hkv, Dk, Dv, False, (700, 130), wide_v=True)
    spec, kpool, vpool, table, table_d = gpu_cache(w, param_format=param_format)
    ospec, okp, ovp, otable = host_cache(w, param_format=param_format)
    got = run_gpu(w, spec, kpool, vpool, table_d, list(w.seq_lens), split_tokens=256)
    want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(w.seq_lens), w.sm_scale)
    assert_close(got, want, f"{shape} long format {param_format}")


MANY_RECORDS = [
    # layers, Hq, Hkv, D, seq_lens: one or two long units cut into 4-tile ranges -- 20 to 36 records per unit, more than
    # the 16 the merge loads in one batch -- beside short and empty ones
    (1, 4, 1, 128, (5000,)),
    (1, 2, 1, 256, (9000, 0, 4100)),
    (2, 8, 2, 64, (6000, 70)),
    (1, 4, 4, (192, 128), (5200,)),
]


@pytest.mark.parametrize("shape", MANY_RECORDS)
@pytest.mark.parametrize("split_tokens", [256, 1024, 4096])
def test_units_shared_by_many_workgroups(shape, split_tokens):
    L, Hq, Hkv, D, lens = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    w = synth.small(41, L, Hq, Hkv, Dk, Dv, False, lens)
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    q = w.q_all().numpy()
    got = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens)
    assert_close(got, oracle.attention(ospec, okp, ovp, q, otable, list(lens), w.sm_scale), f"{shape} split {split_tokens}")
    again = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens)
    assert np.array_equal(got.view(np.uint16), again.view(np.uint16)), "records are merged in record order: identical reruns"
    win = run_gpu(w, spec, kpool, vpool, table_d, list(lens), split_tokens, window=3000)
    assert_close(win, oracle.attention(ospec, okp, ovp, q, otable, list(lens), w.sm_scale, window=3000),
                 f"{shape} split {split_tokens} window 3000")


@pytest.mark.parametrize("shape", [(3, 8, 2, 128, False, (1500, 0, 300, 77, 2100)), (2, 4, 1, 256, False, (5000, 130)),
                                   (2, 16, 1, (576, 512), True, (900, 130, 0, 37))])
def test_planned_calls_equal_plain_calls(shape):
    """q4kv_decode_plan once, then one q4kv_batched_attention_planned call per layer on the same workspace (the decode
    loop of a forward pass): bit-identical to q4kv_batched_attention, within tolerance of the oracle, also when the
    workspace is used again and again (the arrival counters are back at zero after every call) and with a window."""
    L, Hq, Hkv, D, alias, lens = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    w = synth.small(51, L, Hq, Hkv, Dk, Dv, alias, lens)
    spec, kpool, vpool, table, table_d = gpu_cache(w)
    ospec, okp, ovp, otable = host_cache(w)
    lens = list(lens)
    sl = torch.tensor(lens, dtype=torch.int32, device=DEV)
    msl = max(lens)
    q = w.q_all(DEV)
    for window, split in ((0, 0), (200, 256), (0, 256)):
        ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, len(lens), 1, msl, split, 1), dtype=torch.uint8, device=DEV)
        ws.fill_(0xAB)                                              # contents before the plan call do not matter
        b.q4kv_decode_plan(spec, sl, msl, ws, window=window, split_tokens=split, layers_in_call=1)
        want = oracle.attention(ospec, okp, ovp, q.cpu().numpy(), otable, lens, w.sm_scale, window=window)
        for rep in range(3):                                        # the same plan serves every layer, three times over
            out = torch.full((L, len(lens), 1, Hq, Dv), float("nan"), dtype=torch.float16, device=DEV)
            for l in range(L):
                b.q4kv_batched_attention_planned(spec, kpool, vpool, q[l:l + 1], out[l:l + 1], table_d, msl, w.sm_scale, ws,
                                                 window=window, split_tokens=split, layer_begin=l, layer_end=l + 1)
            torch.cuda.synchronize()
            plain = torch.cat([b.q4kv_batched_attention(spec, kpool, vpool, q[l:l + 1], table_d, sl, msl, w.sm_scale, window,
                                                        split, l, l + 1) for l in range(L)])
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int16), plain.view(torch.int16)), f"window {window} split {split} rep {rep}"
            assert_close(out.cpu().numpy(), want, f"planned, window {window} split {split}")
    # a workspace prepared for other arguments: the planned call does nothing
    out = torch.full((1, len(lens), 1, Hq, Dv), 7.0, dtype=torch.float16, device=DEV)
    b.q4kv_batched_attention_planned(spec, kpool, vpool, q[:1], out, table_d, msl, w.sm_scale, ws, window=5, split_tokens=256,
                                     layer_begin=0, layer_end=1)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


@pytest.mark.parametrize("v_mult", [1.4, 1.6, 2.0])
@pytest.mark.parametrize("shape", [(4, 1, 64), (8, 2, 128), (8, 1, 128), (4, 1, 256), (4, 1, (192, 128))])
def test_decode_tolerance_where_the_second_term_is_optional(shape, v_mult):
    """Four and eight query heads per KV head take the second term of p * s per tile, only when a value scale of the
    tile exceeds 0.49.  Values of 1.4 to 2.0 times unit variance put the scales (0.4 to 0.65) on both sides of that
    line, tile by tile, on contexts short enough that a single rounding decides an output."""
    Hq, Hkv, D = shape
    Dk, Dv = D if isinstance(D, tuple) else (D, D)
    lens = (5, 3, 9, 20, 70)
    for seed in range(300, 312):
        w = synth.small(seed, 1, Hq, Hkv, Dk, Dv, False, lens, wide_v=True, v_mult=v_mult, v_every=1)
        spec, kpool, vpool, table, table_d = gpu_cache(w)
        ospec, okp, ovp, otable = host_cache(w)
        got = run_gpu(w, spec, kpool, vpool, table_d, list(lens))
        want = oracle.attention(ospec, okp, ovp, w.q_all().numpy(), otable, list(lens), w.sm_scale)
        assert_close(got, want, f"{shape} seed {seed} values x {v_mult}")
