#!/usr/bin/env python3
"""Benchmark of the Q4 KV-cache hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--skip-cpu-baseline] [--skip-other-configs]

Workload: the 10-agent ragged Gemma-3-12B-shaped configuration (48 layers, 16 query / 8 KV heads,
head_dim 256, context lengths drawn uniformly from [1024, 8192]), synthetic contents.  One step is one
pass of the whole path: a batch-10 decode-attention step over all 48 layers (one call), the quantization
of one fresh 4,096-token fp16 agent cache, and the dequantization of one restored cache.  Everything is
resident in HBM before the timed region.  Prints one JSON line.  The same line carries the step issued as one
call per layer (`per_layer_graph_ms`), the CPU oracle's timing of the same rows (`cpu_baseline`) and, under
`other_configs`, a compact measurement of the other four benchmark configurations (each with its own roofline
and oracle sample), so that one run times every row of the path.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth


# HBM bytes per launch of each workload's dominant kernel, read + written, from the rocprofv3 --pmc runs whose
# summaries are under profiles/ (FETCH_SIZE and WRITE_SIZE scaled by what a plain copy of known size reads).
# Counters cannot be read inside this process, so the figures are constants -- each tied to the sources of the
# kernel it was measured on: `sources` is kernel_sources_hash(files) at the time of the counter run, and
# traffic_for() hands a figure out only while those files are still the same (else null: measure again;
# `--print-sources-hash` prints the current hash of every set of files named here).
DECODE_FILES = ("decode_attention.hip", "stream_k.h", "q4_device.h", "q4kv_internal.h")
LATENT_FILES = ("mla_decode.hip", "stream_k.h", "q4_device.h", "q4kv_internal.h")
CODEC_FILES = ("codec.hip", "q4_device.h", "q4kv_internal.h")
CHUNK_FILES = ("chunk_attention.hip", "q4_device.h", "q4kv_internal.h")
MEASURED_TRAFFIC = {
    "gemma12b_10agents_48layers_ragged_1k_8k_decode": {
        "read": 4795018480, "written": 12899328, "file": "profiles/decode_attention_gemma10_ragged.md",
        "files": DECODE_FILES, "sources": "8f2be424bd49"},
    "llama8b_5agents_32layers_4k_decode": {
        "read": 776870455, "written": 8527872, "file": "profiles/decode_attention_llama8b_5x4k.md",
        "files": DECODE_FILES, "sources": "8f2be424bd49"},
    "dsv2lite_mla_per_head_5agents_27layers_8k_decode": {
        "read": 3190791189, "written": 3088896, "file": "profiles/decode_attention_mla_per_head_5x8k.md",
        "files": DECODE_FILES, "sources": "8f2be424bd49"},
    "dsv2lite_mla_latent_5agents_27layers_32k_decode": {
        "read": 1444160083, "written": 52912630, "file": "profiles/mla_decode_dsv2lite_5x32k.md",
        "files": LATENT_FILES, "sources": "d8ce4d131e95"},
    "quantize_4k_cache": {
        "read": 1610798278, "written": 452984832, "file": "profiles/decode_attention_gemma10_ragged.md",
        "files": CODEC_FILES, "sources": "3f4145ff341c"},
    "dequantize_4k_cache": {
        "read": 453023141, "written": 1610614784, "file": "profiles/decode_attention_gemma10_ragged.md",
        "files": CODEC_FILES, "sources": "3f4145ff341c"},
}


def kernel_sources_hash(files):
    """Short hash over the named kernel sources (what a counter run measured)."""
    import hashlib
    d = os.path.join(ROOT, "paper_2603_04428_amd", "csrc")
    h = hashlib.sha256()
    for f in sorted(files):
        h.update(f.encode())
        h.update(open(os.path.join(d, f), "rb").read())
    return h.hexdigest()[:12]


def traffic_for(name):
    """(bytes per launch, where it was measured) of a workload's dominant kernel, or (None, reason)."""
    m = MEASURED_TRAFFIC.get(name)
    if m is None:
        return None, "no counter run for this workload"
    if m["sources"] != kernel_sources_hash(m["files"]):
        return None, f"counter run {m['file']} was taken on other kernel sources ({m['sources']})"
    return m["read"] + m["written"], m["file"] + " (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy)"


PARAM_FORMAT = 0      # q4kv_param_format of the run (--param-format): 0 binary16, 1 bfloat16 scale / bias


def emit(res):
    """Print the result line; a bfloat16-parameter run says so in dtype, config and kernel name."""
    if PARAM_FORMAT == 1:
        res["dtype"] = res["dtype"].replace("f16 scale/bias", "bf16 scale/bias")
        res["config"]["param_format"] = "bf16"
        roof = res.get("roofline") or {}
        if "kernel" in roof:
            roof["kernel"] = roof["kernel"].replace(",false>", ",true>")
        if roof.get("traffic") is not None:
            roof["traffic"] = None          # the counter runs under profiles/ were made with binary16 parameters
    print(json.dumps(res))


def cpu_baseline(w, layers, agents=None):
    """The CPU oracle, as it stands, on a bounded sample of the same decode workload: all heads of a few layers
    (and, for the long-context configurations, a few agents).  Returns the JSON object; GB/s counts the same
    algorithmic Q4 bytes as the GPU figure."""
    import numpy as np
    import oracle
    agents = list(range(w.num_agents)) if agents is None else list(agents)
    spec = oracle.make_spec(len(layers), w.num_q_heads, w.num_kv_heads, w.k_dim, w.v_dim, w.v_aliases_k,
                            param_format=PARAM_FORMAT)
    lens = [w.seq_lens[a] for a in agents]
    need = [(n + 255) // 256 for n in lens]
    nb = max(1, sum(need))
    table = np.zeros((len(agents), max(1, max(need))), np.int32)
    pos = 0
    for i, k in enumerate(need):
        table[i, :k] = np.arange(pos, pos + k)
        pos += k
    kpool = oracle.Pool(spec, w.k_dim, nb)
    vpool = None if w.v_aliases_k else oracle.Pool(spec, w.v_dim, nb)
    q = np.zeros((len(layers), len(agents), 1, w.num_q_heads, w.k_dim), np.float16)
    for i, l in enumerate(layers):
        for j, a in enumerate(agents):
            n = lens[j]
            k_new = w.k_rows(l, a, 0, n).numpy()[None, None]
            v_new = None if w.v_aliases_k else w.v_rows(l, a, 0, n).numpy()[None, None]
            oracle.append(spec, kpool, vpool, k_new, v_new, table[j:j + 1], np.zeros(1, np.int32), i, i + 1)
            q[i, j] = w.q_rows(l, a).numpy()
    t0 = time.perf_counter()
    _, threads = oracle.attention(spec, kpool, vpool, q, table, lens, w.sm_scale, return_threads=True)
    dt = time.perf_counter() - t0
    nbytes = sum(lens) * len(layers) * w.q4_bytes_per_token_layer()
    step_bytes = sum(w.seq_lens) * w.num_layers * w.q4_bytes_per_token_layer()
    who = f"all {w.num_agents} agents" if len(agents) == w.num_agents else f"agents {agents} of {w.num_agents}"
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "agent_tokens_per_s": w.num_agents / (dt * step_bytes / nbytes),
            "sample": f"decode attention of layers {layers} of {w.num_layers}, {who}, all "
                      f"{w.num_q_heads} query heads ({nbytes / 1e6:.0f} MB of Q4 cache), {dt:.2f} s wall; "
                      "agent_tokens_per_s extrapolates to the whole step"}


def cpu_baseline_codec(x_host):
    """The oracle's quantizer and dequantizer timed on the whole 4,096-token fp16 cache (host copy of the generator's
    values): GB/s over the same bytes as the GPU rows (2 bytes in + 0.5625 out per element, and the reverse)."""
    import numpy as np
    import oracle
    x = x_host.reshape(-1, x_host.shape[-1])
    t0 = time.perf_counter()
    codes, scale, bias = oracle.quantize(x, PARAM_FORMAT)
    tq = time.perf_counter() - t0
    t0 = time.perf_counter()
    back = oracle.dequantize(codes, scale, bias, PARAM_FORMAT)
    td = time.perf_counter() - t0
    nbytes = x.size * 2 + codes.size * 4 + scale.size * 2 + bias.size * 2
    return {"quantize_GBps": nbytes / tq / 1e9, "quantize_s": tq, "dequantize_GBps": nbytes / td / 1e9,
            "dequantize_s": td, "elements": int(x.size), "cores": oracle.max_threads(),
            "sample": "oracle quantize and dequantize of the whole 4,096-token cache "
                      f"({x.size / 1e6:.0f} M elements, {nbytes / 1e9:.2f} GB moved each way)"}, back


def cpu_baseline_chunk(w, layer, agent, kvh):
    """The oracle on one (layer, agent, KV head) of the chunked-append configuration: append of the 512-token chunk
    and causal attention of its 512 rows x n_rep query heads over cache + chunk.  TFLOP/s counts the same
    algorithmic flops as the GPU figure (4 * heads * k_dim * visible keys per row)."""
    import numpy as np
    import oracle
    R, C, n = w.n_rep, w.q_len, w.seq_lens[agent]
    spec = oracle.make_spec(1, R, 1, w.k_dim, w.v_dim, False, param_format=PARAM_FORMAT)
    nb = (n + C + 255) // 256
    kpool, vpool = oracle.Pool(spec, w.k_dim, nb), oracle.Pool(spec, w.v_dim, nb)
    table = np.arange(nb, dtype=np.int32)[None]
    k_all = w.k_rows(layer, agent, 0, n + C, h0=kvh, h1=kvh + 1).numpy()[None, None]
    v_all = w.v_rows(layer, agent, 0, n + C, h0=kvh, h1=kvh + 1).numpy()[None, None]
    oracle.append(spec, kpool, vpool, k_all[:, :, :n], v_all[:, :, :n], table, np.zeros(1, np.int32))
    q = np.ascontiguousarray(w.q_rows(layer, agent).numpy()[:, kvh * R:(kvh + 1) * R])[None, None]
    t0 = time.perf_counter()
    oracle.append(spec, kpool, vpool, k_all[:, :, n:], v_all[:, :, n:], table, np.array([n], np.int32))
    _, threads = oracle.attention(spec, kpool, vpool, q, table, [n + C], w.sm_scale, return_threads=True)
    dt = time.perf_counter() - t0
    flops = 4.0 * R * w.k_dim * (C * n + C * (C + 1) / 2)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"quantize-append + causal chunk attention of layer {layer}, agent {agent} ({n} cached tokens), KV "
                      f"head {kvh}: {C} rows x {R} query heads, {flops / 1e9:.1f} GFLOP, {dt:.2f} s wall"}


MFMA_F16_PEAK_TFLOPS = 2500.0   # MI355X published dense fp16 matrix throughput


def bench_append(args, torch, b, synth, build_device_cache, steps=None, warmup=None):
    """Chunked append (the matrix-core path): per step, q4kv_append of a 512-token chunk for every agent and layer,
    then causal chunk attention of the 512 new queries over cache + chunk, all 48 layers.  Returns the result."""
    dev = "cuda"
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    w = synth.config(4)
    spec, kpool, vpool, table, table_d = build_device_cache(w, dev, poison=False, extra_blocks=0, tokens=w.seq_lens)
    C = w.q_len
    before = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    after = torch.tensor(w.final_lens(), dtype=torch.int32, device=dev)
    k_new = torch.stack([torch.stack([w.k_rows(l, a, n, n + C, dev) for a, n in enumerate(w.seq_lens)])
                         for l in range(w.num_layers)])
    v_new = torch.stack([torch.stack([w.v_rows(l, a, n, n + C, dev) for a, n in enumerate(w.seq_lens)])
                         for l in range(w.num_layers)])
    q = w.q_all(dev)
    out = torch.empty((w.num_layers, w.num_agents, C, w.num_q_heads, w.v_dim), dtype=torch.float16, device=dev)
    ws = torch.empty(16, dtype=torch.uint8, device=dev)
    max_len = max(w.final_lens())
    flops = sum(4.0 * w.num_q_heads * w.k_dim * (C * n + C * (C + 1) / 2) for n in w.seq_lens) * w.num_layers
    q4_bytes = sum(w.final_lens()) * w.num_layers * w.q4_bytes_per_token_layer()

    def step(ev=None):
        if ev:
            ev[0].record()
        b.q4kv_append(spec, kpool, vpool, k_new, v_new, table_d, before)
        if ev:
            ev[1].record()
        b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, after, max_len, w.sm_scale, 0, 0, 0, None, out, ws)
        if ev:
            ev[2].record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    app = [e[0].elapsed_time(e[1]) for e in events]
    att = [e[1].elapsed_time(e[2]) for e in events]
    app_in_step_ms, att_ms = sum(app) / len(app), sum(att) / len(att)
    # the append row by itself: back-to-back appends of the same chunk (they rewrite the same tokens), median
    app_alone = []
    for i in range(24):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        b.q4kv_append(spec, kpool, vpool, k_new, v_new, table_d, before)
        e1.record()
        torch.cuda.synchronize()
        if i >= 4:
            app_alone.append(e0.elapsed_time(e1))
    app_ms = percentile(app_alone, 50)
    tflops = flops / (att_ms * 1e-3) / 1e12
    app_bytes = k_new.numel() * 2 * 2 * (1 + 0.28125)
    res = {
        "metric": "Q4 KV chunked-append attention TFLOP/s (% of dense fp16 MFMA peak) + agent-tokens/s",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": wall * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 matrix operands (K codes exact, scales applied in f32; V dequantized to f16), f32 accumulate, f16 out", "data": "synthetic",
        "config": {"workload": w.name if args.layer_windows == "global" else w.name + " + 5:1 window-1024 layers",
                   "agents": w.num_agents, "layers": w.num_layers, "q_heads": w.num_q_heads,
                   "kv_heads": w.num_kv_heads, "head_dim": w.k_dim, "seq_lens_before": w.seq_lens, "chunk": C},
        "agent_tokens_per_s": w.num_agents * C / ((att_ms + app_in_step_ms) * 1e-3),
        "attention_ms": att_ms, "attention_flops": flops, "q4_bytes_if_read_once": q4_bytes,
        "append_ms": app_ms, "append_GBps": app_bytes / (app_ms * 1e-3) / 1e9,
        "append_ms_inside_the_step": app_in_step_ms,   # right after a 100 ms attention kernel, mean over the steps
        "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / MFMA_F16_PEAK_TFLOPS, "traffic": None,
                     "kernel": "chunk_attention_kernel<256,256,2,1,false>"},
    }
    if not args.skip_cpu_baseline:
        shortest = min(range(w.num_agents), key=lambda a: w.seq_lens[a])
        res["cpu_baseline"] = cpu_baseline_chunk(w, 0, shortest, 0)
    return res


def settle(torch, step, warmup, settle_ms):
    """The untimed part of a run: `warmup` steps, then more of them until `settle_ms` have passed.  For the first
    20-30 ms after the device changes to a kernel with another instruction mix its launches take up to a quarter
    longer (the shared-latent decode kernel: 420 us at first, 500 us after 3 ms, below 400 us from 25 ms on): the
    device finding its clock, not the kernel.  A step of a millisecond or more is past that after its warm-up
    steps anyway; a step of 20-400 us is not."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    while (time.perf_counter() - t0) * 1e3 < settle_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()


def percentile(xs, q):
    xs = sorted(xs)
    pos = (len(xs) - 1) * q / 100.0
    lo = int(pos)
    hi = min(lo + 1, len(xs) - 1)
    return xs[lo] + (xs[hi] - xs[lo]) * (pos - lo)


def per_layer_graph(torch, b, spec, kpool, vpool, q, table_d, seq, max_len, w, window, out_all_layers, planned=True,
                    settle_ms=60.0):
    """One attention call per layer, captured into a graph; returns the median replay time in ms.  Every replay is
    checked against the eager per-layer result (bit-identical: the same launches).  planned: the work plan is made
    once per step (q4kv_decode_plan) and every layer's call is a q4kv_batched_attention_planned; else 48 plain calls."""
    L = w.num_layers
    if isinstance(window, list):
        planned = False          # one window per layer: the layers do not share a plan
    split = b.q4kv_default_split_tokens(spec, w.num_agents, 1, max_len, 1)
    ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, w.num_agents, 1, max_len, split, 1), dtype=torch.uint8,
                     device=q.device)
    out = torch.empty_like(out_all_layers)
    win = window if isinstance(window, list) else [window] * L

    def all_layers():
        if planned:
            b.q4kv_decode_plan(spec, seq, max_len, ws, window=win[0], split_tokens=split, layers_in_call=1)
        for l in range(L):
            if planned:
                b.q4kv_batched_attention_planned(spec, kpool, vpool, q[l:l + 1], out[l:l + 1], table_d, max_len, w.sm_scale,
                                                 ws, window=win[0], split_tokens=split, layer_begin=l, layer_end=l + 1)
            else:
                b.q4kv_batched_attention(spec, kpool, vpool, q[l:l + 1], table_d, seq, max_len, w.sm_scale, win[l], split,
                                         l, l + 1, out[l:l + 1], ws)

    all_layers()
    torch.cuda.synchronize()
    eager = out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        all_layers()                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        all_layers()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < settle_ms:      # see settle()
        graph.replay()
        torch.cuda.synchronize()
    times = []
    for i in range(12):
        out.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        if not torch.equal(out, eager):
            raise RuntimeError("graph replay %d differs from the eager per-layer result" % i)
        if i >= 2:
            times.append(e0.elapsed_time(e1))
    return percentile(times, 50)


def calibration_copy(torch, dev):
    """One plain device-to-device copy kernel of known size: 1 GiB read + 1 GiB written."""
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def bench_latent(args, torch, b, synth, build_device_cache, **kw):
    """Decode over the shared-latent cache (DeepSeek-V2-Lite-shaped: 5 agents x 32,768 tokens x 27 layers, one
    576-wide Q4 row per token read by 16 heads), all layers in one call; reported as HBM GB/s."""
    return bench_decode_only(args, torch, b, build_device_cache, synth.config(3),
                             "mla_decode_kernel<9,8,false> (+ plan_kernel and combine_kernel in the same call)",
                             oracle_sample=([0], [0]), **kw)


def bench_llama(args, torch, b, synth, build_device_cache, **kw):
    """Decode over the Llama-3.1-8B-shaped cache of configuration 1 (5 agents x 4,096 tokens x 32 layers, 32 query /
    8 KV heads, 128 wide): a short call (0.15 ms), so plan and combine weigh in it."""
    return bench_decode_only(args, torch, b, build_device_cache, synth.config(1),
                             "decode_attention_kernel<128,128,4,false> (+ plan_kernel in the same call)",
                             oracle_sample=([0, 10, 21, 31], None), **kw)


def bench_tiny(args, torch, b, synth, build_device_cache, **kw):
    """Configuration 0 (1 agent x 1,024 tokens x 1 layer, Llama-shaped): 1.2 MB of cache that stays in the caches of
    the chip, so the figure of interest is the latency of one call (plan + attention + combine), `decode_us`."""
    return bench_decode_only(args, torch, b, build_device_cache, synth.config(0),
                             "decode_attention_kernel<128,128,4,false> (+ plan_kernel in the same call)",
                             oracle_sample=([0], None), **kw)


def bench_per_head(args, torch, b, synth, build_device_cache, **kw):
    """Decode over the decompressed per-head form of the same model's cache (keys 192, values 128, 16 KV heads)."""
    return bench_decode_only(args, torch, b, build_device_cache, synth.per_head_mla_config(),
                             "decode_attention_kernel<192,128,1,false> (+ plan_kernel in the same call)",
                             oracle_sample=([0, 26], None), **kw)


def bench_restore(args, torch, b, synth, build_device_cache):
    """Save / restore of one agent's cache (Sec. 3.1, 3.2 "Q4 at rest"): a Gemma-3-12B-shaped agent of 32,768 tokens
    (128 blocks x 48 layers, 3.6 GB of Q4) is gathered into a block image and scattered back, device to device and
    straight to / from pinned host memory, and restored from host memory while ten other agents decode."""
    dev = "cuda"
    w = synth.config(2)
    spec, kpool, vpool, table, table_d = build_device_cache(w, dev, poison=False, extra_blocks=128)
    nb = 128
    ids = torch.arange(kpool.num_blocks - nb, kpool.num_blocks, dtype=torch.int32, device=dev)  # the spare blocks
    for pool in (kpool, vpool):            # give the agent to be saved some contents
        pool.codes[:, ids.long()] = torch.randint(-2 ** 31, 2 ** 31 - 1, pool.codes[:, :nb].shape, dtype=torch.int32,
                                                  device=dev)
        pool.scale[:, ids.long()] = 0x3000
        pool.bias[:, ids.long()] = 0x3800
    nbytes = b.q4kv_block_image_bytes(spec, nb)
    dev_image = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    host_image = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return percentile(ts, 50)

    reps = max(3, min(args.steps, 10))
    t_exp_dev = timed(lambda: b.q4kv_export_blocks(spec, kpool, vpool, ids, dev_image), reps)
    t_imp_dev = timed(lambda: b.q4kv_import_blocks(spec, kpool, vpool, ids, dev_image), reps)
    t_exp_host = timed(lambda: b.q4kv_export_blocks(spec, kpool, vpool, ids, host_image), reps)
    t_imp_host = timed(lambda: b.q4kv_import_blocks(spec, kpool, vpool, ids, host_image), reps)
    assert torch.equal(host_image, dev_image.cpu())

    # restore from host memory on a second stream while the ten resident agents decode on the first
    q = w.q_all(dev)
    seq = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    max_len = max(w.seq_lens)
    split = b.q4kv_default_split_tokens(spec, w.num_agents, 1, max_len, w.num_layers)
    ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, w.num_agents, 1, max_len, split, w.num_layers),
                     dtype=torch.uint8, device=dev)
    out = torch.empty((w.num_layers, w.num_agents, 1, w.num_q_heads, w.v_dim), dtype=torch.float16, device=dev)

    def decode():
        b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, seq, max_len, w.sm_scale, 0, split, 0, None, out, ws)

    def restore_direct():          # the import kernel reads the pinned host image itself
        b.q4kv_import_blocks(spec, kpool, vpool, ids, host_image)

    def restore_staged():          # a copy engine brings the image over, the import kernel scatters it on the device
        dev_image.copy_(host_image, non_blocking=True)
        b.q4kv_import_blocks(spec, kpool, vpool, ids, dev_image)

    t_imp_staged = timed(restore_staged, reps)
    t_dec_alone = timed(decode, 20)
    side = torch.cuda.Stream()

    def overlapped(restore):
        """restore on the side stream while decode steps run on the main one -> (restore ms, ms per decode step, steps)"""
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            r0.record()
            restore()
            r1.record()
        steps = []
        while not r1.query():
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            decode()
            e1.record()
            e1.synchronize()
            steps.append(e0.elapsed_time(e1))
        torch.cuda.synchronize()
        inside = steps[:-1] if len(steps) > 1 else steps   # the last step may outlive the restore
        return r0.elapsed_time(r1), percentile(inside, 50), len(steps)

    ov_direct = overlapped(restore_direct)
    ov_staged = overlapped(restore_staged)

    copy_gbps = 2.0 * nbytes / (t_exp_dev * 1e-3) / 1e9
    res = {
        "metric": "Q4 KV cache restore: block image -> pool GB/s + restore time of a 32K-token agent",
        "value": nbytes / (t_imp_host * 1e-3) / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": reps, "warmup": 1,
        "ms_per_step": t_imp_host, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8 (bytes moved as they are)", "data": "synthetic",
        "config": {"workload": "gemma12b_one_agent_32k_tokens_48layers_restore", "blocks": nb, "layers": w.num_layers,
                   "image_bytes": nbytes},
        "restore_from_pinned_host_ms": t_imp_host, "restore_from_pinned_host_GBps": nbytes / (t_imp_host * 1e-3) / 1e9,
        "save_to_pinned_host_ms": t_exp_host, "save_to_pinned_host_GBps": nbytes / (t_exp_host * 1e-3) / 1e9,
        "export_device_ms": t_exp_dev, "import_device_ms": t_imp_dev,
        "device_copy_GBps_read_plus_write": copy_gbps,
        "restore_via_copy_engine_ms": t_imp_staged,
        "decode_ms_alone": t_dec_alone,
        "during_decode_direct": {"restore_ms": ov_direct[0], "decode_ms": ov_direct[1], "decode_steps": ov_direct[2]},
        "during_decode_copy_engine": {"restore_ms": ov_staged[0], "decode_ms": ov_staged[1], "decode_steps": ov_staged[2]},
        "roofline": {"bound": "hbm", "achieved": copy_gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": copy_gbps / HBM_PEAK_GBPS, "traffic": None,
                     "kernel": "image_copy_kernel<true> (pool -> device image; bytes read + written)"},
    }
    emit(res)


def bench_mixed_step(args, torch, b, synth, build_device_cache):
    """Iteration-level interleave of a prefill chunk with decode steps (the paper's concurrent scheduler, Sec. 3.4):
    one more agent appends a 512-token chunk to a 16,384-token cache and attends to it (all 48 layers, matrix cores)
    on a second stream while the ten agents of the headline workload keep decoding (HBM) on the first."""
    dev = "cuda"
    wd = synth.config(2)
    spec, kpool, vpool, table, table_d = build_device_cache(wd, dev, poison=False, extra_blocks=0)
    q = wd.q_all(dev)
    seq = torch.tensor(wd.seq_lens, dtype=torch.int32, device=dev)
    max_len = max(wd.seq_lens)
    split = b.q4kv_default_split_tokens(spec, wd.num_agents, 1, max_len, wd.num_layers)
    ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, wd.num_agents, 1, max_len, split, wd.num_layers),
                     dtype=torch.uint8, device=dev)
    out = torch.empty((wd.num_layers, wd.num_agents, 1, wd.num_q_heads, wd.v_dim), dtype=torch.float16, device=dev)

    def decode():
        b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, seq, max_len, wd.sm_scale, 0, split, 0, None, out, ws)

    wa = synth.small(6, wd.num_layers, wd.num_q_heads, wd.num_kv_heads, wd.k_dim, wd.v_dim, False, (16384,), q_len=512,
                     name="gemma12b_1agent_16k_append512")
    aspec, akp, avp, atable, atable_d = build_device_cache(wa, dev, poison=False, extra_blocks=0, tokens=wa.seq_lens)
    C = wa.q_len
    before = torch.tensor(wa.seq_lens, dtype=torch.int32, device=dev)
    after = torch.tensor(wa.final_lens(), dtype=torch.int32, device=dev)
    k_new = torch.stack([torch.stack([wa.k_rows(l, 0, 16384, 16384 + C, dev)]) for l in range(wa.num_layers)])
    v_new = torch.stack([torch.stack([wa.v_rows(l, 0, 16384, 16384 + C, dev)]) for l in range(wa.num_layers)])
    aq = wa.q_all(dev)
    aout = torch.empty((wa.num_layers, 1, C, wa.num_q_heads, wa.v_dim), dtype=torch.float16, device=dev)
    aws = torch.empty(16, dtype=torch.uint8, device=dev)
    flops = 4.0 * wa.num_q_heads * wa.k_dim * (C * 16384 + C * (C + 1) / 2) * wa.num_layers

    def chunk():
        b.q4kv_append(aspec, akp, avp, k_new, v_new, atable_d, before)
        b.q4kv_batched_attention(aspec, akp, avp, aq, atable_d, after, 16384 + C, wa.sm_scale, 0, 0, 0, None, aout, aws)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return percentile(ts, 50)

    t_dec = timed(decode, 30)
    t_chunk = timed(chunk, 10)
    side = torch.cuda.Stream()
    chunk_ms, dec_ms, dec_steps = [], [], []
    for _ in range(5):
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(side):
            r0.record()
            chunk()
            r1.record()
        steps = []
        while not r1.query():
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            decode()
            e1.record()
            e1.synchronize()
            steps.append(e0.elapsed_time(e1))
        torch.cuda.synchronize()
        chunk_ms.append(r0.elapsed_time(r1))
        dec_ms.append(sum(steps) / len(steps))
        dec_steps.append(len(steps))
    t_chunk_mixed, t_dec_mixed = percentile(chunk_ms, 50), percentile(dec_ms, 50)
    # work done per second when interleaved, relative to running the two one after the other
    n = percentile(dec_steps, 50)
    serial_ms = t_chunk + n * t_dec
    res = {
        "metric": "mixed step: decode steps of 10 agents beside one agent's 512-token append (speed-up over serial)",
        "value": serial_ms / t_chunk_mixed, "unit": "x", "n_gpus": 1, "steps": 5, "warmup": 1,
        "ms_per_step": t_chunk_mixed, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "q4 codes + f16 scale/bias, f32 accumulate, f16 out", "data": "synthetic",
        "config": {"workload": wd.name + " + " + wa.name, "layers": wd.num_layers},
        "decode_ms_alone": t_dec, "chunk_ms_alone": t_chunk, "chunk_TFLOPs_alone": flops / (t_chunk * 1e-3) / 1e12,
        "decode_ms_beside_chunk": t_dec_mixed, "chunk_ms_beside_decode": t_chunk_mixed,
        "decode_steps_per_chunk": n, "serial_ms_for_the_same_work": serial_ms,
        "roofline": None,
    }
    emit(res)


def bench_decode_only(args, torch, b, build_device_cache, w, kernel_name, oracle_sample=None, steps=None, warmup=None):
    """One decode configuration, all layers in one call.  oracle_sample: (layers, agents or None for all) the CPU
    oracle is timed on.  Returns the result."""
    dev = "cuda"
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    spec, kpool, vpool, table, table_d = build_device_cache(w, dev, poison=False, extra_blocks=0)
    q = w.q_all(dev)
    seq = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    max_len = max(w.seq_lens)
    split = args.split_tokens or b.q4kv_default_split_tokens(spec, w.num_agents, 1, max_len, w.num_layers)
    ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, w.num_agents, 1, max_len, split, w.num_layers),
                     dtype=torch.uint8, device=dev)
    out = torch.empty((w.num_layers, w.num_agents, 1, w.num_q_heads, w.v_dim), dtype=torch.float16, device=dev)
    decode_bytes = sum(w.seq_lens) * w.num_layers * w.q4_bytes_per_token_layer()
    flops = 2.0 * sum(w.seq_lens) * w.num_layers * w.num_q_heads * (w.k_dim + w.v_dim)

    def step():
        b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, seq, max_len, w.sm_scale, 0, split, 0, None, out, ws)

    if args.calibrate_copy:
        calibration_copy(torch, dev)
    settle(torch, step, warmup, args.settle_ms)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        events[i][0].record()
        step()
        events[i][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dec = [e[0].elapsed_time(e[1]) for e in events]
    dec_ms = percentile(dec, 50)
    gbps = decode_bytes / (dec_ms * 1e-3) / 1e9
    res = {
        "metric": "Q4 KV decode-attention achieved HBM GB/s (% of peak) + agent-tokens/s",
        "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": wall * 1e3 / steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "q4 codes + f16 scale/bias, f16 matrix operands, f32 accumulate, f16 out", "data": "synthetic",
        "config": {"workload": w.name if args.layer_windows == "global" else w.name + " + 5:1 window-1024 layers",
                   "agents": w.num_agents, "layers": w.num_layers, "q_heads": w.num_q_heads,
                   "kv_heads": w.num_kv_heads, "k_dim": w.k_dim, "v_dim": w.v_dim, "seq_lens": w.seq_lens,
                   "split_tokens": split, "launch": "all layers in one q4kv_batched_attention call"},
        "pct_of_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "agent_tokens_per_s": w.num_agents / (dec_ms * 1e-3),
        "decode_ms": dec_ms, "decode_us": dec_ms * 1e3, "decode_ms_p10": percentile(dec, 10), "decode_ms_p90": percentile(dec, 90),
        "decode_ms_min": min(dec), "decode_bytes": decode_bytes,
        "matrix_TFLOPs": flops / (dec_ms * 1e-3) / 1e12,
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS,
                     "traffic": traffic_for(w.name)[0] if not args.split_tokens else None,
                     "traffic_source": traffic_for(w.name)[1],
                     "kernel": kernel_name},
    }
    if oracle_sample is not None and not args.skip_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, oracle_sample[0], oracle_sample[1])
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=60.0,
                    help="the untimed warm-up goes on until this much time has passed (0: the --warmup steps only)")
    ap.add_argument("--skip-cpu-baseline", action="store_true", help="for profiler runs: leave the oracle leg out")
    ap.add_argument("--split-tokens", type=int, default=0, help="tokens per split-K work item (0: library default)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (a known-size reference for scaling "
                         "the profiler's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--workload", choices=["decode", "append", "latent", "per-head", "llama", "tiny", "restore", "mixed-step"], default="decode",
                    help="decode (default): the headline configuration; append: the chunked-append configuration "
                         "(10 agents, 4,096..32,768 cached tokens, 512-token chunk), reported as TFLOP/s; latent: "
                         "decode over the shared-latent (MLA-shaped) cache, 5 agents x 32,768 tokens x 27 layers; per-head: "
                         "decode over the decompressed form of that cache (keys 192, values 128, 16 KV heads); llama: decode over the "
                         "Llama-shaped cache of configuration 1; tiny: the latency of one call on configuration 0; restore: save "
                         "and restore of one 32,768-token agent through a block image, also while other agents decode; mixed-step: "
                         "one agent's 512-token append on a second stream beside the decode steps of ten others")
    ap.add_argument("--no-per-layer-graph", action="store_true",
                    help="decode workload: leave out the timing of the same step issued as one call per layer, recorded "
                         "into a graph and replayed ('per_layer_graph_ms'); for profiler runs, whose per-kernel "
                         "averages it would mix with the single-launch figures")
    ap.add_argument("--skip-other-configs", action="store_true",
                    help="decode workload: leave out the compact measurements of the other four benchmark "
                         "configurations ('other_configs'); for profiler runs")
    ap.add_argument("--print-sources-hash", action="store_true",
                    help="print the hash of the kernel sources that MEASURED_TRAFFIC entries are tied to, and exit")
    ap.add_argument("--param-format", choices=["f16", "bf16"], default="f16",
                    help="type of the stored scale and bias (decode, append, latent, per-head workloads); f16 is what "
                         "every benchmark configuration specifies")
    ap.add_argument("--layer-windows", choices=["global", "mixed"], default="global",
                    help="decode workload only.  global (default, the headline configuration): every layer attends "
                         "to the whole cache; mixed: five layers with a 1,024-token sliding window, then one global "
                         "layer, repeated (8 global + 40 windowed of 48, Sec. 3.6) through the per-layer window entry")
    args = ap.parse_args()
    if args.print_sources_hash:
        for n in ("DECODE_FILES", "LATENT_FILES", "CODEC_FILES", "CHUNK_FILES"):
            print(n, kernel_sources_hash(globals()[n]))
        return
    if args.gpus != 1:
        sys.exit("bench.py: this path runs on ONE GPU (agents would shard across GPUs with no exchange step); "
                 "run with --gpus 1")

    import torch
    from paper_2603_04428_amd import binding as b
    from paper_2603_04428_amd import synth
    from paper_2603_04428_amd.workload import build_device_cache

    global PARAM_FORMAT
    if args.param_format == "bf16":
        import functools
        PARAM_FORMAT = b.PARAMS_BF16
        build_device_cache = functools.partial(build_device_cache, param_format=b.PARAMS_BF16)
    dev = "cuda"
    if args.workload == "append":
        return emit(bench_append(args, torch, b, synth, build_device_cache))
    if args.workload == "latent":
        return emit(bench_latent(args, torch, b, synth, build_device_cache))
    if args.workload == "per-head":
        return emit(bench_per_head(args, torch, b, synth, build_device_cache))
    if args.workload == "llama":
        return emit(bench_llama(args, torch, b, synth, build_device_cache))
    if args.workload == "tiny":
        return emit(bench_tiny(args, torch, b, synth, build_device_cache))
    if args.workload == "restore":
        return bench_restore(args, torch, b, synth, build_device_cache)
    if args.workload == "mixed-step":
        return bench_mixed_step(args, torch, b, synth, build_device_cache)
    w = synth.config(2)
    spec, kpool, vpool, table, table_d = build_device_cache(w, dev, poison=False, extra_blocks=0)
    q = w.q_all(dev)
    seq = torch.tensor(w.seq_lens, dtype=torch.int32, device=dev)
    max_len = max(w.seq_lens)
    split = args.split_tokens or b.q4kv_default_split_tokens(spec, w.num_agents, 1, max_len, w.num_layers)
    ws = torch.empty(b.q4kv_attention_workspace_bytes(spec, w.num_agents, 1, max_len, split, w.num_layers),
                     dtype=torch.uint8, device=dev)
    out = torch.empty((w.num_layers, w.num_agents, 1, w.num_q_heads, w.v_dim), dtype=torch.float16, device=dev)

    # one fresh 4,096-token fp16 agent cache [layers][K,V][tokens][kv_heads][dim] and its Q4 form
    fresh = torch.stack([torch.stack([w.k_rows(l, 0, 100000, 104096, dev), w.v_rows(l, 0, 100000, 104096, dev)])
                         for l in range(w.num_layers)])
    codes, scale, bias = b.q4kv_quantize(fresh, param_format=PARAM_FORMAT)
    restored = torch.empty_like(fresh)
    quant_bytes = fresh.numel() * 2 + codes.numel() * 4 + scale.numel() * 4
    if args.layer_windows == "mixed":
        window = [0 if l % 6 == 5 else 1024 for l in range(w.num_layers)]
    else:
        window = 0
    visible = sum(sum(min(n, wl) if wl > 0 else n for n in w.seq_lens)
                  for wl in (window if isinstance(window, list) else [0] * w.num_layers))
    decode_bytes = visible * w.q4_bytes_per_token_layer()

    # Row order inside a step: dequantize, quantize, attention.  A kernel that writes much leaves dirty lines in the
    # caches (up to the 256 MB of the memory-side cache), and their write-back is charged to whatever runs next:
    # directly after the dequantize row (1.6 GB written) the attention call measures 6 % slower than after itself,
    # after the quantize row (0.45 GB written) 2 % slower.
    def step(ev=None):
        if ev:
            ev[0].record()
        b.q4kv_dequantize(codes, scale, bias, restored, param_format=PARAM_FORMAT)
        if ev:
            ev[1].record()
        b.q4kv_quantize(fresh, codes, scale, bias, param_format=PARAM_FORMAT)
        if ev:
            ev[2].record()
        b.q4kv_batched_attention(spec, kpool, vpool, q, table_d, seq, max_len, w.sm_scale, window, split, 0, None,
                                 out, ws)
        if ev:
            ev[3].record()

    if args.calibrate_copy:
        calibration_copy(torch, dev)
    settle(torch, step, args.warmup, args.settle_ms)
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    deq = [e[0].elapsed_time(e[1]) for e in events]
    qua = [e[1].elapsed_time(e[2]) for e in events]
    dec = [e[2].elapsed_time(e[3]) for e in events]
    dec_ms = percentile(dec, 50)                  # the figures are medians over the timed steps
    qua_ms = percentile(qua, 50)
    deq_ms = percentile(deq, 50)
    gbps = decode_bytes / (dec_ms * 1e-3) / 1e9

    # the memory system's own ceiling: a kernel that only reads, over the K code pool the decode step reads
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_buf = kpool.codes
    probe_bytes = probe_buf.numel() * probe_buf.element_size() // 16384 * 16384
    probe = []
    for i in range(12):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        b.q4kv_read_probe(probe_buf, sink)
        e1.record()
        torch.cuda.synchronize()
        if i >= 2:
            probe.append(e0.elapsed_time(e1))
    probe_gbps = probe_bytes / (percentile(probe, 50) * 1e-3) / 1e9

    # its ceilings for writes alone and for reads mixed with writes (plain library fill and copy of 1 GiB): the
    # codec rows stream a read + write mix and are to be read against the copy figure
    def library_op_ms(op):
        ms = []
        for i in range(8):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            op()
            e1.record()
            torch.cuda.synchronize()
            if i >= 2:
                ms.append(e0.elapsed_time(e1))
        return percentile(ms, 50)
    fill_src = torch.empty(1 << 28, dtype=torch.int32, device=dev)
    fill_dst = torch.empty_like(fill_src)
    write_probe_gbps = (1 << 30) / (library_op_ms(lambda: fill_src.fill_(1)) * 1e-3) / 1e9
    copy_probe_gbps = 2 * (1 << 30) / (library_op_ms(lambda: fill_dst.copy_(fill_src)) * 1e-3) / 1e9
    del fill_src, fill_dst

    # the same step as one call per layer, recorded once into a graph and replayed (launch-bound form of the loop)
    per_layer_ms = per_layer_plain_ms = None
    if not args.no_per_layer_graph:
        per_layer_ms = per_layer_graph(torch, b, spec, kpool, vpool, q, table_d, seq, max_len, w, window, out,
                                       settle_ms=args.settle_ms)
        per_layer_plain_ms = per_layer_graph(torch, b, spec, kpool, vpool, q, table_d, seq, max_len, w, window, out,
                                             planned=False, settle_ms=args.settle_ms)

    res = {
        "metric": "Q4 KV decode-attention achieved HBM GB/s (% of peak) + agent-tokens/s",
        "value": gbps, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "q4 codes + f16 scale/bias, f32 accumulate, f16 out", "data": "synthetic",
        "config": {"workload": w.name if args.layer_windows == "global" else w.name + " + 5:1 window-1024 layers",
                   "agents": w.num_agents, "layers": w.num_layers, "q_heads": w.num_q_heads,
                   "kv_heads": w.num_kv_heads, "head_dim": w.k_dim, "seq_lens": w.seq_lens,
                   "split_tokens": split, "launch": "all layers in one q4kv_batched_attention call"},
        "pct_of_hbm_peak": 100.0 * gbps / HBM_PEAK_GBPS,
        "agent_tokens_per_s": w.num_agents / (dec_ms * 1e-3),
        "decode_ms": dec_ms, "decode_us": dec_ms * 1e3, "decode_ms_p10": percentile(dec, 10), "decode_ms_p90": percentile(dec, 90),
        "decode_ms_min": min(dec), "decode_ms_mean": sum(dec) / len(dec), "decode_bytes": decode_bytes,
        "read_probe_GBps": probe_gbps, "pct_of_read_probe": 100.0 * gbps / probe_gbps,
        "write_probe_GBps": write_probe_gbps, "copy_probe_GBps": copy_probe_gbps,
        "per_layer_graph_ms": per_layer_ms,
        "per_layer_graph_GBps": None if per_layer_ms is None else decode_bytes / (per_layer_ms * 1e-3) / 1e9,
        "per_layer_graph_frac_of_hbm_peak": None if per_layer_ms is None
        else decode_bytes / (per_layer_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "per_layer_graph_plain_calls_ms": per_layer_plain_ms,
        "per_layer_graph_note": "the same decode step as 48 calls of one layer each (what a forward pass issues), "
                                "recorded into a graph and replayed; every replay bit-identical to the eager calls.  "
                                "per_layer_graph_ms: q4kv_decode_plan once + 48 q4kv_batched_attention_planned (one "
                                "kernel each); per_layer_graph_plain_calls_ms: 48 q4kv_batched_attention (plan kernel + "
                                "attention kernel each)",
        "seed": w.seed,
        "quantize_ms": qua_ms, "quantize_GBps": quant_bytes / (qua_ms * 1e-3) / 1e9,
        "dequantize_ms": deq_ms, "dequantize_GBps": quant_bytes / (deq_ms * 1e-3) / 1e9,
        # traffic: HBM bytes of one launch of the dominant kernel, from the committed rocprofv3 counter runs (they
        # cannot be taken inside this process); only for the exact workload those runs measured
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS,
                     "traffic": traffic_for(w.name)[0] if args.layer_windows == "global" and not args.split_tokens
                     else None,
                     "traffic_source": traffic_for(w.name)[1],
                     "kernel": "decode_attention_kernel<256,256,2,false> (+ plan_kernel in the same call)"},
        "roofline_quantize": {"bound": "hbm", "achieved": quant_bytes / (qua_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                              "unit": "GB/s", "frac": quant_bytes / (qua_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "traffic": traffic_for("quantize_4k_cache")[0],
                              "traffic_source": traffic_for("quantize_4k_cache")[1], "kernel": "quantize_kernel<false>"},
        "roofline_dequantize": {"bound": "hbm", "achieved": quant_bytes / (deq_ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                                "unit": "GB/s", "frac": quant_bytes / (deq_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                                "traffic": traffic_for("dequantize_4k_cache")[0],
                                "traffic_source": traffic_for("dequantize_4k_cache")[1],
                                "kernel": "dequantize_kernel<false>"},
    }
    if not args.skip_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, [0, w.num_layers // 3, 2 * w.num_layers // 3, w.num_layers - 1])
        # the oracle's codec on the same 4,096-token cache, and the round trip checked against the GPU rows
        codec, back = cpu_baseline_codec(fresh.cpu().numpy())
        codec["gpu_dequantize_equals_oracle"] = bool((restored.cpu().numpy().view("uint16") == back.view("uint16").reshape(restored.shape)).all())
        res["cpu_baseline"]["codec"] = codec
        del back
    if not args.skip_other_configs:
        del kpool, vpool, fresh, restored, codes, scale, bias, ws, out, q
        torch.cuda.empty_cache()
        res["other_configs"] = other_configs(args, torch, b, synth, build_device_cache)
    emit(res)


def compact(res):
    """What the headline line keeps of another configuration's result."""
    keep = ("metric", "value", "unit", "dtype", "agent_tokens_per_s", "decode_ms", "decode_us", "attention_ms", "append_ms",
            "append_GBps", "pct_of_hbm_peak", "matrix_TFLOPs", "attention_flops", "decode_bytes", "steps", "warmup",
            "roofline", "cpu_baseline")
    out = {"workload": res["config"]["workload"]}
    out.update({k: res[k] for k in keep if k in res})
    return out


def other_configs(args, torch, b, synth, build_device_cache):
    """The other four benchmark configurations, one after the other with their caches freed in between: the
    1-agent latency case, the Llama-shaped and the shared-latent decode steps, and the chunked append."""
    runs = [("tiny", bench_tiny, dict(steps=max(args.steps, 100), warmup=max(args.warmup, 10))),
            ("llama", bench_llama, dict(steps=max(args.steps, 100), warmup=max(args.warmup, 10))),
            ("latent", bench_latent, dict(steps=max(args.steps, 100), warmup=max(args.warmup, 10))),
            ("append", bench_append, dict(steps=max(min(args.steps, 5), 3), warmup=2))]
    out = []
    for name, fn, kw in runs:
        try:
            out.append(compact(fn(args, torch, b, synth, build_device_cache, **kw)))
        except Exception as e:           # a failure here must not cost the headline line
            out.append({"workload": name, "error": f"{type(e).__name__}: {e}"})
        torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
