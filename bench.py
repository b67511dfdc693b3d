#!/usr/bin/env python3
"""Benchmark of the MixAttention decode / prefill attention path on one MI355X.

Default workload ("decode32k"): the 24-layer MixAttention stack (layers 0 and 12 full, 22 sliding-window layers
W = 1024 in six sharing groups), bf16, batch 32, 32768 tokens of context per sequence.  One step = the whole hot
path for one generated token per sequence: 8 KV appends (writer layers, fused into their decode launch unless
--two-call-append) + 24 decode attentions, with every input already resident in HBM.  Prints ONE JSON line:
metric / value / unit / ms_per_step / config, `roofline` (the full-attention decode launch against the 8 TB/s HBM
peak, timed with events inside the timed region) and `cpu_baseline` (the CPU oracle on a bounded sample).

Other workloads (--workload): decode4k (batch 8, context 4096), prefill32k (batch 1, 32768-token prompt through
the 24 layers), ragged64 (batch 64, context lengths uniform in [1024, 65536], MixAttention stack next to the
all-full 24-layer stack), variants (decode step by layer layout), gen31k (31000-token prompts prefilled, then
1000 tokens generated, batch 32: the shape of the paper's inference-speed measurement, attention stack only).

Everything on the timed path runs in libmixattn's kernels; torch provides device memory, the stream and events.
The CPU oracle is used only for the `cpu_baseline` leg (and never feeds the GPU path).
"""

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="decode32k", choices=["decode32k", "decode4k", "prefill32k", "ragged64", "variants", "gen31k", "serve"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-keys", type=int, default=0)
    ap.add_argument("--balanced", type=int, default=-1)
    ap.add_argument("--prefill-waves", type=int, default=0)
    ap.add_argument("--prefill-heads", type=int, default=0)
    ap.add_argument("--chunks", type=int, default=1, help="prefill32k: feed the prompt in this many equal chunks")
    ap.add_argument("--skip-standard", action="store_true", help="ragged64: time the MixAttention stack only")
    ap.add_argument("--with-standard", action="store_true", help="gen31k: also run the standard 24-layer stack")
    ap.add_argument("--gen-batch", type=int, default=32)
    ap.add_argument("--gen-prompt", type=int, default=31000)
    ap.add_argument("--gen-new", type=int, default=1000)
    ap.add_argument("--serve-requests", type=int, default=96, help="serve: requests to run through the batch slots")
    ap.add_argument("--serve-slots", type=int, default=32, help="serve: sequences decoded together")
    ap.add_argument("--serve-prompt", type=int, nargs=2, default=[8000, 31000], help="serve: prompt length range")
    ap.add_argument("--serve-new", type=int, nargs=2, default=[100, 1000], help="serve: generated length range")
    ap.add_argument("--page-tokens", type=int, default=0,
                    help="hold full-attention caches as pools of pages of this many tokens (0: contiguous)")
    ap.add_argument("--group-decode", action="store_true",
                    help="decode workloads: serve every sliding-window sharing group with one launch (all its queries "
                         "at once; an upper bound a model cannot reach, reported beside the per-layer figure)")
    ap.add_argument("--two-call-append", action="store_true",
                    help="writer layers call append_kv and decode separately instead of append_decode")
    ap.add_argument("--out-dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--graph", type=int, default=-1,
                    help="decode workloads: 1 = the timed steps are replays of one decode step captured into a HIP graph "
                         "(the eager figure is reported beside it), 0 = eager launches only, -1 = workload default")
    ap.add_argument("--headline-only", action="store_true",
                    help="decode32k: skip the prefill32k and ragged64 legs that the default run adds to its line")
    ap.add_argument("--only", default="", help="profiling aid: 'full' or 'sliding' runs only that layer kind per step")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="profiling aid: also run N plain device copies of 1 GiB (known traffic for counter scaling)")
    return ap.parse_args()


def _source_digest(names):
    """sha256 (first 16 hex digits) over the named files of csrc/, in order."""
    import hashlib
    h = hashlib.sha256()
    for name in names:
        with open(os.path.join(ROOT, "paper_2409_15012_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def _traffic_from_profiles(kernel_tag, source=("kernels_decode.hip", "mixattn_host.hip")):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE) in runs of their own, recorded as
    text under profiles/ together with a digest of the sources they were taken with (the decode kernels and the host
    side that plans their launches).  Returns (bytes, note): bytes is None when there is no record or a source has
    changed since (a stale figure is not reported)."""
    path = os.path.join(ROOT, "profiles", "traffic_%s.txt" % kernel_tag)
    value, digest = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                value = float(line.split(":")[1])
            if line.startswith("kernel_source_sha256_16:"):
                digest = line.split(":")[1].split()[0]
    except OSError:
        return None, "no recorded counter run"
    if digest != _source_digest(source):
        return None, "recorded counter run (profiles/traffic_%s.txt) is for older sources (%s)" % (kernel_tag, ", ".join(source))
    return value, "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs recorded in profiles/traffic_%s.txt" % kernel_tag


def _paging(page_tokens, capacity):
    """Layout keyword arguments for a pool that holds exactly every sequence at its capacity."""
    if not page_tokens:
        return {}
    return {"page_tokens": page_tokens,
            "pool_tokens": sum((c + page_tokens - 1) // page_tokens for c in capacity) * page_tokens}


def build_decode_stack(mx, wl, torch, layers, batch, Hq, Hkv, d, seq_lens, extra, out_dtype, dev, seed, page_tokens=0):
    """Creates a layout, fills every writer cache with seq_lens[b] seeded tokens, returns (layout, per-layer inputs)."""
    capacity = [n + extra for n in seq_lens]
    lay = mx.Layout(layers, batch, Hq, Hkv, d, capacity=capacity, kv_dtype="bf16", out_dtype=out_dtype,
                    **_paging(page_tokens, capacity))
    total = int(sum(seq_lens))
    qs, ks, vs = [], [], []
    for li in range(len(layers)):
        qs.append(wl.randn(wl.layer_seed(seed, li, "q"), (batch, Hq, d), torch.bfloat16, dev))
        ci, is_writer = lay.cache_of(li)
        if is_writer:
            kind, W, _ = layers[li]
            if kind == wl.SLIDING:
                # a ring keeps the last W tokens only, so W tokens per sequence fill it completely (decode cost
                # depends on min(n, W), not on n); later appends wrap around as usual
                lens = [min(n, W) for n in seq_lens]
                k = wl.randn(wl.layer_seed(seed, li, "k", 1), (sum(lens), Hkv, d), torch.bfloat16, dev)
                v = wl.randn(wl.layer_seed(seed, li, "v", 1), (sum(lens), Hkv, d), torch.bfloat16, dev)
                lay.load_kv(li, k, v, lens)
            else:
                k = wl.randn(wl.layer_seed(seed, li, "k", 1), (total, Hkv, d), torch.bfloat16, dev)
                v = wl.randn(wl.layer_seed(seed, li, "v", 1), (total, Hkv, d), torch.bfloat16, dev)
                lay.load_kv(li, k, v, seq_lens)
            del k, v
            torch.cuda.empty_cache()
            ks.append(wl.randn(wl.layer_seed(seed, li, "k"), (batch, Hkv, d), torch.bfloat16, dev))
            vs.append(wl.randn(wl.layer_seed(seed, li, "v"), (batch, Hkv, d), torch.bfloat16, dev))
        else:
            ks.append(None)
            vs.append(None)
    torch.cuda.synchronize()
    return lay, qs, ks, vs


def run_decode(args, mx, wl, torch, w, layers=None, label=None):
    dev = "cuda:0"
    layers = layers or w.layers
    B, Hq, Hkv, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    use_graph = args.graph == 1 and not args.group_decode
    total_steps = (args.warmup + args.steps) * (2 if use_graph else 1) + (2 if use_graph else 0)
    # the first timed step decodes at exactly the workload's context length
    # (of the graph replays when those are what is timed: the eager steps then run just below it)
    graph_shift = (args.warmup + args.steps + 1) if use_graph else 0
    seq_lens = [max(1, n - 1 - args.warmup - graph_shift) for n in w.seq_lens]
    lay, qs, ks, vs = build_decode_stack(mx, wl, torch, layers, B, Hq, Hkv, d, seq_lens, total_steps + 1,
                                         args.out_dtype, dev, w.seed, args.page_tokens)
    if args.chunk_keys:
        lay.set_param(mx.PARAM_CHUNK_KEYS, args.chunk_keys)
    if args.balanced >= 0:
        lay.set_param(mx.PARAM_BALANCED, args.balanced)
    out = torch.empty((B, Hq, d), dtype=lay.out_torch, device=dev)
    full_layers = [li for li, t in enumerate(layers) if t[0] == wl.FULL]
    kinds = {"": None, "full": wl.FULL, "sliding": wl.SLIDING}[args.only]

    # sliding-window sharing groups for --group-decode: writer layer -> all layers on its ring, queries stacked
    groups = {}
    if args.group_decode:
        for li, (kind, W, cid) in enumerate(layers):
            if kind == wl.SLIDING and layers[lay.writer_of(li)][0] == wl.SLIDING:
                groups.setdefault(lay.writer_of(li), []).append(li)
        group_q = {wr: torch.stack([qs[li] for li in ls]).contiguous() for wr, ls in groups.items()}
        group_out = {wr: torch.empty((len(ls), B, Hq, d), dtype=lay.out_torch, device=dev) for wr, ls in groups.items()}
    grouped = {li for ls in groups.values() for li in ls}

    def step(events=None):
        for li in range(len(layers)):
            if li in grouped:
                if li in groups and kinds in (None, wl.SLIDING):
                    lay.decode_group(groups[li], group_q[li], ks[li], vs[li], group_out[li])
                continue
            skip = kinds is not None and layers[li][0] != kinds
            fused = ks[li] is not None and not args.two_call_append and not skip
            if ks[li] is not None and not fused:
                lay.append_kv(li, ks[li], vs[li])
            if skip:
                continue
            timed = events is not None and li in full_layers
            if timed:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record()
            if fused:
                lay.append_decode(li, ks[li], vs[li], qs[li], out)
            else:
                lay.decode(li, qs[li], out)
            if timed:
                e1.record()
                events.append((li, e0, e1))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = eager_ms = (t1 - t0) * 1e3 / args.steps
    graph_ms = None
    if use_graph:
        # the same step captured once and replayed: every replay appends one token per sequence and attends one
        # position further (lengths live on the device; the host is told with account_replays)
        lay.reserve_steps(args.warmup + args.steps + 1)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        for _ in range(args.warmup):
            graph.replay()
            lay.account_replays(1)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
            lay.account_replays(1)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        ms_per_step = graph_ms
        del graph

    # logical KV bytes of one step, taken at the mid-point length (n grows by one per step)
    ctx_lens = [n + args.warmup + 1 + graph_shift + args.steps // 2 for n in seq_lens]
    per_tok = 2 * Hkv * d * 2
    kv_step = 0
    kv_full_launch = 0
    for li, (kind, W, _) in enumerate(layers):
        tok = sum(n if kind == wl.FULL else min(n, W) for n in ctx_lens)
        if li in grouped and li not in groups:
            continue   # a group launch reads the ring once for all its layers
        if kinds is None or kind == kinds:
            kv_step += tok * per_tok
        if kind == wl.FULL:
            kv_full_launch = tok * per_tok
    qo_bytes = B * Hq * d * (2 + (2 if args.out_dtype == "bf16" else 4))
    full_ms = [e0.elapsed_time(e1) for (_, e0, e1) in events]
    res = {
        "eager_ms_per_step": eager_ms, "graph_ms_per_step": graph_ms,
        "ms_per_step": ms_per_step,
        "tokens_per_s": B / (ms_per_step * 1e-3),
        "kv_bytes_per_step": kv_step,
        "logical_gbs": kv_step / (ms_per_step * 1e-3) / 1e9,
        "kv_bytes_resident": lay.kv_bytes_live(),
        "kv_bytes_allocated": lay.kv_bytes_allocated(),
        "full_layer_ms": (sum(full_ms) / len(full_ms)) if full_ms else None,
        "full_layer_bytes": kv_full_launch + qo_bytes,
    }
    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.copy_calibration):
            dst.copy_(src)
        torch.cuda.synchronize()
    lay.close()
    del lay
    torch.cuda.empty_cache()
    return res


def cpu_baseline_decode(wl, torch, w, budget_s=15.0):
    """Times the fp64 oracle on a bounded sample of the decode workload and scales to tokens/s.

    Sample: one sequence, one KV head (its G query heads), one full layer at the workload's context and one
    sliding layer at its window, repeated until about `budget_s` seconds of CPU work were measured.
    Whole step = batch * n_kv_heads such samples per layer, 2 full + 22 sliding layers (linear scaling).
    """
    import numpy as np
    from oracle.mixattn_oracle import LayerSpec, OracleStack
    G, d = w.n_q_heads // w.n_kv_heads, w.head_dim
    n = w.context
    W = max(t[1] for t in w.layers)
    layers = [LayerSpec(0, 0, 0), LayerSpec(1, W, 1)]
    ora = OracleStack(layers, 1, G, 1, d)
    k = wl.randn(w.seed + 1, (n, 1, d), torch.bfloat16).double().numpy()
    v = wl.randn(w.seed + 2, (n, 1, d), torch.bfloat16).double().numpy()
    ora.load(0, k, v, [n])
    ora.load(1, k, v, [n])
    q = wl.randn(w.seed + 3, (1, G, d), torch.bfloat16).double().numpy()
    t_full = t_slide = 0.0
    reps = 0
    t_start = time.perf_counter()
    cpu_start = time.process_time()
    while time.perf_counter() - t_start < budget_s:
        a = time.perf_counter()
        ora.decode(0, q)
        b = time.perf_counter()
        ora.decode(1, q)
        c = time.perf_counter()
        t_full += b - a
        t_slide += c - b
        reps += 1
    wall = time.perf_counter() - t_start
    # threads the oracle's numpy calls actually kept busy: CPU time over wall time
    threads = max(1, int(round((time.process_time() - cpu_start) / wall)))
    t_full /= reps
    t_slide /= reps
    n_full = sum(1 for t in w.layers if t[0] == wl.FULL)
    n_slide = len(w.layers) - n_full
    step_s = w.batch * w.n_kv_heads * (n_full * t_full + n_slide * t_slide)
    return {
        "value": w.batch / step_s, "unit": "tokens/s", "cores": threads, "host_cores": os.cpu_count(), "kind": "oracle",
        "sample": "1 sequence x 1 KV head (%d query heads): one full-layer decode at n=%d and one sliding-layer "
                  "decode at W=%d, %d repetitions (%.1f s); scaled linearly to batch %d x %d KV heads x "
                  "(%d full + %d sliding layers); cores = threads the oracle's numpy calls kept busy (CPU time / "
                  "wall time), host_cores = os.cpu_count() of the box"
                  % (G, n, W, reps, time.perf_counter() - t_start, w.batch, w.n_kv_heads, n_full, n_slide),
    }


def run_prefill(args, mx, wl, torch, w):
    dev = "cuda:0"
    B, S, Hq, Hkv, d = w.batch, w.prefill_len, w.n_q_heads, w.n_kv_heads, w.head_dim
    lay = mx.Layout(w.layers, B, Hq, Hkv, d, capacity=[S] * B, kv_dtype="bf16", out_dtype=args.out_dtype,
                    **_paging(args.page_tokens, [S] * B))
    if args.prefill_waves:
        lay.set_param(mx.PARAM_PREFILL_WAVES, args.prefill_waves)
    if args.prefill_heads:
        lay.set_param(mx.PARAM_PREFILL_HEADS, args.prefill_heads)
    # one q per layer kind is enough to time (values do not change the cost); K/V per writer layer
    q = wl.randn(wl.layer_seed(w.seed, 0, "q"), (B, S, Hq, d), torch.bfloat16, dev)
    kv = {}
    for li in w.writer_layers():
        kv[li] = (wl.randn(wl.layer_seed(w.seed, li, "k"), (B, S, Hkv, d), torch.bfloat16, dev),
                  wl.randn(wl.layer_seed(w.seed, li, "v"), (B, S, Hkv, d), torch.bfloat16, dev))
    out = torch.empty((B, S, Hq, d), dtype=lay.out_torch, device=dev)
    writer_of = [lay.writer_of(li) for li in range(len(w.layers))]

    n_chunks = max(1, args.chunks)
    assert S % n_chunks == 0
    C = S // n_chunks

    def step(events=None):
        lay.reset()
        for ch in range(n_chunks):  # chunk by chunk through the whole stack, as a serving loop would
            sl = slice(ch * C, (ch + 1) * C)
            for li in range(len(w.layers)):
                k, v = kv[writer_of[li]]
                kk, vv = k[:, sl], v[:, sl]
                if n_chunks > 1:
                    kk, vv = kk.contiguous(), vv.contiguous()
                if writer_of[li] != li:
                    kk = vv = None  # readers follow their writer directly: reuse the staged prompt
                qq = q[:, sl].contiguous() if n_chunks > 1 else q
                oo = out[:, sl] if n_chunks == 1 else out_chunk
                timed = events is not None and li == 0 and ch == n_chunks - 1
                if timed:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record()
                lay.prefill(li, qq, kk, vv, oo)
                if timed:
                    e1.record()
                    events.append((e0, e1))

    out_chunk = torch.empty((B, C, Hq, d), dtype=lay.out_torch, device=dev) if n_chunks > 1 else None
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    pairs_full = S * (S + 1) // 2
    flops = 0
    for kind, W, _ in w.layers:
        pairs = pairs_full if kind == wl.FULL or W >= S else (W * (W + 1) // 2 + (S - W) * W)
        flops += 4 * d * pairs * Hq * B
    full_ms = sum(e0.elapsed_time(e1) for e0, e1 in events) / len(events)
    lay.close()
    return {"ms_per_step": ms, "flops": flops, "tflops": flops / (ms * 1e-3) / 1e12,
            "full_layer_ms": full_ms, "full_layer_flops": 4 * d * pairs_full * Hq * B}


def run_generation(args, mx, wl, torch, layers, label):
    """Prompt prefill followed by a generation loop through the attention stack (Section 4, "Inference Speed and
    Memory Consumption": 31000 input and 1000 output tokens per request).  Every sequence of the batch has the same
    prompt length; one K/V prompt tensor pair and one set of per-token tensors are reused for all layers (values do
    not change the cost)."""
    dev = "cuda:0"
    B, S, T = args.gen_batch, args.gen_prompt, args.gen_new
    Hq, Hkv, d = 32, 8, 128
    lay = mx.Layout(layers, B, Hq, Hkv, d, capacity=[S + T] * B, kv_dtype="bf16", out_dtype=args.out_dtype,
                    **_paging(args.page_tokens, [S + T] * B))
    writer_of = [lay.writer_of(li) for li in range(len(layers))]
    q = wl.randn(1, (B, S, Hq, d), torch.bfloat16, dev)
    k = wl.randn(2, (B, S, Hkv, d), torch.bfloat16, dev)
    v = wl.randn(3, (B, S, Hkv, d), torch.bfloat16, dev)
    out = torch.empty((B, S, Hq, d), dtype=lay.out_torch, device=dev)
    q1 = wl.randn(4, (B, Hq, d), torch.bfloat16, dev)
    k1 = wl.randn(5, (B, Hkv, d), torch.bfloat16, dev)
    v1 = wl.randn(6, (B, Hkv, d), torch.bfloat16, dev)
    out1 = torch.empty((B, Hq, d), dtype=lay.out_torch, device=dev)

    def prefill():
        for li in range(len(layers)):
            if writer_of[li] == li:
                lay.prefill(li, q, k, v, out)
            else:
                lay.prefill(li, q, None, None, out)   # readers reuse the prompt copy their cache keeps staged

    def decode_step():
        for li in range(len(layers)):
            if writer_of[li] == li:
                lay.append_decode(li, k1, v1, q1, out1)
            else:
                lay.decode(li, q1, out1)

    # warm-up on the same layout (kernels, planner memo), then the timed run from empty caches
    prefill()
    for _ in range(3):
        decode_step()
    torch.cuda.synchronize()
    lay.reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    prefill()
    staging = lay.staging_bytes()
    lay.release_prefill()   # the prompt copies are not needed by the generation loop (synchronises)
    t1 = time.perf_counter()
    for _ in range(T):
        decode_step()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    r = {"label": label, "batch": B, "prompt": S, "new_tokens": T, "prefill_s": t1 - t0, "decode_s": t2 - t1,
         "total_s": t2 - t0, "output_tokens_per_s": B * T / (t2 - t0), "decode_only_tokens_per_s": B * T / (t2 - t1),
         "ms_per_decode_step": (t2 - t1) * 1e3 / T, "kv_bytes_resident": lay.kv_bytes_live(),
         "kv_bytes_allocated": lay.kv_bytes_allocated(), "staging_bytes_during_prefill": staging}
    lay.close()
    return r


def run_serving(args, mx, wl, torch, layers, label):
    """Requests of mixed lengths served through a fixed number of batch slots (Section 4 measures 300 requests
    through a serving engine): a slot whose request has produced its last token is released and idles until the
    next request's prompt is prefilled into it (several new prompts go through the stack in one variable-length
    call), while the other slots keep decoding.  Full caches are paged; values of q/k/v do not change the cost, so
    one set of tensors serves all layers."""
    import random
    dev = "cuda:0"
    B, R = args.serve_slots, args.serve_requests
    Hq, Hkv, d = 32, 8, 128
    rng = random.Random(20240915)
    reqs = [(rng.randint(*args.serve_prompt), rng.randint(*args.serve_new)) for _ in range(R)]
    p_max, t_max = args.serve_prompt[1], args.serve_new[1]
    cap = [p_max + t_max] * B
    page = args.page_tokens or 256
    lay = mx.Layout(layers, B, Hq, Hkv, d, capacity=cap, kv_dtype="bf16", out_dtype=args.out_dtype,
                    **_paging(page, cap))
    writer_of = [lay.writer_of(li) for li in range(len(layers))]
    rows = B * p_max
    q = wl.randn(1, (rows, Hq, d), torch.bfloat16, dev)
    k = wl.randn(2, (rows, Hkv, d), torch.bfloat16, dev)
    v = wl.randn(3, (rows, Hkv, d), torch.bfloat16, dev)
    out = torch.empty((rows, Hq, d), dtype=lay.out_torch, device=dev)
    q1 = wl.randn(4, (B, Hq, d), torch.bfloat16, dev)
    k1 = wl.randn(5, (B, Hkv, d), torch.bfloat16, dev)
    v1 = wl.randn(6, (B, Hkv, d), torch.bfloat16, dev)
    out1 = torch.empty((B, Hq, d), dtype=lay.out_torch, device=dev)

    def prefill(lens):
        n = sum(lens)
        for li in range(len(layers)):
            if writer_of[li] == li:
                lay.prefill_varlen(li, q[:n], k[:n], v[:n], lens, out[:n])
            else:
                lay.prefill_varlen(li, q[:n], None, None, lens, out[:n])   # the cache's staged copy of the chunk

    def decode_step():
        for li in range(len(layers)):
            if writer_of[li] == li:
                lay.append_decode(li, k1, v1, q1, out1)
            else:
                lay.decode(li, q1, out1)

    def serve(requests):
        pending = list(requests)
        for b in range(B):      # every slot starts idle
            lay.release_sequence(b)
        left = [0] * B          # tokens the slot's request still has to generate (0: idle)
        steps = prefills = generated = prompt_tokens = 0
        while pending or any(left):
            lens = [0] * B
            for b in range(B):
                if left[b] == 0 and pending:
                    p_len, t_len = pending.pop(0)
                    lens[b], left[b] = p_len, t_len
            if any(lens):
                prefill(lens)
                prefills += 1
                prompt_tokens += sum(lens)
            decode_step()
            steps += 1
            for b in range(B):
                if left[b]:
                    generated += 1
                    left[b] -= 1
                    if left[b] == 0:
                        lay.release_sequence(b)
        return steps, prefills, generated, prompt_tokens

    # warm-up: a few short requests through every code path (kernels, staging areas, planner), then start over
    serve([(args.serve_prompt[1], 3)] * min(B, 2) + [(1000, 2)] * 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    steps, prefills, generated, prompt_tokens = serve(reqs)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    r = {"label": label, "slots": B, "requests": R, "prompt_tokens": prompt_tokens, "generated_tokens": generated,
         "decode_steps": steps, "prefill_calls": prefills, "total_s": t1 - t0,
         "output_tokens_per_s": generated / (t1 - t0), "requests_per_s": R / (t1 - t0),
         "kv_bytes_allocated": lay.kv_bytes_allocated(), "staging_bytes": lay.staging_bytes(), "page_tokens": page}
    lay.close()
    del lay
    torch.cuda.empty_cache()
    return r


def ragged_comparison(args, mx, wl, torch, warmup, steps, cycle_caches):
    """Configuration 4: the MixAttention stack next to the standard 24-layer stack on a ragged batch of 64 (context
    lengths uniform in [1024, 65536]).  cycle_caches = 0: the standard stack is built whole (24 private caches, about
    209 GB).  cycle_caches = n > 0: it is timed as 24 full-attention layers that cycle over n distinct caches (n of
    them append, the others only read); every cache is far larger than the 256 MB last-level cache, so the HBM
    traffic of a step is that of 24 private caches, and its KV bytes are computed from the lengths.  -1: not run."""
    w = wl.config(4)
    a = argparse.Namespace(**vars(args))
    a.warmup, a.steps, a.only, a.group_decode = warmup, steps, "", False
    if a.graph < 0:
        a.graph = 1
    r_mix = run_decode(a, mx, wl, torch, w)
    per_tok = 2 * w.n_kv_heads * w.head_dim * 2
    ctx = sum(w.seq_lens)
    res = {"workload": w.name, "sum_context": int(ctx), "steps": steps, "warmup": warmup,
           "mix_ms_per_step": r_mix["ms_per_step"], "mix_eager_ms_per_step": r_mix["eager_ms_per_step"],
           "mix_tokens_per_s": r_mix["tokens_per_s"], "mix_logical_GBps": r_mix["logical_gbs"],
           "mix_kv_bytes_read_per_step": r_mix["kv_bytes_per_step"], "mix_kv_bytes_resident": r_mix["kv_bytes_resident"],
           "mix_full_layer_ms": r_mix["full_layer_ms"],
           "mix_full_layer_GBps": r_mix["full_layer_bytes"] / (r_mix["full_layer_ms"] * 1e-3) / 1e9,
           "mix_full_layer_bytes": r_mix["full_layer_bytes"]}
    res["mix_full_layer_traffic"], res["mix_full_layer_traffic_source"] = _traffic_from_profiles("decode_full_%s" % w.name)
    if cycle_caches < 0:
        return res
    torch.cuda.empty_cache()
    if cycle_caches == 0:
        layers, how = wl.layout_full24(), "24 private caches, built whole"
    else:
        layers = [(wl.FULL, 0, i % cycle_caches) for i in range(24)]
        how = ("24 full-attention launches per step cycling over %d distinct caches of %.1f GB each (each far larger "
               "than the last-level cache, so HBM traffic equals that of 24 private caches); KV bytes computed from "
               "the lengths" % (cycle_caches, ctx * per_tok / 1e9))
    r_std = run_decode(a, mx, wl, torch, w, layers=layers)
    res.update({"standard_ms_per_step": r_std["ms_per_step"], "standard_eager_ms_per_step": r_std["eager_ms_per_step"],
                "standard_logical_GBps": r_std["logical_gbs"], "standard_how": how,
                "standard_kv_bytes_read_per_step": r_std["kv_bytes_per_step"],
                "standard_kv_bytes_resident": 24 * ctx * per_tok,
                "step_time_ratio_standard_over_mix": r_std["ms_per_step"] / r_mix["ms_per_step"],
                "kv_bytes_ratio_standard_over_mix": 24 * ctx * per_tok / r_mix["kv_bytes_resident"]})
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus %d is not "
              "supported. Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2409_15012_amd import binding as mx
    from paper_2409_15012_amd import workloads as wl
    mx.load()
    if not torch.cuda.is_available():
        print("bench.py needs a GPU (the library has no CPU path)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    base = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic"}
    if args.workload in ("decode32k", "decode4k"):
        w = wl.config(2 if args.workload == "decode32k" else 1)
        if args.graph < 0:
            args.graph = 1
        r = run_decode(args, mx, wl, torch, w)
        line = dict(base)
        line.update({
            "metric": "decode tokens/s through the 24-layer MixAttention attention stack (decode-attn HBM GB/s "
                      "alongside)",
            "value": r["tokens_per_s"], "unit": "tokens/s", "ms_per_step": r["ms_per_step"],
            "config": {"workload": w.name, "batch": w.batch, "context": w.context, "window": 1024,
                       "layers": "24: 0,12 full; 22 sliding in groups {1-4,5-8,9-11},{13-16,17-20,21-23}",
                       "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                       "out_dtype": args.out_dtype, "only": args.only or "all", "page_tokens": args.page_tokens,
                       "group_decode": bool(args.group_decode),
                       "step": ("one HIP-graph replay of the captured step (8 fused append+decode launches, 16 decode "
                                "launches)" if r["graph_ms_per_step"] else "eager launches")},
            "eager_ms_per_step": r["eager_ms_per_step"], "graph_ms_per_step": r["graph_ms_per_step"],
            "kv_bytes_read_per_step": r["kv_bytes_per_step"],
            "kv_bytes_resident": r["kv_bytes_resident"],
            "decode_attn_logical_GBps": r["logical_gbs"],
            "decode_attn_pct_of_8TBps": 100.0 * r["logical_gbs"] / HBM_PEAK_GBS,
        })
        if r["full_layer_ms"]:
            ach = r["full_layer_bytes"] / (r["full_layer_ms"] * 1e-3) / 1e9
            traffic, traffic_note = _traffic_from_profiles("decode_full_%s" % w.name)
            line["roofline"] = {"kernel": "one full-attention layer with its fused append: decode_tiled_kernel<out, full, fused append>, or decode_balanced_kernel + combine_balanced_kernel when the planner cuts the blocks into equal runs",
                                "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                "frac": ach / HBM_PEAK_GBS, "launch_ms": r["full_layer_ms"],
                                "bytes_per_launch": r["full_layer_bytes"],
                                "traffic": traffic, "traffic_source": traffic_note}
        if args.workload == "decode32k" and not args.headline_only and not args.only and not args.group_decode:
            # the other two measurements the metric names, each on its own configuration, in the same run
            try:
                pa = argparse.Namespace(**vars(args))
                pa.warmup, pa.steps, pa.chunks = 1, 3, 1
                wp = wl.config(3)
                rp = run_prefill(pa, mx, wl, torch, wp)
                line["prefill"] = {
                    "workload": wp.name, "ms": rp["ms_per_step"], "tflops": rp["tflops"], "useful_flops": rp["flops"],
                    "full_layer_ms": rp["full_layer_ms"],
                    "full_layer_tflops": rp["full_layer_flops"] / (rp["full_layer_ms"] * 1e-3) / 1e12,
                    "full_layer_frac_of_2.5PF": rp["full_layer_flops"] / (rp["full_layer_ms"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "frac_of_2.5PF": rp["tflops"] / MFMA_BF16_PEAK_TFLOPS, "steps": pa.steps, "warmup": pa.warmup,
                    "note": "24-layer stack, batch 1, 32768-token prompt, unmasked pairs only; full_layer = layer 0 incl. cache commit"}
            except Exception as e:  # reported, never hidden
                line["prefill"] = {"error": repr(e)}
            torch.cuda.empty_cache()
            try:
                line["ragged64"] = ragged_comparison(args, mx, wl, torch, warmup=2, steps=10, cycle_caches=3)
            except Exception as e:
                line["ragged64"] = {"error": repr(e)}
            torch.cuda.empty_cache()
        if not args.no_cpu_baseline:
            line["cpu_baseline"] = cpu_baseline_decode(wl, torch, w)
    elif args.workload == "prefill32k":
        w = wl.config(3)
        r = run_prefill(args, mx, wl, torch, w)
        line = dict(base)
        ach = r["full_layer_flops"] / (r["full_layer_ms"] * 1e-3) / 1e12
        line.update({
            "metric": "prefill attention TFLOP/s (unmasked pairs only), 24-layer MixAttention stack",
            "value": r["tflops"], "unit": "TFLOP/s", "ms_per_step": r["ms_per_step"],
            "config": {"workload": w.name, "batch": 1, "seq_len": w.prefill_len, "window": 1024,
                       "out_dtype": args.out_dtype, "chunks": max(1, args.chunks), "page_tokens": args.page_tokens},
            "useful_flops_per_step": r["flops"],
            "roofline": None if args.chunks > 1 else {"kernel": "prefill_tiled_kernel (full causal layer, incl. cache commit)", "bound": "mfma",
                         "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": ach / MFMA_BF16_PEAK_TFLOPS, "launch_ms": r["full_layer_ms"], "traffic": None},
        })
    elif args.workload == "variants":
        # decode step of several layer layouts at the decode32k shape (batch 32, context 32768): how the mix of
        # standard / sliding layers and the amount of sharing move KV bytes and step time (Sections 3, 5.1, 5.2)
        w = wl.config(2)
        if args.graph < 0:
            args.graph = 1
        rows = {}
        for name, layers in [("mix24 (2 full unshared + 22 sliding in 6 groups)", wl.layout_mix24()),
                             ("ma-like (1 full cache read by 4 layers, sliding pairs)", wl.layout_variant("ma")),
                             ("ma-offset-like", wl.layout_variant("ma_offset")),
                             ("ma-pairs-like (2 full caches, each read twice)", wl.layout_variant("ma_pairs")),
                             ("all sliding, no sharing", wl.layout_variant("sliding")),
                             ("standard (24 full, no sharing)", wl.layout_full24())]:
            r = run_decode(args, mx, wl, torch, w, layers=layers)
            rows[name] = {"ms_per_step": r["ms_per_step"], "tokens_per_s": r["tokens_per_s"],
                          "kv_bytes_resident": r["kv_bytes_resident"], "kv_bytes_read_per_step": r["kv_bytes_per_step"],
                          "logical_GBps": r["logical_gbs"], "n_caches": len({c for _, _, c in layers})}
        base_row = rows["mix24 (2 full unshared + 22 sliding in 6 groups)"]
        line = dict(base)
        line.update({"metric": "decode tokens/s by layer layout, batch 32, context 32768", "value": base_row["tokens_per_s"],
                     "unit": "tokens/s", "ms_per_step": base_row["ms_per_step"],
                     "config": {"workload": "layout variants at " + w.name, "batch": w.batch, "context": w.context},
                     "layouts": rows})
    elif args.workload == "gen31k":
        r_mix = run_generation(args, mx, wl, torch, wl.layout_mix24(), "mix24")
        line = dict(base)
        line.update({
            "metric": "output tokens/s, %d-token prompts + %d generated tokens, batch %d, attention stack only "
                      "(prefill + generation loop)" % (args.gen_prompt, args.gen_new, args.gen_batch),
            "value": r_mix["output_tokens_per_s"], "unit": "tokens/s", "steps": args.gen_new, "warmup": 3,
            "ms_per_step": r_mix["ms_per_decode_step"],
            "config": {"workload": "gen_b%d_in%d_out%d" % (args.gen_batch, args.gen_prompt, args.gen_new),
                       "batch": args.gen_batch, "prompt": args.gen_prompt, "new_tokens": args.gen_new,
                       "window": 1024, "out_dtype": args.out_dtype, "page_tokens": args.page_tokens},
            "mix": r_mix,
        })
        if args.with_standard:
            r_std = run_generation(args, mx, wl, torch, wl.layout_full24(), "standard24")
            line["standard"] = r_std
            line["total_time_ratio_standard_over_mix"] = r_std["total_s"] / r_mix["total_s"]
            line["kv_bytes_ratio_standard_over_mix"] = r_std["kv_bytes_resident"] / r_mix["kv_bytes_resident"]
    elif args.workload == "serve":
        r_mix = run_serving(args, mx, wl, torch, wl.layout_mix24(), "mix24")
        line = dict(base)
        line.update({
            "metric": "output tokens/s, %d requests of mixed lengths through %d batch slots, attention stack only "
                      "(continuous batching: paged full caches, idle slots, variable-length prefill)"
                      % (args.serve_requests, args.serve_slots),
            "value": r_mix["output_tokens_per_s"], "unit": "tokens/s", "steps": r_mix["decode_steps"], "warmup": 0,
            "ms_per_step": r_mix["total_s"] * 1e3 / r_mix["decode_steps"],
            "config": {"workload": "serve_r%d_b%d" % (args.serve_requests, args.serve_slots),
                       "prompt_range": args.serve_prompt, "new_token_range": args.serve_new, "window": 1024,
                       "out_dtype": args.out_dtype},
            "mix": r_mix,
        })
        if args.with_standard:
            r_std = run_serving(args, mx, wl, torch, wl.layout_full24(), "standard24")
            line["standard"] = r_std
            line["total_time_ratio_standard_over_mix"] = r_std["total_s"] / r_mix["total_s"]
            line["kv_bytes_ratio_standard_over_mix"] = r_std["kv_bytes_allocated"] / r_mix["kv_bytes_allocated"]
    else:  # ragged64
        r = ragged_comparison(args, mx, wl, torch, warmup=args.warmup, steps=args.steps,
                              cycle_caches=0 if not args.skip_standard else -1)
        w = wl.config(4)
        line = dict(base)
        line.update({
            "metric": "decode tokens/s, ragged batch 64, MixAttention stack (standard 24-layer stack alongside)",
            "value": r["mix_tokens_per_s"], "unit": "tokens/s", "ms_per_step": r["mix_ms_per_step"],
            "config": {"workload": w.name, "batch": w.batch, "context": "uniform[1024,65536] seeded",
                       "sum_context": int(sum(w.seq_lens)), "window": 1024, "out_dtype": args.out_dtype},
            "ragged64": r,
            "roofline": {"kernel": "one full-attention layer of the ragged batch: decode_balanced_kernel<out, fused append> + combine_balanced_kernel",
                         "bound": "hbm", "achieved": r["mix_full_layer_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": r["mix_full_layer_GBps"] / HBM_PEAK_GBS, "launch_ms": r["mix_full_layer_ms"],
                         "bytes_per_launch": r["mix_full_layer_bytes"], "traffic": r["mix_full_layer_traffic"],
                         "traffic_source": r["mix_full_layer_traffic_source"]},
        })
    print(json.dumps(line))


if __name__ == "__main__":
    main()
