#!/usr/bin/env python3
"""Benchmark of the chunked-prefill hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload opt13b] [--mode eager|graph]

One "step" is one pass of the whole hot path over one scheduled batch of synthetic input: host chunk
packing + per-chunk metadata, one metadata upload, then for every chunk in order ONE launch that does the
chunk's attention and its KV append (TetriInfer Sec. 3.3.3: prefill one ChunkSize chunk at a time;
--two-launches runs the two kernels separately).  Q/K/V of every chunk and the page pool are resident in
HBM before the timed region.  Prints ONE JSON line.

`value` = algorithmic attention flops of a step / step time with a COLD cache: consecutive steps rotate over
independent copies of every buffer the caller owns (inputs, output, page pool, metadata; one library handle), so
that more than twice the 256 MB last-level cache is touched before a buffer comes round again.  `warm_cache` is
the same step on one set of buffers, back to back.  `roofline` is the attention kernel alone, its launch durations
measured with HIP events (on the launch stream) around graph-replayed groups of launches that rotate over the same
buffer sets.

Beside the contract's fields the line carries stand-alone measurements taken after the timed region:
`per_chunk`, `roofline.per_chunk_bound_frac` (each chunk against the roofline that binds it:
max(flops / MFMA peak, bytes / HBM peak) / duration), `roofline.library_gemm_same_box` (what the vendor library's bf16
GEMM reaches on the same box, for scale), `append`, `kv_transfer` (request-level KV export /
import, Sec. 3.3.4), `fp8_prefill` (the first chunks' fused launches over a cache of FP8 codes, against the same
launches over the 16-bit pool), `decode` (one decode iteration of 64 requests x 2048 cached tokens on the same head
shape, 16-bit and FP8 cache) and `cpu_baseline` (the CPU oracle on this machine's host cores over a bounded sample of the same
workload).  Other modes: --policy / --sched-batch (prefill scheduler, Sec. 3.3.2), --chunk-size /
--prompt-len, --sweep (the ChunkSize saturation experiment of Sec. 2.2 in one run), --layer-sweep (the same
for a whole decoder layer), --export (KV export inside the step).
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, scaled
# by a plain copy of known size.  A profiled figure, not one of this run: (bytes, the summary that holds it).
PROFILED_TRAFFIC = {("opt13b", "fused"): (76.3e6, "profiles/attn_tile_kernel_opt13b_hbm_traffic.md")}


# ---- algorithmic work of a chunk: what the method must do (masked pairs and padding rows count zero)
def chunk_pairs(segs):
    """Unmasked (query, key) pairs per query head: sum over segments of n * ctx + n (n + 1) / 2."""
    return sum(n * start + n * (n + 1) // 2 for _req, start, n in segs)


def chunk_flops(segs, hq, d):
    """QK^T and PV: 4 * D * Hq * pairs."""
    return 4 * d * hq * chunk_pairs(segs)


def chunk_attn_bytes(segs, hq, hkv, d, page=16):
    """HBM bytes of one attention launch: Q in and out once, K and V once, the block table."""
    n = sum(x[2] for x in segs)
    kv = sum((start + ln) * hkv * d * 2 * 2 for _r, start, ln in segs)
    bt = sum(-(-start // page) * 4 for _r, start, _ln in segs)
    return 2 * n * hq * d * 2 + kv + bt


def chunk_append_bytes(segs, hkv, d):
    """The new K and V rows read once more and written once."""
    n = sum(x[2] for x in segs)
    return 2 * 2 * n * hkv * d * 2


def set_options(pipe, args):
    if args.variant is not None:
        pipe.handle.tetri_set_option("attn_variant", args.variant)
    for kv in args.opt:
        key, value = kv.split("=")
        pipe.handle.tetri_set_option(key, int(value))


def layer_sweep(torch, np, synth, tetri, PrefillPipeline, dev):
    """Throughput and latency of one OPT-13B-shaped decoder layer's prefill against the prompt length C
    (one chunk, empty cache): where throughput goes flat is the accelerator-saturate threshold that
    Sec. 2.2 / Sec. 3.3.3 take as ChunkSize.  The attention is this library's fused launch; the four
    projections (QKV 5120x15360, out 5120x5120, MLP 5120x20480 and back) are library GEMMs through
    torch.matmul, here only as the context the paper's experiment needs."""
    hidden, heads, d = 5120, 40, 128
    shapes = [(hidden, 3 * hidden), (hidden, hidden), (hidden, 4 * hidden), (4 * hidden, hidden)]
    weights = [(torch.randn(k, n, device=dev) * 0.02).to(torch.bfloat16) for k, n in shapes]

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1) / reps

    rows = []
    for C in (128, 256, 512, 1024, 2048, 4096, 8192):
        w = dataclasses.replace(synth.workload("opt13b"), prompt_lens=[C], order=[0], chunk_size=C,
                                num_pages=C // 16 + 8)
        pipe = PrefillPipeline(w.prompt_lens, w.order, C, heads, heads, d, w.num_pages, synth.place_pages(w), w.scale,
                               device=dev)
        q = (torch.randn((1, C, heads, d), device=dev) * w.std).to(torch.bfloat16)
        k = (torch.randn((1, C, heads, d), device=dev) * w.std).to(torch.bfloat16)
        v = torch.randn_like(k)
        out = torch.zeros_like(q)
        pool = synth.pool_sentinel((w.num_pages, 2, heads, 16, d), device=dev)
        pipe.bind(q, k, v, pool, out)
        pipe.step()
        torch.cuda.synchronize()
        attn_ms = timed(lambda: pipe.launch_fused(0))
        x = [(torch.randn(C, kdim, device=dev) * 0.02).to(torch.bfloat16) for kdim, _n in shapes]
        gemm_ms = sum(timed(lambda i=i: torch.matmul(x[i], weights[i])) for i in range(4))
        attn_flops = chunk_flops(pipe.chunk_segments(0), heads, d)
        gemm_flops = sum(2.0 * C * kdim * n for kdim, n in shapes)
        rows.append({"C": C, "attn_ms": round(attn_ms, 5), "gemm_ms": round(gemm_ms, 5),
                     "layer_ms": round(attn_ms + gemm_ms, 5),
                     "attn_tflops": round(attn_flops / attn_ms / 1e9, 1), "gemm_tflops": round(gemm_flops / gemm_ms / 1e9, 1),
                     "layer_tflops": round((attn_flops + gemm_flops) / (attn_ms + gemm_ms) / 1e9, 1),
                     "tokens_per_ms": round(C / (attn_ms + gemm_ms), 1)})
        del pipe, pool
    print(json.dumps({"metric": "layer_prefill_saturation_sweep", "unit": "TFLOP/s", "data": "synthetic",
                      "config": {"workload": "one OPT-13B-shaped decoder layer (hidden 5120, 40x128 heads), one prompt of C tokens, "
                                             "empty cache, bf16; attention = this library, projections = library GEMMs"},
                      "rows": rows}))
    return 0


def chunk_sweep(torch, np, synth, tetri, PrefillPipeline, dev, args):
    """The saturation experiment of Sec. 2.2 (the token count per iteration beyond which prefill throughput stays
    flat) for the attention of one prompt of --prompt-len tokens (default 8192) with the workload's head shape: one
    row per ChunkSize, the whole step (pack, metadata, upload, every chunk's fused launch) timed on one set of
    buffers.  One JSON line."""
    base = synth.workload(args.workload)
    plen = args.prompt_len or 8192
    rows = []
    for C in (128, 256, 512, 1024, 2048, 4096, 8192):
        if C > plen:
            break
        w = dataclasses.replace(base, prompt_lens=[plen], order=[0], chunk_size=C, num_pages=-(-plen // base.page_size) + 64)
        pipe = PrefillPipeline(w.prompt_lens, w.order, C, w.num_q_heads, w.num_kv_heads, w.head_dim, w.num_pages,
                               synth.place_pages(w), w.scale, device=dev, page_size=w.page_size)
        set_options(pipe, args)
        nC = pipe.n_chunks
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed)
        q = (torch.randn((nC, C, w.num_q_heads, w.head_dim), device=dev, generator=gen) * w.std).to(torch.bfloat16)
        k = (torch.randn((nC, C, w.num_kv_heads, w.head_dim), device=dev, generator=gen) * w.std).to(torch.bfloat16)
        v = (torch.randn((nC, C, w.num_kv_heads, w.head_dim), device=dev, generator=gen) * w.std).to(torch.bfloat16)
        out = torch.zeros_like(q)
        pool = synth.pool_sentinel((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), device=dev)
        pipe.bind(q, k, v, pool, out)
        flops = sum(chunk_flops(pipe.chunk_segments(c), w.num_q_heads, w.head_dim) for c in range(nC))
        for _ in range(10):
            pipe.step()
        torch.cuda.synchronize()
        steps = max(10, min(100, args.steps))
        t0 = time.perf_counter()
        for _ in range(steps):
            pipe.step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        tf = flops / (ms * 1e-3) / 1e12
        rows.append({"chunk_size": C, "chunks": nC, "steps": steps, "ms_per_step": round(ms, 5), "ms_per_chunk": round(ms / nC, 5),
                     "tflops": round(tf, 1), "frac_of_mfma_peak": round(tf / PEAK_BF16_MFMA_TFLOPS, 4),
                     "tokens_per_ms": round(plen / ms, 1)})
        del pipe, pool, q, k, v, out
    print(json.dumps({"metric": "chunk_size_saturation_sweep", "unit": "TFLOP/s", "data": "synthetic", "dtype": "bf16", "n_gpus": 1,
                      "config": {"workload": "%s head shape (%dx%d query heads, %d kv heads, page size %d): one prompt of %d tokens, "
                                             "whole step per ChunkSize, one set of buffers, seed %d" % (
                                                 base.name, base.num_q_heads, base.head_dim, base.num_kv_heads, base.page_size, plen,
                                                 base.seed)},
                      "rows": rows}))
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="opt13b", choices=["tiny", "opt13b", "packed", "heavy", "gqa"])
    ap.add_argument("--mode", default="eager", choices=["graph", "eager"])
    ap.add_argument("--settle", type=float, default=0.5, help="seconds of untimed steps before the warmup")
    ap.add_argument("--two-launches", action="store_true", help="separate attention and append launches per chunk")
    ap.add_argument("--calib-copy", action="store_true",
                    help="finish with one 256 MiB device-to-device copy (known traffic, to calibrate HBM counters)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--variant", type=int, default=None, help="attention kernel variant (measurement only)")
    ap.add_argument("--opt", action="append", default=[], metavar="KEY=VALUE",
                    help="tetri_set_option on the benchmark's handles (measurement only), e.g. --opt split_keys=0")
    ap.add_argument("--buffer-sets", type=int, default=0,
                    help="independent copies of every buffer that the steps rotate over (0: enough to touch more than "
                         "twice the last-level cache between repeats; 1: one set, a warm cache)")
    ap.add_argument("--policy", default=None, choices=["fcfs", "sjf", "ljf"],
                    help="order the workload's requests with tetri_schedule (Sec. 3.3.2) before packing")
    ap.add_argument("--sched-batch", type=int, default=0, help="PrefillSchedBatch: requests per sorted group (0: all)")
    ap.add_argument("--export", default=None, choices=["request", "chunk"],
                    help="add the KV export to the step: after the last chunk (request-level) or per chunk on a second "
                         "stream while the next chunk is prefilled (chunk-level), Sec. 3.3.4")
    ap.add_argument("--layer-sweep", action="store_true",
                    help="instead of the benchmark: the paper's saturation experiment (Sec. 2.2) for one 13B-shaped "
                         "decoder layer: this library's attention of a C-token prompt plus the layer's four projections "
                         "as plain library GEMMs, for C = 128 .. 8192")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark: the ChunkSize saturation sweep (Sec. 2.2) of one prompt of --prompt-len "
                         "tokens (default 8192) for ChunkSize 128 .. 8192; one JSON line with a row per ChunkSize")
    ap.add_argument("--chunk-size", type=int, default=None, help="ChunkSize override")
    ap.add_argument("--prompt-len", type=int, default=None, help="replace the workload's prompts by one prompt of this length")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2401_11181_amd import synth, tetri
    from paper_2401_11181_amd.prefill import PrefillPipeline

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.layer_sweep:
        return layer_sweep(torch, np, synth, tetri, PrefillPipeline, dev)
    if args.sweep:
        return chunk_sweep(torch, np, synth, tetri, PrefillPipeline, dev, args)
    w = synth.workload(args.workload)
    if args.prompt_len is not None:
        w = dataclasses.replace(w, name=w.name + "-len%d" % args.prompt_len, prompt_lens=[args.prompt_len], order=[0],
                                num_pages=max(w.num_pages, -(-args.prompt_len // w.page_size) + 64))
    if args.chunk_size is not None:
        w = dataclasses.replace(w, name=w.name + "-chunk%d" % args.chunk_size, chunk_size=args.chunk_size)
    if args.policy is not None:
        order = tetri.tetri_schedule(w.prompt_lens, {"fcfs": tetri.TETRI_FCFS, "sjf": tetri.TETRI_SJF, "ljf": tetri.TETRI_LJF}[args.policy],
                                     args.sched_batch)
        w = dataclasses.replace(w, name="%s-%s%d" % (w.name, args.policy, args.sched_batch), order=[int(x) for x in order])
    tables = synth.place_pages(w)
    fused = not args.two_launches

    def new_pipe(export=None, handle=None):
        pp = PrefillPipeline(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                             w.num_pages, tables, w.scale, device=dev, page_size=w.page_size,
                             use_graph=(args.mode == "graph"), fused=fused, export=export, handle=handle)
        if handle is None:
            set_options(pp, args)
        return pp

    pipe = new_pipe(args.export)
    nC, C = pipe.n_chunks, w.chunk_size
    segs_of = [pipe.chunk_segments(c) for c in range(nC)]

    # inputs: what the QKV projection of each chunk would hand to this path, resident in HBM
    q = torch.zeros((nC, C, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    k = torch.zeros((nC, C, w.num_kv_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    v = torch.zeros_like(k)
    out = torch.zeros_like(q)
    host_reqs = {}
    for c in range(nC):
        at = 0
        for req, start, n in segs_of[c]:
            if req not in host_reqs:
                host_reqs[req] = synth.request_qkv(w, req)
            rq, rk, rv = host_reqs[req]
            q[c, at:at + n] = rq[start:start + n].to(dev)
            k[c, at:at + n] = rk[start:start + n].to(dev)
            v[c, at:at + n] = rv[start:start + n].to(dev)
            at += n
            if start + n == w.prompt_lens[req] and args.workload in ("packed", "gqa"):
                del host_reqs[req]
    pool = synth.pool_sentinel((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), device=dev)
    pipe.bind(q, k, v, pool, out)

    flops = [chunk_flops(s, w.num_q_heads, w.head_dim) for s in segs_of]
    attn_bytes = [chunk_attn_bytes(s, w.num_q_heads, w.num_kv_heads, w.head_dim, w.page_size) for s in segs_of]
    app_bytes_of = [chunk_append_bytes(s, w.num_kv_heads, w.head_dim) for s in segs_of]
    total_flops = float(sum(flops))

    # ---- cold cache: independent copies of every buffer (inputs, output, page pool) that consecutive steps rotate
    # over, so that more than twice the 256 MB last-level cache is touched before a buffer comes round again.  In a
    # model the chunk's own rows are warm (the projection just wrote them) and the cached context is cold: the
    # truth lies between this figure and `warm_cache`.
    per_set = (q.numel() + k.numel() + v.numel() + out.numel()) * 2 + sum(w.prompt_lens) * 2 * w.num_kv_heads * w.head_dim * 2
    n_sets = args.buffer_sets or int(min(16, max(4, -(-(600 << 20) // per_set) + 1)))
    if n_sets * (pool.numel() * 2 + per_set) > (96 << 30) or args.export:
        n_sets = 1
    sets, keep = [pipe], []
    for _ in range(n_sets - 1):
        pp = new_pipe(handle=pipe.handle)           # one handle: the library's own scratch memory is the same in every step
        bufs = (q.clone(), k.clone(), v.clone(), pool.clone(), torch.zeros_like(out))
        pp.bind(*bufs)
        keep.append(bufs)
        sets.append(pp)

    # ---- settle: a fresh process shows one stall of tens of milliseconds a few hundred steps in
    # (clocks / runtime start-up); run past it, untimed, before the W warmup steps
    t_settle = time.perf_counter()
    n_settle = 0
    while time.perf_counter() - t_settle < args.settle:
        for i in range(20):
            sets[i % n_sets].step()
        torch.cuda.synchronize()
        n_settle += 20
    # ---- warmup, then exactly K timed steps bracketed by synchronisations
    for i in range(args.warmup):
        sets[i % n_sets].step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        sets[i % n_sets].step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # ---- the same on one set of buffers, back to back
    warm = None
    if n_sets > 1:
        for _ in range(args.warmup):
            pipe.step()
        torch.cuda.synchronize()
        tw0 = time.perf_counter()
        for _ in range(args.steps):
            pipe.step()
        torch.cuda.synchronize()
        warm_ms = (time.perf_counter() - tw0) * 1e3 / args.steps
        warm = {"value": round(total_flops / (warm_ms * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "ms_per_step": round(warm_ms, 5),
                "steps": args.steps}

    # ---- per-kernel durations: HIP events (on the launch stream) around groups of R back-to-back launches of one
    # chunk's kernel, replayed from a HIP graph so that the host launch path does not sit between the kernels;
    # duration = group time / R.  The i-th launch of a group runs on buffer set i mod n_sets.
    R = max(10, n_sets) // n_sets * n_sets
    reps = max(3, min(20, args.steps // 10))
    stream = torch.cuda.current_stream()
    spread = []                                     # (p10, p90) of every group_time call, in call order

    def group_time(launch):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(R):
                launch(i)
        g.replay()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            g.replay()
            e1.record(stream)
            e1.synchronize()
            times.append(e0.elapsed_time(e1) / R)
        spread.append((float(np.percentile(times, 10)), float(np.percentile(times, 90))))
        return float(np.median(times))

    torch.cuda.synchronize()
    for pp in sets:
        pp.host_plan(0)
        pp.meta_dev.copy_(pp.stage[0])
    torch.cuda.synchronize()
    n_meas = min(nC, 64)
    if fused:
        attn_ms = np.array([group_time(lambda i, c=c: sets[i % n_sets].launch_fused(c)) for c in range(n_meas)])
    else:
        attn_ms = np.array([group_time(lambda i, c=c: sets[i % n_sets].launch_attn(c)) for c in range(n_meas)])
    app_ms = np.array([group_time(lambda i, c=c: sets[i % n_sets].launch_append(c)) for c in range(min(nC, 8))])
    warm_attn_ms = None
    if n_sets > 1:
        warm_attn_ms = [group_time(lambda i, c=c: (pipe.launch_fused(c) if fused else pipe.launch_attn(c))) for c in range(min(nC, 8))]
        warm["attn_ms_median"] = [round(x, 5) for x in warm_attn_ms]
        warm["note"] = "attn_ms_median: the first %d chunks' launches, each repeated on one set of buffers" % len(warm_attn_ms)
    attn_avg_ms = float(attn_ms.mean())                 # average duration of one attention launch
    attn_flops_per_launch = float(sum(flops[:n_meas])) / n_meas
    achieved_tflops = attn_flops_per_launch / (attn_avg_ms * 1e-3) / 1e12
    launch_bytes = [attn_bytes[c] + (app_bytes_of[c] if fused else 0) for c in range(n_meas)]
    app_bytes = float(np.mean(app_bytes_of[:len(app_ms)]))
    app_avg_ms = float(app_ms.mean())
    # each chunk against the roofline that binds it: the longer of its MFMA time and its HBM time, over its duration
    mfma_s = [flops[c] / (PEAK_BF16_MFMA_TFLOPS * 1e12) for c in range(n_meas)]
    hbm_s = [launch_bytes[c] / (PEAK_HBM_GBS * 1e9) for c in range(n_meas)]
    bound_frac = [max(mfma_s[c], hbm_s[c]) / (float(attn_ms[c]) * 1e-3) for c in range(n_meas)]
    traffic, traffic_src = PROFILED_TRAFFIC.get((w.name, "fused" if fused else "two"), (None, None))

    result = {
        "metric": "chunked_prefill_attention_tflops",
        "value": round(value, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "settle_steps": n_settle,
        "ms_per_step": round(ms_per_step, 5),
        "ms_per_chunk": round(ms_per_step / nC, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "%s: %d prompt(s), %d tokens, %d chunks of ChunkSize %d, %dx%d query heads, %d kv heads, "
                        "page size %d, causal, seed %d" % (w.name, len(w.prompt_lens), sum(w.prompt_lens), nC, C,
                                                           w.num_q_heads, w.head_dim, w.num_kv_heads, w.page_size,
                                                           w.seed),
            "chunk_size": C, "launch_mode": args.mode, "kv_export_in_step": args.export,
            "cache": ("cold: steps rotate over %d independent sets of buffers, %d bytes touched between repeats" % (
                n_sets, int(per_set * (n_sets - 1)))) if n_sets > 1 else "warm: one set of buffers",
            "buffer_sets": n_sets,
            "segments_per_chunk": {"mean": round(float(np.mean([len(s) for s in segs_of])), 2),
                                   "max": int(max(len(s) for s in segs_of))},
            "step": "pack + metadata + upload + per chunk " +
                    ("(attention launch, kv append launch)" if args.two_launches else "one fused attention+append launch"),
        },
        "warm_cache": warm,
        "roofline": {
            "bound": "mfma", "kernel": "attn_tile_kernel" + ("" if args.two_launches else " (with fused kv append)"),
            "achieved": round(achieved_tflops, 3), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved_tflops / PEAK_BF16_MFMA_TFLOPS, 5),
            "avg_launch_ms": round(attn_avg_ms, 5), "flops_per_launch": attn_flops_per_launch,
            "launches_timed": "groups of %d graph-replayed launches rotating over %d buffer set(s)" % (R, n_sets),
            "traffic": traffic, "traffic_source": traffic_src,
            "algorithmic_bytes_per_launch": float(np.mean(launch_bytes)),
            "per_chunk_bound": ["mfma" if mfma_s[c] >= hbm_s[c] else "hbm" for c in range(n_meas)],
            "per_chunk_bound_frac": [round(x, 4) for x in bound_frac],
        },
        "per_chunk": {
            "attn_ms_median": [round(float(x), 5) for x in attn_ms],
            "attn_ms_p10": [round(spread[i][0], 5) for i in range(len(attn_ms))],
            "attn_ms_p90": [round(spread[i][1], 5) for i in range(len(attn_ms))],
            "attn_tflops": [round(flops[c] / (float(attn_ms[c]) * 1e-3) / 1e12, 2) for c in range(len(attn_ms))],
            "append_ms_median": [round(float(x), 5) for x in app_ms],
        },
        "append": {"kernel": "kv_append_kernel (stand-alone launch)", "avg_launch_ms": round(app_avg_ms, 5),
                   "achieved_GBs": round(app_bytes / (app_avg_ms * 1e-3) / 1e9, 1), "peak_GBs": PEAK_HBM_GBS,
                   "frac": round(app_bytes / (app_avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    }
    # what the last step left in set 0's output, for the check against the oracle below
    pipe.step()
    torch.cuda.synchronize()
    out_host = out.float().cpu().numpy()
    del sets[1:], keep

    # ---- the step after the hot path: request-level KV export of the whole batch and its import on a
    # receiver (Sec. 3.3.4), timed like the kernels above; moved bytes = payload read + payload written
    n_req = len(w.prompt_lens)
    total_tokens = int(sum(w.prompt_lens))
    payload = 2 * w.num_kv_heads * w.head_dim * total_tokens * 2
    if 0 < payload <= (8 << 30):
        d_bt = torch.from_numpy(np.ascontiguousarray(pipe.req_bt)).to(dev)
        d_cu = torch.from_numpy(np.concatenate([[0], np.cumsum(w.prompt_lens)]).astype(np.int32)).to(dev)
        xbuf = torch.zeros(payload // 2, dtype=torch.bfloat16, device=dev)
        exp_ms = group_time(lambda i: pipe.handle.tetri_kv_export(pool, d_bt, d_cu, None, n_req, total_tokens, xbuf))
        imp_ms = group_time(lambda i: pipe.handle.tetri_kv_import(xbuf, d_bt, d_cu, None, n_req, total_tokens, pool))
        result["kv_transfer"] = {
            "kernel": "kv_transfer_kernel (request-level, %d request(s), %d tokens)" % (n_req, total_tokens),
            "payload_bytes": payload, "bound": "hbm", "peak_GBs": PEAK_HBM_GBS,
            "export_ms": round(exp_ms, 5), "export_GBs": round(2 * payload / (exp_ms * 1e-3) / 1e9, 1),
            "export_frac": round(2 * payload / (exp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "import_ms": round(imp_ms, 5), "import_GBs": round(2 * payload / (imp_ms * 1e-3) / 1e9, 1),
            "import_frac": round(2 * payload / (imp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        }
        del xbuf

    # ---- for scale: what the vendor library's bf16 GEMM reaches on this machine right now (the 13B layer's QKV projection
    # on 8192 tokens through torch.matmul, 20 launches back to back between two events); context for roofline.frac, not a target
    ga = torch.randn((8192, 5120), device=dev).to(torch.bfloat16)
    gb = torch.randn((5120, 15360), device=dev).to(torch.bfloat16)
    gc_ = torch.empty((8192, 15360), dtype=torch.bfloat16, device=dev)
    for _ in range(3):
        torch.matmul(ga, gb, out=gc_)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(20):
        torch.matmul(ga, gb, out=gc_)
    e1.record(stream)
    e1.synchronize()
    gemm_ms = e0.elapsed_time(e1) / 20
    result["roofline"]["library_gemm_same_box"] = {
        "op": "torch.matmul bf16 8192x5120 @ 5120x15360", "ms": round(gemm_ms, 4),
        "tflops": round(2 * 8192 * 5120 * 15360 / (gemm_ms * 1e-3) / 1e12, 1),
        "frac_of_peak": round(2 * 8192 * 5120 * 15360 / (gemm_ms * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)}
    del ga, gb, gc_

    # ---- the same chunks over a cache of FP8 E4M3 codes (this build's extension): every chunk's fused launch
    # (attention over the codes cached so far + quantising append), repeated on one set of buffers like warm_cache
    if int(np.prod(pool.shape)) <= (16 << 30):
        k8 = v8 = float(w.std) / 32.0
        pool8 = torch.zeros(tuple(pool.shape), dtype=torch.uint8, device=dev)
        for c in range(nC):
            pipe.launch_fused_fp8(c, pool8, k8, v8, 1)
        torch.cuda.synchronize()
        n8 = min(nC, 8)
        fp8_ms = [group_time(lambda i, c=c: pipe.launch_fused_fp8(c, pool8, k8, v8, 1)) for c in range(n8)]
        ref_ms = warm_attn_ms if warm_attn_ms is not None else [float(x) for x in attn_ms[:n8]]
        result["fp8_prefill"] = {
            "kernel": "attn_tile_kernel<D, KS, FP8> (tetri_chunk_prefill_attn_fp8 with append, the first %d chunks)" % n8,
            "attn_ms_median": [round(x, 5) for x in fp8_ms],
            "tflops": round(float(sum(flops[:n8])) / (sum(fp8_ms) * 1e-3) / 1e12, 1),
            "time_vs_16_bit_pool": round(sum(fp8_ms) / sum(ref_ms[:n8]), 3) if fused else None,
        }
        del pool8

    # ---- the decode instance's counterpart (Sec. 3.4): one decode iteration of 64 requests with 2048
    # cached tokens each, same head shape, scattered pages; bytes = the cached K and V, read once
    dB, dctx = 64, 2048
    d_need = -(-(dctx + 1) // w.page_size)
    kv_bytes = dB * dctx * 2 * w.num_kv_heads * w.head_dim * 2
    if kv_bytes <= (16 << 30):
        dh = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, 64, dB * d_need, d_need, 8)
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed)
        dpool = (torch.randn((dB * d_need, 2, w.num_kv_heads, w.page_size, w.head_dim), device=dev, generator=gen) * w.std).to(torch.bfloat16)
        dq = (torch.randn((dB, w.num_q_heads, w.head_dim), device=dev, generator=gen) * w.std).to(torch.bfloat16)
        dk = (torch.randn((dB, w.num_kv_heads, w.head_dim), device=dev, generator=gen) * w.std).to(torch.bfloat16)
        dv = torch.randn(dk.shape, device=dev, generator=gen).to(torch.bfloat16)
        dout = torch.zeros_like(dq)
        dbt = torch.from_numpy(np.random.default_rng(w.seed).permutation(dB * d_need).astype(np.int32).reshape(dB, d_need)).to(dev)
        dcl = torch.full((dB,), dctx, dtype=torch.int32, device=dev)
        dec_ms = group_time(lambda i: dh.tetri_decode_attn(dq, dk, dv, dpool, dbt, dcl, dB, dctx, w.scale, dout))
        result["decode"] = {
            "kernel": "decode_attn_kernel (%d requests x %d cached tokens, %dx%d query heads, %d kv heads)" % (
                dB, dctx, w.num_q_heads, w.head_dim, w.num_kv_heads),
            "bound": "hbm", "kv_bytes": kv_bytes, "ms": round(dec_ms, 5),
            "achieved_GBs": round(kv_bytes / (dec_ms * 1e-3) / 1e9, 1), "peak_GBs": PEAK_HBM_GBS,
            "frac": round(kv_bytes / (dec_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "tokens_per_s": round(dB / (dec_ms * 1e-3), 1),
        }
        # the same iteration over an FP8 E4M3 cache (this build's extension): half the bytes
        dcodes = torch.randint(0, 0x78, tuple(dpool.shape), dtype=torch.uint8, device=dev, generator=gen)
        dec8_ms = group_time(lambda i: dh.tetri_decode_attn_fp8(dq, dk, dv, dcodes, dbt, dcl, dB, dctx, w.scale,
                                                                1.0 / 64, 1.0 / 64, 0, dout))
        result["decode"]["fp8"] = {
            "kernel": "decode_attn_kernel<D, FP8> (same batch, cache of E4M3 codes)", "kv_bytes": kv_bytes // 2,
            "ms": round(dec8_ms, 5), "achieved_GBs": round(kv_bytes / 2 / (dec8_ms * 1e-3) / 1e9, 1),
            "frac": round(kv_bytes / 2 / (dec8_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "tokens_per_s": round(dB / (dec8_ms * 1e-3), 1),
        }
        dh.close()
        del dpool, dcodes

    # ---- the CPU oracle on the host cores of this machine (reported baseline, not the target)
    if not args.no_cpu_baseline:
        from oracle import tetri_oracle
        from oracle import packer as opacker
        lib = tetri_oracle.load()
        threads = os.cpu_count() or 1
        omp = None
        try:
            import ctypes
            omp = ctypes.CDLL("libgomp.so.1")
            threads = int(omp.omp_get_max_threads())
        except OSError:
            pass
        plan = opacker.pack_chunks(w.prompt_lens, w.order, C)
        max_blocks = max(len(t) for t in tables)
        if w.num_pages <= 4096:
            # small pool: whole chunk passes of the same workload (attention + append, all heads) until about 10 s
            opool = np.zeros((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), dtype=np.float32)
            sample_flops, cpu_s, n_done, worst = 0.0, 0.0, 0, 0.0
            qh, kh, vh = q.float().cpu().numpy(), k.float().cpu().numpy(), v.float().cpu().numpy()
            n_pass = 0
            while cpu_s < 10.0 and n_pass < 50:
                opool[:] = 0
                for c, segs in enumerate(plan):
                    cu, ctx = opacker.chunk_arrays(segs)
                    bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
                    for i, (req, _s, _n) in enumerate(segs):
                        bt[i, :len(tables[req])] = tables[req]
                    ts = time.perf_counter()
                    o = tetri_oracle.chunk_prefill_attn(qh[c], kh[c], vh[c], opool, bt, cu, ctx, w.scale, lib=lib)
                    tetri_oracle.kv_append(kh[c], vh[c], opool, bt, cu, ctx, lib=lib)
                    cpu_s += time.perf_counter() - ts
                    sample_flops += flops[c]
                    n_done += 1
                    if n_pass == 0:
                        worst = max(worst, float(np.abs(o - out_host[c]).max()))
                    if cpu_s > 30.0:
                        break
                n_pass += 1
            result["cpu_baseline"] = {
                "value": round(sample_flops / cpu_s / 1e12, 6), "unit": "TFLOP/s", "cores": threads,
                "kind": "oracle", "seconds": round(cpu_s, 3),
                "sample": "%d chunk passes (attention + append, all heads) over the %d chunks of the same workload, "
                          "repeated until about 10 s of CPU time" % (n_done, nC),
            }
            result["parity_check"] = {"max_abs_vs_oracle": round(worst, 6), "chunks": min(n_done, nC)}
            # one thread: the first chunk of the same workload, once (if the OpenMP runtime lets the count be set)
            if omp is not None:
                try:
                    omp.omp_set_num_threads(1)
                    cu0, ctx0 = opacker.chunk_arrays(plan[0])
                    bt0 = np.zeros((len(plan[0]), max_blocks), dtype=np.int32)
                    for i, (req, _s, _n) in enumerate(plan[0]):
                        bt0[i, :len(tables[req])] = tables[req]
                    opool[:] = 0
                    ts = time.perf_counter()
                    tetri_oracle.chunk_prefill_attn(qh[0], kh[0], vh[0], opool, bt0, cu0, ctx0, w.scale, lib=lib)
                    one_s = time.perf_counter() - ts
                    omp.omp_set_num_threads(threads)
                    result["cpu_baseline"]["single_thread"] = {"value": round(flops[0] / one_s / 1e12, 6), "unit": "TFLOP/s",
                                                               "sample": "attention of chunk 0, once", "seconds": round(one_s, 3)}
                except AttributeError:
                    pass
        else:
            # large pool (the 16K-token prompt, the GQA batch): the oracle computes sampled (row, head) outputs of a few
            # chunks one by one, the cached context rebuilt in a compact pool with the oracle's own append (the
            # result does not depend on where the pages lie).  Chunks: for a batch, those that hold the two shortest
            # prompts and the longest prompt's last chunk; for one prompt the first, middle and last chunk.  All real
            # rows, every eighth query head.  Stops taking chunks after 30 s.
            by_len = np.argsort(w.prompt_lens, kind="stable")
            if len(w.prompt_lens) > 2:
                want = {int(by_len[0]), int(by_len[1])}
                chunks = [c for c, s in enumerate(plan) if any(r in want for r, _a, _n in s)][:4]
                chunks.append(max(c for c, s in enumerate(plan) if any(r == int(by_len[-1]) for r, _a, _n in s)))
                chunks = sorted(set(chunks))
            else:
                chunks = sorted({0, nC // 2, nC - 1})
            heads = np.arange(0, w.num_q_heads, 8, dtype=np.int32)
            cpu_s, sample_flops, worst, n_samples, done = 0.0, 0.0, 0.0, 0, []
            P, Hkv, D = w.page_size, w.num_kv_heads, w.head_dim
            for c in chunks:
                if cpu_s > 30.0:
                    break
                segs = plan[c]
                need = [-(-(start + n) // P) for _req, start, n in segs]
                cpool = np.zeros((max(1, sum(need)), 2, Hkv, P, D), dtype=np.float32)
                bt = np.zeros((len(segs), max(need)), dtype=np.int32)
                at = 0
                for i, (req, start, n) in enumerate(segs):
                    bt[i, :need[i]] = np.arange(at, at + need[i])
                    at += need[i]
                    if start > 0:
                        _rq, rk, rv = host_reqs[req] if req in host_reqs else synth.request_qkv(w, req)
                        tetri_oracle.kv_append(rk[:start].float().numpy(), rv[:start].float().numpy(), cpool, bt[i:i + 1],
                                               np.array([0, start], dtype=np.int32), np.array([0], dtype=np.int32), lib=lib)
                cu, ctx = opacker.chunk_arrays(segs)
                n_real = int(cu[-1])
                rows = np.repeat(np.arange(n_real, dtype=np.int32), len(heads))
                hh = np.tile(heads, n_real)
                qc, kc, vc = q[c].float().cpu().numpy(), k[c].float().cpu().numpy(), v[c].float().cpu().numpy()
                ts = time.perf_counter()
                ref = tetri_oracle.chunk_prefill_attn_samples(qc, kc, vc, cpool, bt, cu, ctx, w.scale, rows, hh, lib=lib)
                cpu_s += time.perf_counter() - ts
                sample_flops += flops[c] * len(heads) / w.num_q_heads
                n_samples += len(rows)
                done.append(c)
                worst = max(worst, float(np.abs(ref - out_host[c][rows, hh]).max()))
            cpu_tflops = sample_flops / cpu_s / 1e12
            result["cpu_baseline"] = {
                "value": round(cpu_tflops, 6), "unit": "TFLOP/s", "cores": threads, "kind": "oracle", "seconds": round(cpu_s, 3),
                "sample": "attention of chunks %s of the same workload: all real rows, query heads %s (%d (row, head) outputs, "
                          "%.1f GFLOP of the workload's %.1f)" % (done, [int(x) for x in heads], n_samples, sample_flops / 1e9,
                                                                total_flops / 1e9),
                "whole_workload_seconds_extrapolated": round(total_flops / (cpu_tflops * 1e12), 1),
                "extrapolation": "the workload's flops / the sample's rate: an estimate, not a measurement",
            }
            result["parity_check"] = {"max_abs_vs_oracle": round(worst, 6), "chunks": done, "samples": n_samples}
    if args.calib_copy:
        a = torch.zeros(256 << 20, dtype=torch.uint8, device=dev)
        b = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        torch.cuda.synchronize()
        a.copy_(b)
        torch.cuda.synchronize()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
