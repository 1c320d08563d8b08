#!/usr/bin/env python3
"""Benchmark of the chunked-prefill hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload opt13b] [--mode graph|eager]

One "step" is one pass of the whole hot path over one scheduled batch of synthetic input:
host chunk packing + per-chunk metadata, one metadata upload, then for every chunk in order one
attention launch and one KV-append launch (TetriInfer Sec. 3.3.3: prefill one ChunkSize chunk at
a time).  Q/K/V of every chunk and the page pool are resident in HBM before the timed region.
Prints ONE JSON line.  `value` = algorithmic attention flops of a step / step time.

Beside the contract's fields the line carries stand-alone measurements taken after the timed region (HIP
events around graph-replayed groups of launches): `per_chunk`, `append`, `kv_transfer` (request-level KV
export / import of the batch, Sec. 3.3.4) and `decode` (one decode iteration of 64 requests x 2048 cached
tokens on the same head shape).  Other modes: --policy / --sched-batch (prefill scheduler, Sec. 3.3.2),
--chunk-size / --prompt-len and --layer-sweep (the saturation experiment of Sec. 2.2), --export (KV export
inside the step at request or chunk granularity).
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
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by a
# plain copy of known size (figures and commands: profiles/attn_tile_kernel_opt13b_hbm_traffic.md)
MEASURED_TRAFFIC_BYTES = {("opt13b", "fused"): 76.5e6}


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
        attn_flops = pipe.flops(0)
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
                    help="tetri_set_option on the benchmark's handle (measurement only), e.g. --opt split_keys=0")
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
    ap.add_argument("--chunk-size", type=int, default=None, help="ChunkSize override (the saturation sweep of Sec. 2.2)")
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
    pipe = PrefillPipeline(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                           w.num_pages, tables, w.scale, device=dev, page_size=w.page_size,
                           use_graph=(args.mode == "graph"), fused=not args.two_launches, export=args.export)
    if args.variant is not None:
        pipe.handle.tetri_set_option("attn_variant", args.variant)
    for kv in args.opt:
        key, value = kv.split("=")
        pipe.handle.tetri_set_option(key, int(value))
    nC, C = pipe.n_chunks, w.chunk_size

    # inputs: what the QKV projection of each chunk would hand to this path, resident in HBM
    q = torch.zeros((nC, C, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    k = torch.zeros((nC, C, w.num_kv_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    v = torch.zeros_like(k)
    out = torch.zeros_like(q)
    host_reqs = {}
    for c in range(nC):
        at = 0
        for req, start, n in pipe.chunk_segments(c):
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

    flops = [pipe.flops(c) for c in range(nC)]
    total_flops = float(sum(flops))

    # ---- settle: a fresh process shows one stall of tens of milliseconds a few hundred steps in
    # (clocks / runtime start-up); run past it, untimed, before the W warmup steps
    t_settle = time.perf_counter()
    n_settle = 0
    while time.perf_counter() - t_settle < args.settle:
        for _ in range(20):
            pipe.step()
        torch.cuda.synchronize()
        n_settle += 20
    # ---- warmup, then exactly K timed steps bracketed by synchronisations
    for _ in range(args.warmup):
        pipe.step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        pipe.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-kernel durations: HIP events (on the launch stream) around groups of R back-to-back
    # launches of one chunk's kernel, replayed from a HIP graph so that the host launch path does not
    # sit between the kernels; duration = group time / R
    R, reps = 10, max(3, min(20, args.steps // 10))
    stream = torch.cuda.current_stream()

    spread = []                                     # (p10, p90) of every group_time call, in call order

    def group_time(launch):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(R):
                launch()
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
    pipe.host_plan(0)
    pipe.meta_dev.copy_(pipe.stage[0])
    torch.cuda.synchronize()
    main_launch = pipe.launch_attn if args.two_launches else pipe.launch_fused
    attn_ms = np.array([group_time(lambda c=c: main_launch(c)) for c in range(min(nC, 64))])
    app_ms = np.array([group_time(lambda c=c: pipe.launch_append(c)) for c in range(min(nC, 8))])
    n_meas = len(attn_ms)
    attn_avg_ms = float(attn_ms.mean())                 # average duration of one attention launch
    attn_flops_per_launch = float(sum(flops[:n_meas])) / n_meas
    achieved_tflops = attn_flops_per_launch / (attn_avg_ms * 1e-3) / 1e12
    app_bytes = float(np.mean([pipe.append_bytes(c) for c in range(len(app_ms))]))
    app_avg_ms = float(app_ms.mean())
    attn_med, app_med = attn_ms, app_ms

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
            "segments_per_chunk": {"mean": round(float(np.mean([len(pipe.chunk_segments(c)) for c in range(nC)])), 2),
                                   "max": int(max(len(pipe.chunk_segments(c)) for c in range(nC)))},
            "step": "pack + metadata + upload + per chunk " +
                    ("(attention launch, kv append launch)" if args.two_launches else "one fused attention+append launch"),
        },
        "roofline": {
            "bound": "mfma", "kernel": "attn_tile_kernel" + ("" if args.two_launches else " (with fused kv append)"),
            "achieved": round(achieved_tflops, 3), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved_tflops / PEAK_BF16_MFMA_TFLOPS, 5),
            "avg_launch_ms": round(attn_avg_ms, 5), "flops_per_launch": attn_flops_per_launch,
            "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, "two" if args.two_launches else "fused")),
            "algorithmic_bytes_per_launch": float(np.mean([pipe.attn_bytes(c) + (0 if args.two_launches else
                                                           pipe.append_bytes(c)) for c in range(n_meas)])),
        },
        "per_chunk": {
            "attn_ms_median": [round(float(x), 5) for x in attn_med],
            "attn_ms_p10": [round(spread[i][0], 5) for i in range(len(attn_med))],
            "attn_ms_p90": [round(spread[i][1], 5) for i in range(len(attn_med))],
            "attn_tflops": [round(flops[c] / (float(attn_med[c]) * 1e-3) / 1e12, 2) for c in range(len(attn_med))],
            "append_ms_median": [round(float(x), 5) for x in app_med],
        },
        "append": {"kernel": "kv_append_kernel (stand-alone launch)", "avg_launch_ms": round(app_avg_ms, 5),
                   "achieved_GBs": round(app_bytes / (app_avg_ms * 1e-3) / 1e9, 1), "peak_GBs": PEAK_HBM_GBS,
                   "frac": round(app_bytes / (app_avg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
    }

    # ---- cold cache: the same step rotated over independent copies of every buffer (inputs, output, page pool), so
    # that more than twice the 256 MB last-level cache is touched before a buffer comes round again.  In a model
    # the chunk's own rows are warm (the projection just wrote them) and the cached context is cold; `value` above
    # has everything warm, this figure everything cold.
    per_set = (q.numel() + k.numel() + v.numel() + out.numel()) * 2 + sum(w.prompt_lens) * 2 * w.num_kv_heads * w.head_dim * 2
    n_sets = int(min(16, max(4, -(-(600 << 20) // per_set) + 1)))
    if n_sets * (pool.numel() * 2 + per_set) <= (64 << 30) and not args.export:
        sets = [pipe]
        keep = []
        for _ in range(n_sets - 1):
            pp = PrefillPipeline(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                                 w.num_pages, tables, w.scale, device=dev, page_size=w.page_size,
                                 use_graph=(args.mode == "graph"), fused=not args.two_launches)
            if args.variant is not None:
                pp.handle.tetri_set_option("attn_variant", args.variant)
            for kv in args.opt:
                key, value = kv.split("=")
                pp.handle.tetri_set_option(key, int(value))
            bufs = (q.clone(), k.clone(), v.clone(), pool.clone(), torch.zeros_like(out))
            pp.bind(*bufs)
            keep.append(bufs)
            sets.append(pp)
        cold_steps = max(n_sets * 4, min(args.steps, 200) // n_sets * n_sets)
        for i in range(2 * n_sets):
            sets[i % n_sets].step()
        torch.cuda.synchronize()
        tc0 = time.perf_counter()
        for i in range(cold_steps):
            sets[i % n_sets].step()
        torch.cuda.synchronize()
        cold_ms = (time.perf_counter() - tc0) * 1e3 / cold_steps
        result["cold_cache"] = {"value": round(total_flops / (cold_ms * 1e-3) / 1e12, 3), "unit": "TFLOP/s",
                                "ms_per_step": round(cold_ms, 5), "steps": cold_steps, "buffer_sets": n_sets,
                                "bytes_touched_between_repeats": int(per_set * (n_sets - 1))}
        del sets, keep

    # ---- the step after the hot path: request-level KV export of the whole batch and its import on a
    # receiver (Sec. 3.3.4), timed like the kernels above; moved bytes = payload read + payload written
    n_req = len(w.prompt_lens)
    total_tokens = int(sum(w.prompt_lens))
    payload = 2 * w.num_kv_heads * w.head_dim * total_tokens * 2
    if 0 < payload <= (8 << 30):
        d_bt = torch.from_numpy(np.ascontiguousarray(pipe.req_bt)).to(dev)
        d_cu = torch.from_numpy(np.concatenate([[0], np.cumsum(w.prompt_lens)]).astype(np.int32)).to(dev)
        xbuf = torch.zeros(payload // 2, dtype=torch.bfloat16, device=dev)
        exp_ms = group_time(lambda: pipe.handle.tetri_kv_export(pool, d_bt, d_cu, None, n_req, total_tokens, xbuf))
        imp_ms = group_time(lambda: pipe.handle.tetri_kv_import(xbuf, d_bt, d_cu, None, n_req, total_tokens, pool))
        result["kv_transfer"] = {
            "kernel": "kv_transfer_kernel (request-level, %d request(s), %d tokens)" % (n_req, total_tokens),
            "payload_bytes": payload, "bound": "hbm", "peak_GBs": PEAK_HBM_GBS,
            "export_ms": round(exp_ms, 5), "export_GBs": round(2 * payload / (exp_ms * 1e-3) / 1e9, 1),
            "export_frac": round(2 * payload / (exp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
            "import_ms": round(imp_ms, 5), "import_GBs": round(2 * payload / (imp_ms * 1e-3) / 1e9, 1),
            "import_frac": round(2 * payload / (imp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
        }
        del xbuf

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
        dec_ms = group_time(lambda: dh.tetri_decode_attn(dq, dk, dv, dpool, dbt, dcl, dB, dctx, w.scale, dout))
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
        dec8_ms = group_time(lambda: dh.tetri_decode_attn_fp8(dq, dk, dv, dcodes, dbt, dcl, dB, dctx, w.scale,
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
        try:
            import ctypes
            omp = ctypes.CDLL("libgomp.so.1")
            threads = int(omp.omp_get_max_threads())
        except OSError:
            pass
        # bounded sample: whole chunks of the same workload until about 10 s of CPU work
        plan = opacker.pack_chunks(w.prompt_lens, w.order, C)
        opool = np.zeros((w.num_pages if w.num_pages <= 4096 else 1, 2, w.num_kv_heads, w.page_size, w.head_dim),
                         dtype=np.float32)
        sample_flops, cpu_s, n_done, worst = 0.0, 0.0, 0, 0.0
        out_host = out.float().cpu().numpy()
        if w.num_pages <= 4096:
            qh, kh, vh = q.float().cpu().numpy(), k.float().cpu().numpy(), v.float().cpu().numpy()
            max_blocks = max(len(t) for t in tables)
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
            except (NameError, AttributeError):
                pass
        else:
            result["cpu_baseline"] = None
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
