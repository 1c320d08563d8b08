"""GPU-side test plumbing: run a synthetic workload through the C library, chunk by chunk."""
import numpy as np
import torch

from oracle import packer as opacker
from paper_2401_11181_amd import synth
from paper_2401_11181_amd.prefill import ChunkedPrefill

DEV = "cuda:0"


def workload_tensors(w):
    """Per-request bf16 CPU tensors and block tables of a workload."""
    qs, ks, vs = [], [], []
    for r in range(len(w.prompt_lens)):
        q, k, v = synth.request_qkv(w, r)
        qs.append(q), ks.append(k), vs.append(v)
    return qs, ks, vs, synth.place_pages(w)


def set_variant(sess, variant):
    """Kernel variant of a session (see gpu_prefill)."""
    sess.handle.tetri_set_option("attn_variant", variant if variant < 10 else (1 if variant in (11, 15) else 2))
    if variant in (10, 11, 13):
        sess.handle.tetri_set_option("split_min_stages", 2)
        sess.handle.tetri_set_option("split_bias_stages", 0)
    if variant == 13:
        sess.handle.tetri_set_option("split_share_q8", 128)
    if variant == 12:
        sess.handle.tetri_set_option("split_keys", 0)
    if variant in (14, 15, 16, 17):
        sess.handle.tetri_set_option("stream_wgs", {14: 5, 15: 5, 16: 2, 17: 200}[variant])


def gpu_prefill(w, qs, ks, vs, tables, append_first=False, pad_fill=None, keep_chunks=False, variant=0, fused=False):
    """Run the whole batch on the GPU.  Returns (outs per request [n,Hq,D] bf16 cpu, pool tensor, session)."""
    sess = ChunkedPrefill(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                          w.num_pages, tables, device=DEV, page_size=w.page_size)
    # variants 0 / 1 / 2: the library's choice / 4-wavefront / 8-wavefront workgroups, each with the library's
    # choice of how the work is handed out; 10 / 11: 8- / 4-wavefront workgroups, tail mode with every key range of
    # two or more stages handing its last third to a helper workgroup (the library itself only does so for long
    # ones); 13: half of it (helpers settle their first tile late); 12: one workgroup per row tile, nothing
    # divided; 14 / 15: stream mode with 5 workgroups per head group, 8 / 4 wavefronts; 16: with 2 (every workgroup
    # runs many jobs); 17: with 200 (a stage per workgroup: as many pieces per tile as it has stages)
    set_variant(sess, variant)
    pool = synth.pool_sentinel((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), device=DEV)
    dq = [t.to(DEV) for t in qs]
    dk = [t.to(DEV) for t in ks]
    dv = [t.to(DEV) for t in vs]
    outs = [torch.zeros_like(t) for t in qs]
    chunk_outs = []
    for c in range(sess.n_chunks):
        sess.validate(c)
        q, k, v = sess.gather_chunk(dq, c), sess.gather_chunk(dk, c), sess.gather_chunk(dv, c)
        segs = sess.chunk_segments(c)
        n_real = sum(n for _, _, n in segs)
        if pad_fill is not None and n_real < w.chunk_size:
            q[n_real:], k[n_real:], v[n_real:] = pad_fill, pad_fill, pad_fill
        out = torch.full((w.chunk_size, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
        if fused:
            sess.attn_append(c, q, k, v, pool, w.scale, out)
        elif append_first:
            sess.append(c, k, v, pool)
            sess.attn(c, q, k, v, pool, w.scale, out)
        else:
            sess.attn(c, q, k, v, pool, w.scale, out)
            sess.append(c, k, v, pool)
        torch.cuda.synchronize()
        o = out.cpu()
        at = 0
        for req, start, n in segs:
            outs[req][start:start + n] = o[at:at + n]
            at += n
        assert not o[n_real:].any(), "padding rows of out must be +0"
        assert (o[n_real:].view(torch.int16) == 0).all()
        if keep_chunks:
            chunk_outs.append(o)
    return outs, pool, sess, chunk_outs


def oracle_prefill(oracle, w, qs, ks, vs, tables):
    """The same batch through the CPU oracle (float32 data).  Returns (outs, float32 pool)."""
    pool = np.zeros((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), dtype=np.float32)
    outs, plan = oracle.prefill([t.float().numpy() for t in qs], [t.float().numpy() for t in ks],
                                [t.float().numpy() for t in vs], w.order, w.chunk_size, pool, tables, w.scale)
    return outs, pool, plan


def oracle_pool_bits(oracle, w, ks, vs, tables):
    """The KV pool as bf16 bit patterns after appending every chunk with the oracle."""
    sent = synth.pool_sentinel((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), dtype=torch.int16)
    pool = sent.numpy().view(np.uint16).copy()
    kb = [t.view(torch.int16).numpy().view(np.uint16) for t in ks]
    vb = [t.view(torch.int16).numpy().view(np.uint16) for t in vs]
    max_blocks = max(len(t) for t in tables)
    for segs in opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size):
        cu, ctx = opacker.chunk_arrays(segs)
        bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
        for i, (req, _s, _n) in enumerate(segs):
            bt[i, :len(tables[req])] = tables[req]
        oracle.kv_append(oracle.gather_chunk(kb, segs, w.chunk_size), oracle.gather_chunk(vb, segs, w.chunk_size),
                         pool, bt, cu, ctx)
    return pool


def compare(gpu_outs, ref_outs, max_abs=2e-2, mean_abs=2e-3, rel_l2=1e-2, label=""):
    """spec tolerances: max-abs 2e-2, mean-abs 2e-3 (bf16 inputs, fp32 oracle) + relative L2."""
    g = np.concatenate([t.float().numpy().reshape(-1) for t in gpu_outs]).astype(np.float64)
    r = np.concatenate([np.asarray(t).reshape(-1) for t in ref_outs]).astype(np.float64)
    assert np.isfinite(g).all(), label + ": non-finite GPU output"
    err = np.abs(g - r)
    rel = np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-30)
    stats = dict(max_abs=err.max(), mean_abs=err.mean(), rel_l2=rel)
    assert err.max() <= max_abs and err.mean() <= mean_abs and rel <= rel_l2, (label, stats)
    return stats


def oracle_chunk_samples(oracle, w, segs, q_chunk, k_chunk, v_chunk, ks, vs, rows, heads):
    """Oracle outputs of sampled (row, head) pairs of one chunk of a large workload.

    The cached context of the chunk's segments is rebuilt in a compact float32 pool with the
    oracle's own append (physical placement does not matter: pinned by the paging invariant), so
    that the full-size pool never has to exist on the host.  q/k/v_chunk: float32 [C,H,D] rows of the
    chunk; ks/vs: per-request bf16 tensors (only the chunk's requests are touched).
    """
    P, Hkv, D = w.page_size, w.num_kv_heads, w.head_dim
    pages_per_seg = [-(-(start + n) // P) for _req, start, n in segs]
    pool = np.zeros((max(1, sum(pages_per_seg)), 2, Hkv, P, D), dtype=np.float32)
    max_blocks = max(pages_per_seg)
    bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
    at = 0
    for i, (req, start, n) in enumerate(segs):
        bt[i, :pages_per_seg[i]] = np.arange(at, at + pages_per_seg[i])
        at += pages_per_seg[i]
        if start > 0:
            kc = ks[req][:start].float().numpy()
            vc = vs[req][:start].float().numpy()
            oracle.kv_append(kc, vc, pool, bt[i:i + 1], [0, start], [0])
    cu, ctx = opacker.chunk_arrays(segs)
    return oracle.chunk_prefill_attn_samples(q_chunk, k_chunk, v_chunk, pool, bt, cu, ctx, w.scale, rows, heads)


NAN_CODE = 0x7F     # the FP8 pattern that is not a number: fills unused slots of pools of codes, so that a stray read shows


def gpu_prefill_fp8(w, qs, ks, vs, tables, k_scale, v_scale, variant=0, pad_fill=None):
    """The whole batch on the GPU over a cache of FP8 codes: every chunk attends to the codes cached so far and
    its own rows, and caches the codes of its rows (one fused launch per chunk).  Returns (outs per request, pool of
    codes [uint8 tensor], session)."""
    sess = ChunkedPrefill(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                          w.num_pages, tables, device=DEV, page_size=w.page_size)
    set_variant(sess, variant)
    pool = torch.full((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), NAN_CODE, dtype=torch.uint8, device=DEV)
    dq, dk, dv = [t.to(DEV) for t in qs], [t.to(DEV) for t in ks], [t.to(DEV) for t in vs]
    outs = [torch.zeros_like(t) for t in qs]
    for c in range(sess.n_chunks):
        q, k, v = sess.gather_chunk(dq, c), sess.gather_chunk(dk, c), sess.gather_chunk(dv, c)
        segs = sess.chunk_segments(c)
        n_real = sum(n for _, _, n in segs)
        if pad_fill is not None and n_real < w.chunk_size:
            q[n_real:], k[n_real:], v[n_real:] = pad_fill, pad_fill, pad_fill
        out = torch.full((w.chunk_size, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
        sess.attn_fp8(c, q, k, v, pool, w.scale, k_scale, v_scale, 1, out)
        torch.cuda.synchronize()
        o = out.cpu()
        at = 0
        for req, start, n in segs:
            outs[req][start:start + n] = o[at:at + n]
            at += n
        assert (o[n_real:].view(torch.int16) == 0).all(), "padding rows of out must be +0"
    return outs, pool, sess


def oracle_prefill_fp8(w, qs, ks, vs, tables, k_scale, v_scale):
    """The same batch through the CPU oracle of prefill over a cache of codes.  Returns (outs, pool of codes)."""
    from oracle import prefill_fp8, tetri_oracle
    codes = np.full((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), NAN_CODE, dtype=np.uint8)
    qf, kf, vf = [t.float().numpy() for t in qs], [t.float().numpy() for t in ks], [t.float().numpy() for t in vs]
    outs = [np.zeros(t.shape, dtype=np.float64) for t in qf]
    max_blocks = max(len(t) for t in tables)
    for segs in opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size):
        cu, ctx = opacker.chunk_arrays(segs)
        bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
        for i, (req, _s, _n) in enumerate(segs):
            bt[i, :len(tables[req])] = tables[req]
        q = tetri_oracle.gather_chunk(qf, segs, w.chunk_size)
        k = tetri_oracle.gather_chunk(kf, segs, w.chunk_size)
        v = tetri_oracle.gather_chunk(vf, segs, w.chunk_size)
        o = prefill_fp8.chunk_prefill_attn_fp8(q, k, v, codes, bt, cu, ctx, w.scale, k_scale, v_scale)
        prefill_fp8.prefill_append_fp8(k, v, codes, bt, cu, ctx, k_scale, v_scale)
        for i, (req, start, n) in enumerate(segs):
            outs[req][start:start + n] = o[cu[i]:cu[i] + n]
    return outs, codes
