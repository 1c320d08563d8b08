"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times:
ONE fused launch per chunk (tetri_chunk_prefill_attn_append), kernel and workgroup shape chosen by the library.

packed: every output element and the whole pool.  heavy and gqa: sampled (row, head) outputs the oracle
computes one by one from the same seeded inputs, plus closed-form checks of the pool (each request's pages hold
exactly its K and V, every other page keeps the sentinel).  The samples are aimed: first and last row of every
segment of a checked chunk, the rows on both sides of every 32-row block edge near a segment boundary and of a few
others, random rows elsewhere; for gqa additionally every row of four query heads in the chunks of the two
shortest prompts and of the longest one.
"""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import packer as opacker
from paper_2401_11181_amd import synth
from paper_2401_11181_amd.prefill import ChunkedPrefill
import gpu_common as gc

pytestmark = pytest.mark.gpu
DEV = gc.DEV


def test_packed_config_full(oracle):
    """64 chunks of 512 rows packed from 286 lognormal prompts: all outputs, whole pool."""
    w = synth.workload("packed")
    qs, ks, vs, tables = gc.workload_tensors(w)
    outs, pool, sess, _ = gc.gpu_prefill(w, qs, ks, vs, tables, fused=True)
    assert sess.n_chunks == 64
    ref, _, _ = gc.oracle_prefill(oracle, w, qs, ks, vs, tables)
    print(gc.compare(outs, ref, label="packed"))
    bits = gc.oracle_pool_bits(oracle, w, ks, vs, tables)
    assert np.array_equal(pool.cpu().view(torch.int16).numpy().view(np.uint16), bits)
    # the sharp distribution on the same plan
    ws = synth.sharp(w)
    ws.seed = 2003
    qs, ks, vs, _ = gc.workload_tensors(ws)
    outs, _, _, _ = gc.gpu_prefill(ws, qs, ks, vs, tables, fused=True)
    ref, _, _ = gc.oracle_prefill(oracle, ws, qs, ks, vs, tables)
    print(gc.compare(outs, ref, label="packed-sharp"))


def aimed_rows(segs, n_samples, rng):
    """Rows of a chunk worth checking: both ends of every segment, both sides of the 32-row block edges next to
    them and of a few random ones, then random rows up to n_samples."""
    rows, at = [], 0
    for _req, _start, n in segs:
        rows += [at, at + n - 1]
        for e in (32, 64, n // 32 * 32, n // 2 // 32 * 32):
            rows += [at + min(max(e - 1, 0), n - 1), at + min(e, n - 1)]
        at += n
    n_real = at
    rows += [int(x) // 32 * 32 - int(x) % 2 for x in rng.integers(32, max(n_real, 33), size=4) if x < n_real]
    rows = [r for r in dict.fromkeys(rows) if 0 <= r < n_real]
    if len(rows) < n_samples:
        rows += [int(x) for x in rng.integers(0, n_real, size=n_samples - len(rows))]
    return np.asarray(rows, dtype=np.int32)


def run_sampled(oracle, w, check_chunks, n_samples, seed, dense_chunks=(), dense_heads=(), options=None):
    """Run the whole workload on the GPU, one fused launch per chunk as bench.py does; check sampled outputs
    of the given chunks (every row of `dense_heads` in `dense_chunks`) and the pool."""
    qs, ks, vs, tables = gc.workload_tensors(w)
    sess = ChunkedPrefill(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                          w.num_pages, tables, device=DEV, page_size=w.page_size)
    for key, value in (options or {}).items():
        sess.handle.tetri_set_option(key, value)
    plan = opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size)
    assert [sess.chunk_segments(c) for c in range(sess.n_chunks)] == [list(c) for c in plan]
    pool = synth.pool_sentinel((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), device=DEV)
    dq = [t.to(DEV) for t in qs]
    dk = [t.to(DEV) for t in ks]
    dv = [t.to(DEV) for t in vs]
    rng = np.random.default_rng(seed)
    check_chunks = [c % sess.n_chunks for c in check_chunks]
    dense_chunks = [c % sess.n_chunks for c in dense_chunks]
    worst = dict(max_abs=0.0, mean_abs=0.0, rel_l2=0.0)
    for c in range(sess.n_chunks):
        q, k, v = sess.gather_chunk(dq, c), sess.gather_chunk(dk, c), sess.gather_chunk(dv, c)
        out = torch.full((w.chunk_size, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
        sess.attn_append(c, q, k, v, pool, w.scale, out)
        if c not in check_chunks and c not in dense_chunks:
            continue
        sess.validate(c)
        segs = plan[c]
        n_real = sum(n for _, _, n in segs)
        if c in dense_chunks:
            rows = np.repeat(np.arange(n_real, dtype=np.int32), len(dense_heads))
            heads = np.tile(np.asarray(dense_heads, dtype=np.int32), n_real)
        else:
            rows = aimed_rows(segs, n_samples, rng)
            heads = rng.integers(0, w.num_q_heads, size=len(rows)).astype(np.int32)
        ref = gc.oracle_chunk_samples(oracle, w, segs, q.float().cpu().numpy(), k.float().cpu().numpy(),
                                      v.float().cpu().numpy(), ks, vs, rows, heads)
        got = out.float().cpu().numpy()[rows, heads]
        assert not out[n_real:].any()
        err = np.abs(got - ref)
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert np.isfinite(got).all()
        assert err.max() <= 2e-2 and err.mean() <= 2e-3 and rel <= 1e-2, (c, err.max(), err.mean(), rel)
        worst = dict(max_abs=max(worst["max_abs"], err.max()), mean_abs=max(worst["mean_abs"], err.mean()),
                     rel_l2=max(worst["rel_l2"], rel))
    torch.cuda.synchronize()
    # pool closed form: each request's pages hold exactly its K and V in token order ...
    P = w.page_size
    touched = torch.zeros(w.num_pages, dtype=torch.bool, device=DEV)
    for r, n in enumerate(w.prompt_lens):
        pages = torch.from_numpy(tables[r].astype(np.int64)).to(DEV)
        touched[pages] = True
        blk = pool[pages]                                        # [pages, 2, Hkv, P, D]
        for which, src in ((0, dk[r]), (1, dv[r])):
            got = blk[:, which].permute(0, 2, 1, 3).reshape(-1, w.num_kv_heads, w.head_dim)
            assert torch.equal(got[:n].view(torch.int16), src.view(torch.int16)), (r, which)
            if n % P:                                            # the unused tail of the last page
                assert (got[n:].view(torch.int16) == 0x3B5A).all()
    # ... and every other page still holds the sentinel
    assert (pool[~touched].view(torch.int16) == 0x3B5A).all()
    return worst


def test_heavy_config_sampled(oracle):
    """One 16384-token prompt in 32 chunks, pages scattered over a 32768-page pool (10.7 GB)."""
    w = synth.workload("heavy")
    print(run_sampled(oracle, w, check_chunks=[0, 1, 7, 15, 30, 31], n_samples=64, seed=4))


def test_gqa_config_sampled(oracle):
    """8 prompts of 4k..32k tokens, 32 query heads on 8 kv heads, ChunkSize 2048, packed chunks."""
    w = synth.workload("gqa")
    plan = opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size)
    two_segs = [c for c, segs in enumerate(plan) if len(segs) == 2]
    assert two_segs, "the workload has chunks that merge the end of one prompt with the start of the next"
    # every row of four query heads (one per kv-head group of four) in the chunks of the two shortest prompts and
    # the last chunk of the longest one
    by_len = np.argsort(w.prompt_lens, kind="stable")
    dense_reqs = {int(by_len[0]), int(by_len[1])}
    dense = [c for c, segs in enumerate(plan) if any(req in dense_reqs for req, _s, _n in segs)]
    longest = int(by_len[-1])
    dense.append(max(c for c, segs in enumerate(plan) if any(req == longest for req, _s, _n in segs)))
    print("gqa: two-segment chunks", two_segs, "dense chunks", dense, flush=True)
    print(run_sampled(oracle, w, check_chunks=[0, 8, 9, 30, 50, -2, -1] + two_segs, n_samples=48, seed=5,
                      dense_chunks=dense, dense_heads=(1, 10, 19, 28)))


@pytest.mark.parametrize("chunk_size,stream_wgs", [(1024, 0), (1024, 6), (4096, 0)], ids=["1024", "1024-stream6", "4096"])
def test_large_chunk_sizes_sampled(oracle, chunk_size, stream_wgs):
    """One 8192-token prompt on the 13B head shape (40 x 128) with ChunkSize 1024 and 4096: launches with more row
    tiles than compute units, which the library runs with four-wavefront workgroups, one per tile (1.25 and 5 per
    compute unit).  With `stream_wgs` 6 the ChunkSize-1024 launches instead give every head six eight-wavefront
    workgroups that divide the head's stages evenly among them (tiles of many pieces), at full size."""
    base = synth.workload("opt13b")
    w = dataclasses.replace(base, name="opt13b-len8192-chunk%d" % chunk_size, prompt_lens=[8192], order=[0],
                            chunk_size=chunk_size, num_pages=8192 // base.page_size + 64, seed=3000 + chunk_size)
    n_chunks = 8192 // chunk_size
    opts = {"stream_wgs": stream_wgs} if stream_wgs else {}
    print(run_sampled(oracle, w, check_chunks=sorted({0, 1, n_chunks // 2, n_chunks - 1}), n_samples=96, seed=6, options=opts))
