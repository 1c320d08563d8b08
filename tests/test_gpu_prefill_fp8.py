"""GPU parity of chunked prefill over a cache of FP8 codes (tetri_chunk_prefill_attn_fp8) against its oracle
(oracle/prefill_fp8.py): outputs to the tolerances of the 16-bit path (the codes both sides read are the same
bytes, so the arithmetic that differs is the same as there), the codes the launch caches bit for bit.
Unused slots of every pool hold the code that is not a number: a stray read of one would show in the output.
"""
import numpy as np
import pytest
import torch

from paper_2401_11181_amd import synth, tetri
from paper_2401_11181_amd.prefill import ChunkedPrefill
from oracle import fp8 as ofp8
from oracle import packer as opacker
from oracle import prefill_fp8 as oprefill
import gpu_common as gc
from test_gpu_parity import CASES, VARIANTS

pytestmark = pytest.mark.gpu
DEV = gc.DEV
K_SCALE, V_SCALE = 0.0137, 0.0171          # values of about N(0, 1) use codes up to about +-300 of +-448


@pytest.fixture(params=VARIANTS, ids=["auto", "wave4", "wave8", "tails", "tails-wave4", "whole", "tails-half", "stream5", "stream5-wave4", "stream2", "stream200"])
def variant(request):
    return request.param


_oracle_runs = {}


def oracle_run(w, qs, ks, vs, tables, k_scale, v_scale):
    """The oracle's result of a case, computed once for all kernel variants."""
    key = (w.name, w.seed, k_scale, v_scale, w.scale)
    if key not in _oracle_runs:
        _oracle_runs[key] = gc.oracle_prefill_fp8(w, qs, ks, vs, tables, k_scale, v_scale)
    return _oracle_runs[key]


def run_case(w, variant, k_scale=K_SCALE, v_scale=V_SCALE):
    qs, ks, vs, tables = gc.workload_tensors(w)
    outs, pool, _sess = gc.gpu_prefill_fp8(w, qs, ks, vs, tables, k_scale, v_scale, variant=variant)
    ref, codes = oracle_run(w, qs, ks, vs, tables, k_scale, v_scale)
    stats = gc.compare(outs, ref, label=w.name)
    assert np.array_equal(pool.cpu().numpy(), codes), w.name + ": the cache of codes differs from the oracle's"
    return stats


@pytest.mark.parametrize("name", sorted(CASES))
def test_shapes(name, variant):
    lens, chunk, hq, hkv, d = CASES[name]
    w = synth.small("fp8-" + name, lens, chunk, hq, hkv, d, seed=300 + sorted(CASES).index(name))
    print(name, run_case(w, variant))


def test_more_than_64_segments_in_a_chunk(variant):
    rng = np.random.default_rng(152)
    lens = [int(x) for x in rng.integers(1, 5, size=150)]
    w = synth.small("fp8-many-segments", lens, 256, 4, 2, 128, seed=152)
    print(run_case(w, variant))


@pytest.mark.parametrize("scales", [(2.0 ** -6, 2.0 ** -5), (0.11, 0.0031), (3.0e-3, 0.4)], ids=["pow2", "coarse-k", "saturating-k"])
def test_scales_of_the_cache(scales, variant):
    """Coarse scales quantise hard (the oracle reads the same codes: the bar stays), small ones saturate at +-448."""
    w = synth.small("fp8-cache-scales", [333, 70], 128, 4, 2, 128, seed=331)
    print(scales, run_case(w, variant, *scales))


@pytest.mark.parametrize("scale", [0.0, -0.2, 1.7])
def test_softmax_scales(scale, variant):
    w = synth.small("fp8-scale", [200, 45], 64, 2, 2, 64, seed=332, scale=scale)
    print(scale, run_case(w, variant))


def test_without_append_the_pool_is_only_read(variant):
    w = synth.small("fp8-read-only", [300, 90], 128, 4, 2, 128, seed=333)
    qs, ks, vs, tables = gc.workload_tensors(w)
    outs, pool, sess = gc.gpu_prefill_fp8(w, qs, ks, vs, tables, K_SCALE, V_SCALE, variant=variant)
    c = sess.n_chunks - 1
    dq, dk, dv = [t.to(DEV) for t in qs], [t.to(DEV) for t in ks], [t.to(DEV) for t in vs]
    q, k, v = sess.gather_chunk(dq, c), sess.gather_chunk(dk, c), sess.gather_chunk(dv, c)
    before = pool.clone()
    a = torch.zeros_like(q)
    b = torch.zeros_like(q)
    sess.attn_fp8(c, q, k, v, pool, w.scale, K_SCALE, V_SCALE, 0, a)
    torch.cuda.synchronize()
    assert torch.equal(pool, before)
    sess.attn_fp8(c, q, k, v, pool, w.scale, K_SCALE, V_SCALE, 1, b)      # rewrites the codes the chain wrote
    torch.cuda.synchronize()
    assert torch.equal(pool, before) and torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("fill", [3.0e4, float("nan")])
def test_padding_rows_are_inert(fill, variant):
    w = synth.small("fp8-pad", [100, 37], 64, 2, 2, 128, seed=334)
    qs, ks, vs, tables = gc.workload_tensors(w)
    ref, pool_ref, _ = gc.gpu_prefill_fp8(w, qs, ks, vs, tables, K_SCALE, V_SCALE, variant=variant)
    out, pool, _ = gc.gpu_prefill_fp8(w, qs, ks, vs, tables, K_SCALE, V_SCALE, variant=variant, pad_fill=fill)
    for x, y in zip(ref, out):
        assert torch.equal(x, y)
    assert torch.equal(pool_ref, pool)


def test_rejects_bad_scales_and_flags():
    w = synth.small("fp8-errors", [40], 64, 2, 2, 128, seed=335)
    qs, ks, vs, tables = gc.workload_tensors(w)
    sess = ChunkedPrefill(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim, w.num_pages, tables, device=DEV)
    q = torch.zeros((64, 2, 128), dtype=torch.bfloat16, device=DEV)
    pool = torch.zeros((w.num_pages, 2, 2, 16, 128), dtype=torch.uint8, device=DEV)
    for ks_, vs_, app in ((0.0, 1.0, 1), (1.0, -2.0, 1), (float("inf"), 1.0, 0), (float("nan"), 1.0, 0), (1.0, 1.0, 2)):
        with pytest.raises(tetri.TetriError) as info:
            sess.attn_fp8(0, q, q, q, pool, 1.0, ks_, vs_, app, q.clone())
        assert info.value.status == tetri.TETRI_ERR_INVALID_ARG


def chunk_over_random_cache(w, c_index, seed, variant=0, options=None):
    """Chunk c_index of workload w over a cache of random codes (about N(0, std^2) after scaling): the launch, with
    append.  Returns what a comparison needs."""
    tables = synth.place_pages(w)
    sess = ChunkedPrefill(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                          w.num_pages, tables, device=DEV, page_size=w.page_size)
    gc.set_variant(sess, variant)
    for key, value in (options or {}).items():
        sess.handle.tetri_set_option(key, value)
    codes = synth.random_kv_codes((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), seed, K_SCALE, V_SCALE, std=w.std)
    segs = sess.chunk_segments(c_index)
    qs, ks, vs = {}, {}, {}
    for req, _start, _n in segs:
        qs[req], ks[req], vs[req] = synth.request_qkv(w, req)
    gather = lambda per: torch.cat([per[req][start:start + n] for req, start, n in segs] +
                                   [torch.zeros((w.chunk_size - sum(n for _, _, n in segs),) + tuple(per[segs[0][0]].shape[1:]), dtype=torch.bfloat16)])
    q, k, v = gather(qs), gather(ks), gather(vs)
    pool = codes.to(DEV)
    out = torch.full((w.chunk_size, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
    sess.attn_fp8(c_index, q.to(DEV), k.to(DEV), v.to(DEV), pool, w.scale, K_SCALE, V_SCALE, 1, out)
    torch.cuda.synchronize()
    cu, ctx = opacker.chunk_arrays(segs)
    max_blocks = max(len(t) for t in tables)
    bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
    for i, (req, _s, _n) in enumerate(segs):
        bt[i, :len(tables[req])] = tables[req]
    return dict(q=q.float().numpy(), k=k.float().numpy(), v=v.float().numpy(), codes=codes.numpy(), bt=bt, cu=cu, ctx=ctx,
                out=out.float().cpu().numpy(), pool=pool.cpu().numpy(), segs=segs)


def check_appended_rows(r, rows):
    """The codes the launch cached for the sampled chunk rows, and nothing else changed in the pool."""
    P = r["pool"].shape[3]
    changed = r["pool"] != r["codes"]
    allowed = np.zeros(r["pool"].shape, dtype=bool)
    for s in range(len(r["ctx"])):
        for t in range(r["cu"][s + 1] - r["cu"][s]):
            pos = r["ctx"][s] + t
            allowed[r["bt"][s][pos // P], :, :, pos % P, :] = True
    assert not (changed & ~allowed).any(), "the launch wrote outside the slots of the chunk's rows"
    for row in rows:
        s = max(x for x in range(len(r["ctx"])) if r["cu"][x] <= row)
        pos = r["ctx"][s] + row - r["cu"][s]
        got = r["pool"][r["bt"][s][pos // P], :, :, pos % P, :]
        assert np.array_equal(got[0], ofp8.quantize(r["k"][row], K_SCALE)), ("K codes of chunk row", row)
        assert np.array_equal(got[1], ofp8.quantize(r["v"][row], V_SCALE)), ("V codes of chunk row", row)


@pytest.mark.parametrize("variant_", [0, 12, 14], ids=["auto", "whole", "stream5"])
def test_opt13b_last_chunk_full_size(variant_):
    """The bench shape (40 x 128 heads, ChunkSize 512), its last chunk over 1536 cached tokens of codes: every output."""
    w = synth.workload("opt13b")
    r = chunk_over_random_cache(w, 3, 401, variant=variant_)
    ref = oprefill.chunk_prefill_attn_fp8(r["q"], r["k"], r["v"], r["codes"], r["bt"], r["cu"], r["ctx"], w.scale, K_SCALE, V_SCALE)
    print(gc.compare([torch.from_numpy(r["out"])], [ref], label="fp8-opt13b"))
    sharp = synth.sharp(w)
    r = chunk_over_random_cache(sharp, 3, 402, variant=variant_)
    ref = oprefill.chunk_prefill_attn_fp8(r["q"], r["k"], r["v"], r["codes"], r["bt"], r["cu"], r["ctx"], sharp.scale, K_SCALE, V_SCALE)
    print(gc.compare([torch.from_numpy(r["out"])], [ref], label="fp8-opt13b-sharp"))
    check_appended_rows(r, [0, 1, 15, 16, 255, 300, 511])


def sampled(w, c_index, seed, n_samples, options=None):
    r = chunk_over_random_cache(w, c_index, seed, options=options)
    rng = np.random.default_rng(seed)
    n_real = int(r["cu"][-1])
    edge = [0, 31, 32, 127, 128, n_real - 1] + [int(x) for x in r["cu"][1:-1]] + [int(x) - 1 for x in r["cu"][1:-1]]
    rows = sorted(set([x for x in edge if 0 <= x < n_real] + [int(x) for x in rng.integers(0, n_real, size=n_samples)]))
    pairs = sorted((int(h), row) for row in rows for h in rng.choice(w.num_q_heads, size=2, replace=False))
    heads, rows2 = [h for h, _ in pairs], [row for _, row in pairs]
    ref = oprefill.chunk_prefill_attn_fp8_samples(r["q"], r["k"], r["v"], r["codes"], r["bt"], r["cu"], r["ctx"], w.scale,
                                                  K_SCALE, V_SCALE, rows2, heads)
    got = np.stack([r["out"][row, h] for h, row in pairs])
    print(w.name, c_index, gc.compare([torch.from_numpy(got)], [ref], label="fp8-sampled-" + w.name))
    assert not r["out"][n_real:].any()
    check_appended_rows(r, rows[:6])


def test_heavy_last_chunk_sampled():
    """One 16 384-token prompt, 40 x 128 heads: the last chunk (15 872 cached tokens), stream mode as the library picks."""
    sampled(synth.sharp(synth.workload("heavy")), 31, 411, 24)


def test_gqa_shape_sampled():
    """32 query / 8 kv heads, ChunkSize 2048 (four-wavefront workgroups with the fused quantising append): a chunk in the
    middle of a long prompt, and the chunk that holds the end of one prompt and the start of the next."""
    w = synth.sharp(synth.workload("gqa"))
    sess_lens = opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size)
    two = [i for i, segs in enumerate(sess_lens) if len(segs) == 2]
    sampled(w, two[0], 412, 16)
    long_mid = max(range(len(sess_lens)), key=lambda i: sess_lens[i][0][1] if len(sess_lens[i]) == 1 else -1)
    sampled(w, long_mid, 413, 16)


def test_packed_shape_sampled():
    """286 short prompts in 64 chunks of 512 at 40 x 128 heads: the chunk with the most segments, and one whose first
    segment continues a prompt that began in the chunk before (cached tokens of one segment, none of the others)."""
    w = synth.sharp(synth.workload("packed"))
    plan = opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size)
    most = max(range(len(plan)), key=lambda i: len(plan[i]))
    cont = max(range(len(plan)), key=lambda i: plan[i][0][1])          # the longest carried-over context
    assert plan[cont][0][1] > 0
    sampled(w, most, 415, 24)
    sampled(w, cont, 416, 24)


@pytest.mark.parametrize("chunk", [1024, 4096])
def test_large_chunk_sizes_sampled(chunk):
    """ChunkSize 1024 / 4096 at 40 x 128 heads over an 8192-token prompt: the second chunk."""
    w = synth.small("fp8-c%d" % chunk, [8192], chunk, 40, 40, 128, seed=420 + chunk // 1024, slack_pages=0)
    sampled(w, 1, 414, 16)
