"""GPU parity of tetri_decode_attn (through the C ABI) against the numpy decode oracle.

Tolerances as for the prefill attention (bf16 inputs, fp32 accumulation): max-abs <= 2e-2, mean-abs <=
2e-3, relative L2 <= 1e-2.  A request of n synthetic tokens is used as a cache of its first n - 1
tokens plus the new token n - 1.
"""
import numpy as np
import pytest
import torch

from oracle import decode as odecode
from paper_2401_11181_amd import synth, tetri
import gpu_common as gc

pytestmark = pytest.mark.gpu
DEV = gc.DEV


def build(w, stale=None):
    """Device and host inputs of one decode iteration of workload w (ctx_b = prompt_lens[b] - 1)."""
    tables = synth.place_pages(w)
    B = len(w.prompt_lens)
    mb = max(max(len(t) for t in tables), 1)
    bt = np.zeros((B, mb), dtype=np.int32)
    pool = synth.pool_sentinel((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim))
    if stale is not None:
        pool.fill_(stale)
    q, k, v = [], [], []
    P = w.page_size
    for r in range(B):
        bt[r, :len(tables[r])] = tables[r]
        rq, rk, rv = synth.request_qkv(w, r)
        n = w.prompt_lens[r]
        for j in range(n - 1):
            pool[tables[r][j // P], 0, :, j % P, :] = rk[j]
            pool[tables[r][j // P], 1, :, j % P, :] = rv[j]
        q.append(rq[n - 1]), k.append(rk[n - 1]), v.append(rv[n - 1])
    ctx = np.array([n - 1 for n in w.prompt_lens], dtype=np.int32)
    return torch.stack(q), torch.stack(k), torch.stack(v), pool, bt, ctx


def run_gpu(w, q, k, v, pool, bt, ctx, parts=0, max_ctx=None):
    h = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, 64, w.num_pages, bt.shape[1], 8)
    if parts:
        h.tetri_set_option("decode_parts", parts)
    out = torch.full(q.shape, 7.0, dtype=torch.bfloat16, device=DEV)
    d_pool = pool.to(DEV)
    before = d_pool.clone()
    h.tetri_decode_attn(q.to(DEV), k.to(DEV), v.to(DEV), d_pool, torch.from_numpy(bt).to(DEV),
                        torch.from_numpy(ctx).to(DEV), len(ctx), int(ctx.max()) if max_ctx is None else max_ctx,
                        w.scale, out)
    torch.cuda.synchronize()
    assert torch.equal(d_pool.view(torch.int16), before.view(torch.int16)), "decode must not write the pool"
    h.close()
    return out.cpu()


def reference(w, q, k, v, pool, bt, ctx):
    clean = torch.nan_to_num(pool.float(), nan=0.0, posinf=0.0, neginf=0.0).numpy()   # slots >= ctx are never used
    return odecode.decode_attn(q.float().numpy(), k.float().numpy(), v.float().numpy(), clean, bt, ctx, w.scale)


CASES = {
    # name: (lengths n = ctx + 1, Hq, Hkv, D)
    "ragged-mha": ([1, 2, 16, 17, 32, 33, 34, 128, 129, 130, 500], 2, 2, 128),
    "gqa2": ([150, 40, 1], 4, 2, 128),
    "gqa4": ([150, 40, 257], 8, 2, 128),
    "gqa8": ([300, 31], 8, 1, 128),
    "gqa3-d64": ([150, 40, 65], 6, 2, 64),
    "mha-d64": ([97, 1, 64, 33], 3, 3, 64),
    "gqa32": ([200, 77], 32, 1, 128),
}


@pytest.mark.parametrize("parts", [0, 1, 3], ids=["auto", "whole", "three-parts"])
@pytest.mark.parametrize("name", sorted(CASES))
def test_decode_shapes(name, parts):
    lens, hq, hkv, d = CASES[name]
    w = synth.small("dec-" + name, lens, 64, hq, hkv, d, seed=300 + sorted(CASES).index(name))
    args = build(w)
    out = run_gpu(w, *args, parts=parts)
    print(name, gc.compare([out], [reference(w, *args)], label=name))


def test_many_parts_more_than_steps():
    """More parts than some requests have 32-key steps: the empty parts are skipped on both sides."""
    w = synth.small("dec-parts", [1, 40, 700, 33], 64, 4, 2, 128, seed=320)
    args = build(w)
    out = run_gpu(w, *args, parts=9)
    print(gc.compare([out], [reference(w, *args)], label="parts9"))


def test_sharp_scores_and_scales():
    for scale in (0.0, -0.3, 1.5):
        w = synth.small("dec-scale", [90, 45, 260], 64, 4, 2, 64, seed=321, scale=scale)
        args = build(w)
        print(scale, gc.compare([run_gpu(w, *args, parts=2)], [reference(w, *args)], label="scale"))


def test_spiky_key_far_back():
    """One cached key scores about +20 above the rest: the running maximum moves once, early."""
    w = synth.small("dec-spiky", [400], 64, 2, 2, 128, seed=322)
    q, k, v, pool, bt, ctx = build(w)
    tables = synth.place_pages(w)
    j = 37
    pool[tables[0][j // 16], 0, :, j % 16, :] = 0.0
    pool[tables[0][j // 16], 0, :, j % 16, 0] = 16.0
    q[:, :, 0] = 20.0 * (128 ** 0.5) / 16.0
    out = run_gpu(w, q, k, v, pool, bt, ctx)
    print(gc.compare([out], [reference(w, q, k, v, pool, bt, ctx)], label="spiky"))


@pytest.mark.parametrize("stale", [float("nan"), 3.0e4])
def test_stale_page_contents_are_inert(stale):
    """Slots at and past ctx hold NaN / huge values: same bits as with the ordinary sentinel."""
    w = synth.small("dec-stale", [100, 37, 16, 17], 64, 4, 2, 128, seed=323)
    a = run_gpu(w, *build(w))
    b = run_gpu(w, *build(w, stale=stale))
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_deterministic_and_independent_of_the_hint():
    w = synth.small("dec-det", [300, 120, 55], 64, 8, 2, 128, seed=324)
    args = build(w)
    a = run_gpu(w, *args, parts=4)
    b = run_gpu(w, *args, parts=4)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    # the hint only changes how the keys are split: same function, same tolerance
    c = run_gpu(w, *args, max_ctx=args[4].shape[1] * 16)
    print(gc.compare([c], [reference(w, *args)], label="hint"))


def test_agrees_with_the_prefill_kernel_on_one_token_segments():
    """tetri_chunk_prefill_attn on a chunk of one-token segments computes the same function."""
    w = synth.small("dec-vs-prefill", [150, 40, 7, 33], 64, 4, 2, 128, seed=325)
    q, k, v, pool, bt, ctx = build(w)
    out = run_gpu(w, q, k, v, pool, bt, ctx)
    B = len(ctx)
    h = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, B, w.num_pages, bt.shape[1], B)
    ref = torch.zeros(q.shape, dtype=torch.bfloat16, device=DEV)
    h.tetri_chunk_prefill_attn(q.to(DEV), k.to(DEV), v.to(DEV), pool.to(DEV), torch.from_numpy(bt).to(DEV),
                               torch.arange(B + 1, dtype=torch.int32, device=DEV), torch.from_numpy(ctx).to(DEV),
                               B, w.scale, ref)
    torch.cuda.synchronize()
    h.close()
    assert (out.float() - ref.cpu().float()).abs().max() <= 2e-2


def test_argument_errors():
    w = synth.small("dec-err", [20, 5], 64, 4, 2, 128, seed=326)
    q, k, v, pool, bt, ctx = build(w)
    h = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, 64, w.num_pages, bt.shape[1], 8)
    dq, dk, dv, dp = q.to(DEV), k.to(DEV), v.to(DEV), pool.to(DEV)
    dbt, dctx = torch.from_numpy(bt).to(DEV), torch.from_numpy(ctx).to(DEV)
    out = torch.zeros_like(dq)
    ok = lambda **kw: dict(dict(q=dq, k_new=dk, v_new=dv, kv_pages=dp, block_table=dbt, ctx_lens=dctx, num_reqs=2,
                                max_ctx_len=19, scale=w.scale, out=out), **kw)
    for bad in (ok(q=None), ok(k_new=None), ok(v_new=None), ok(kv_pages=None), ok(block_table=None), ok(ctx_lens=None),
                ok(out=None), ok(num_reqs=0), ok(max_ctx_len=-1), ok(max_ctx_len=bt.shape[1] * 16 + 1),
                ok(scale=float("nan")), ok(q=dq.view(-1)[1:])):
        with pytest.raises(tetri.TetriError) as e:
            h.tetri_decode_attn(**bad)
        assert e.value.status == tetri.TETRI_ERR_INVALID_ARG
    h.tetri_decode_attn(**ok())
    torch.cuda.synchronize()
    h.close()


def test_opt13b_heads_batch():
    """OPT-13B head shape (40 x 128, MHA), 12 requests with contexts up to 2048, every output element."""
    rng = np.random.default_rng(327)
    lens = [int(x) for x in rng.integers(1, 2049, size=10)] + [2048, 2049]
    w = synth.small("dec-opt13b", lens, 512, 40, 40, 128, seed=328, std=1.0 / np.sqrt(128.0))
    args = build(w)
    out = run_gpu(w, *args)
    print(gc.compare([out], [reference(w, *args)], label="opt13b-decode"))
    sharp = synth.sharp(w)
    args = build(sharp)
    print(gc.compare([run_gpu(sharp, *args)], [reference(sharp, *args)], label="opt13b-decode-sharp"))


@pytest.mark.parametrize("name,parts", [("ragged-mha", 0), ("gqa4", 3), ("gqa3-d64", 0), ("mha-d64", 2), ("gqa32", 1)])
def test_fused_decode_append_equals_two_calls(name, parts):
    """tetri_decode_attn_append == tetri_decode_attn then tetri_kv_append (cu = 0..B), bit for bit, and the
    pool equals the numpy placement of the new tokens."""
    lens, hq, hkv, d = CASES[name]
    w = synth.small("decf-" + name, lens, 64, hq, hkv, d, seed=340)
    q, k, v, pool, bt, ctx = build(w)
    B = len(ctx)
    h = tetri.Tetri(hq, hkv, d, max(B, 16), w.num_pages, bt.shape[1], max(B, 8))
    if parts:
        h.tetri_set_option("decode_parts", parts)
    dq, dk, dv = q.to(DEV), k.to(DEV), v.to(DEV)
    dbt, dctx = torch.from_numpy(bt).to(DEV), torch.from_numpy(ctx).to(DEV)
    pool_a, pool_b = pool.to(DEV), pool.to(DEV)
    out_a = torch.zeros_like(dq)
    out_b = torch.zeros_like(dq)
    h.tetri_decode_attn(dq, dk, dv, pool_a, dbt, dctx, B, int(ctx.max()), w.scale, out_a)
    kpad = torch.zeros((max(B, 16), hkv, d), dtype=torch.bfloat16, device=DEV)
    vpad = torch.zeros_like(kpad)
    kpad[:B], vpad[:B] = dk, dv
    h.tetri_kv_append(kpad, vpad, pool_a, dbt, torch.arange(B + 1, dtype=torch.int32, device=DEV), dctx, B)
    h.tetri_decode_attn_append(dq, dk, dv, pool_b, dbt, dctx, B, int(ctx.max()), w.scale, out_b)
    torch.cuda.synchronize()
    assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))
    assert torch.equal(pool_a.view(torch.int16), pool_b.view(torch.int16))
    want = pool.clone()
    for b in range(B):
        L = int(ctx[b])
        want[bt[b, L // 16], 0, :, L % 16, :] = k[b]
        want[bt[b, L // 16], 1, :, L % 16, :] = v[b]
    assert torch.equal(pool_b.cpu().view(torch.int16), want.view(torch.int16))
    h.close()


def test_decode_loop_extends_the_cache(oracle):
    """Prefill a prompt's first tokens with the chunked-prefill path, then decode the rest token by token
    with the fused call: every decode output equals that row of the one-shot oracle prefill, and the
    final pool equals the oracle's."""
    w = synth.small("dec-loop", [75, 41], 32, 4, 2, 128, seed=341)
    qs, ks, vs, tables = gc.workload_tensors(w)
    ref, _, _ = gc.oracle_prefill(oracle, w, qs, ks, vs, tables)
    n_dec = 9
    short = synth.small("dec-loop", [n - n_dec for n in w.prompt_lens], 32, 4, 2, 128, seed=341)
    short.num_pages = w.num_pages
    cut = lambda ts: [t[:n - n_dec] for t, n in zip(ts, w.prompt_lens)]
    _, pool, _, _ = gc.gpu_prefill(short, cut(qs), cut(ks), cut(vs), tables, fused=True)
    B = len(w.prompt_lens)
    mb = max(len(t) for t in tables)
    bt = np.zeros((B, mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt[r, :len(t)] = t
    h = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, 64, w.num_pages, mb, 8)
    dbt = torch.from_numpy(bt).to(DEV)
    outs = [[] for _ in range(B)]
    for step in range(n_dec):
        pos = [n - n_dec + step for n in w.prompt_lens]
        dq = torch.stack([qs[r][pos[r]] for r in range(B)]).to(DEV)
        dk = torch.stack([ks[r][pos[r]] for r in range(B)]).to(DEV)
        dv = torch.stack([vs[r][pos[r]] for r in range(B)]).to(DEV)
        out = torch.zeros_like(dq)
        h.tetri_decode_attn_append(dq, dk, dv, pool, dbt, torch.tensor(pos, dtype=torch.int32, device=DEV), B,
                                   max(pos), w.scale, out)
        torch.cuda.synchronize()
        for r in range(B):
            outs[r].append(out[r].cpu())
    got = [torch.stack(o) for o in outs]
    want = [ref[r][n - n_dec:] for r, n in enumerate(w.prompt_lens)]
    print(gc.compare(got, want, label="decode-loop"))
    bits = gc.oracle_pool_bits(oracle, w, ks, vs, tables)
    assert np.array_equal(pool.cpu().view(torch.int16).numpy().view(np.uint16), bits)
    h.close()
