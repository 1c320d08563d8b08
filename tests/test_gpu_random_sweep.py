"""Seeded random sweep of small workloads through every GPU entry point against the oracles.

Shapes are drawn, not hand-picked: prompt lengths from 1 to a few hundred (so that tiles, pages and chunks
are cut at arbitrary places), ChunkSize from 8 to 256, head counts with group sizes 1..8, both head
dimensions, scales of either sign.  Every case checks the prefill outputs (tolerances of the benchmark spec),
the KV pool bit for bit, a request-level export bit for bit and one decode iteration.
"""
import numpy as np
import pytest
import torch

from oracle import decode as odecode, kv_transfer
from paper_2401_11181_amd import synth, tetri
import gpu_common as gc

pytestmark = pytest.mark.gpu
DEV = gc.DEV


def draw(seed):
    rng = np.random.default_rng([2024, seed])
    d = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 3, 5]))
    g = int(rng.choice([1, 1, 2, 3, 4, 8]))
    n_req = int(rng.integers(1, 7))
    kind = rng.integers(0, 3)
    if kind == 0:
        lens = [int(x) for x in rng.integers(1, 40, size=n_req)]
    elif kind == 1:
        lens = [int(x) for x in rng.integers(1, 400, size=n_req)]
    else:
        lens = [int(min(400, max(1, np.rint(np.exp(rng.normal(4.0, 1.0)))))) for _ in range(n_req)]
    chunk = int(rng.choice([8, 16, 24, 32, 64, 100, 128, 256]))
    scale = float(rng.choice([1.0, -1.0])) * float(rng.uniform(0.2, 1.5)) / np.sqrt(d)
    order = [int(x) for x in rng.permutation(n_req)]
    return synth.small("sweep%d" % seed, lens, chunk, hkv * g, hkv, d, seed=5000 + seed, scale=scale, order=order)


@pytest.mark.parametrize("seed", range(24))
def test_random_workload(oracle, seed):
    w = draw(seed)
    print(w.prompt_lens, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim, round(w.scale, 4), flush=True)
    qs, ks, vs, tables = gc.workload_tensors(w)
    variant = [0, 10, 11, 13, 14, 15, 16, 17][seed % 8]
    outs, pool, sess, _ = gc.gpu_prefill(w, qs, ks, vs, tables, fused=(seed % 2 == 0), variant=variant)
    ref, _, _ = gc.oracle_prefill(oracle, w, qs, ks, vs, tables)
    gc.compare(outs, ref, label=w.name)
    bits = gc.oracle_pool_bits(oracle, w, ks, vs, tables)
    assert np.array_equal(pool.cpu().view(torch.int16).numpy().view(np.uint16), bits)
    # request-level export of the cache just built
    B = len(w.prompt_lens)
    mb = max(len(t) for t in tables)
    bt = np.zeros((B, mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt[r, :len(t)] = t
    cu = np.concatenate([[0], np.cumsum(w.prompt_lens)]).astype(np.int32)
    h = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, 64, w.num_pages, mb, 8)
    d_bt = torch.from_numpy(bt).to(DEV)
    buf = torch.zeros(2 * w.num_kv_heads * w.head_dim * int(cu[-1]), dtype=torch.int16, device=DEV)
    h.tetri_kv_export(pool, d_bt, torch.from_numpy(cu).to(DEV), None, B, int(cu[-1]), buf)
    # one decode iteration: every request's last token as the new one
    ctx = np.array([n - 1 for n in w.prompt_lens], dtype=np.int32)
    q = torch.stack([qs[r][ctx[r]] for r in range(B)])
    k = torch.stack([ks[r][ctx[r]] for r in range(B)])
    v = torch.stack([vs[r][ctx[r]] for r in range(B)])
    out = torch.zeros(q.shape, dtype=torch.bfloat16, device=DEV)
    if seed % 3 == 0:
        h.tetri_set_option("decode_parts", 1 + seed % 5)
    h.tetri_decode_attn(q.to(DEV), k.to(DEV), v.to(DEV), pool, d_bt, torch.from_numpy(ctx).to(DEV), B, int(ctx.max()),
                        w.scale, out)
    torch.cuda.synchronize()
    assert np.array_equal(buf.cpu().numpy().view(np.uint16), kv_transfer.kv_export(bits, bt, cu))
    dref = odecode.decode_attn(q.float().numpy(), k.float().numpy(), v.float().numpy(), pool.float().cpu().numpy(),
                               bt, ctx, w.scale)
    gc.compare([out.cpu()], [dref], label=w.name + "-decode")
    h.close()
