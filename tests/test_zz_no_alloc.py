"""tetri_decode_attn_static (the entry point that allocates nothing: the parts of split requests live in a static
device array of the library) against tetri_decode_attn, through the C ABI.

Two calls in a row on one handle, the second with a smaller input, so that the array still holds the first call's
parts when the second runs.  With the same "decode_parts" the two entry points must give the same bits; with the
library's own choice of parts (which depends on the scratch size) they must agree within the attention tolerances
(max-abs 2e-2, mean-abs 2e-3, relative L2 1e-2) and both meet the oracle.  Sizes beyond the array are rejected.
"""
import ctypes

import numpy as np
import pytest
import torch

from oracle import decode as odecode
from paper_2401_11181_amd import synth, tetri
import gpu_common as gc

pytestmark = pytest.mark.gpu
DEV = gc.DEV


def make_batch(lens, hq, hkv, d, seed):
    w = synth.small("noalloc", lens, 64, hq, hkv, d, seed=seed)
    tables = synth.place_pages(w)
    B, P = len(lens), w.page_size
    mb = max(len(t) for t in tables)
    bt = np.zeros((B, mb), dtype=np.int32)
    pool = synth.pool_sentinel((w.num_pages, 2, hkv, P, d))
    q, k, v = [], [], []
    for r in range(B):
        bt[r, :len(tables[r])] = tables[r]
        rq, rk, rv = synth.request_qkv(w, r)
        n = lens[r]
        for j in range(n - 1):
            pool[tables[r][j // P], 0, :, j % P, :] = rk[j]
            pool[tables[r][j // P], 1, :, j % P, :] = rv[j]
        q.append(rq[n - 1]), k.append(rk[n - 1]), v.append(rv[n - 1])
    ctx = np.array([n - 1 for n in lens], dtype=np.int32)
    return w, torch.stack(q), torch.stack(k), torch.stack(v), pool, bt, ctx


def test_static_scratch_decode_matches_decode():
    hq, hkv, d = 8, 2, 128
    big = make_batch([700, 333, 1500, 64, 1021], hq, hkv, d, seed=901)
    small = make_batch([90, 411], hq, hkv, d, seed=902)
    pages = max(big[0].num_pages, small[0].num_pages)
    mb = max(big[5].shape[1], small[5].shape[1])
    h = tetri.Tetri(hq, hkv, d, 64, pages, mb, 8)
    for parts in (0, 3, 7):
        h.tetri_set_option("decode_parts", parts)
        for w, q, k, v, pool, bt, ctx in (big, small):         # the second call is the smaller one
            B = len(ctx)
            btp = np.zeros((B, mb), dtype=np.int32)
            btp[:, :bt.shape[1]] = bt
            args = (q.to(DEV), k.to(DEV), v.to(DEV), pool.to(DEV), torch.from_numpy(btp).to(DEV),
                    torch.from_numpy(ctx).to(DEV), B, int(ctx.max()), w.scale)
            out_static = torch.full(q.shape, 7.0, dtype=torch.bfloat16, device=DEV)
            out_heap = torch.full(q.shape, 5.0, dtype=torch.bfloat16, device=DEV)
            h.tetri_decode_attn_static(*args, out_static)
            h.tetri_decode_attn(*args, out_heap)
            torch.cuda.synchronize()
            if parts:
                assert torch.equal(out_static.view(torch.int16), out_heap.view(torch.int16)), (parts, B)
            gc.compare([out_static.cpu()], [out_heap.float().cpu().numpy()], label="static-vs-heap parts=%d B=%d" % (parts, B))
            clean = torch.nan_to_num(pool.float(), nan=0.0).numpy()
            ref = odecode.decode_attn(q.float().numpy(), k.float().numpy(), v.float().numpy(), clean, btp, ctx, w.scale)
            gc.compare([out_static.cpu()], [ref], label="static-vs-oracle parts=%d B=%d" % (parts, B))
    h.close()


def test_static_scratch_decode_rejects_sizes_beyond_the_array():
    hq, hkv, d = 8, 2, 128
    h = tetri.Tetri(hq, hkv, d, 64, 64, 4, 8)
    limit = (8 << 20) // (2 * (d + 2) * 4) // hq          # requests that still fit two parts each
    z = torch.zeros(16, dtype=torch.bfloat16, device=DEV)  # never dereferenced: the call is rejected on the host
    with pytest.raises(tetri.TetriError) as e:
        h.tetri_decode_attn_static(z, z, z, z, z.view(torch.int32), z.view(torch.int32), limit + 1, 10, 0.1, z)
    assert e.value.status == tetri.TETRI_ERR_INVALID_ARG and "static scratch" in str(e.value)
    h.close()
