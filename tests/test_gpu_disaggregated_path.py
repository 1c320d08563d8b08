"""The whole data path of a disaggregated request on one GPU (TetriInfer Sec. 3: prefill instance ->
dispatcher -> decode instance): chunked prefill into the prefill instance's pool, request-level export,
import into a second pool with another page placement, then decode iterations on that pool.  Every
decoded row must equal the row of one-shot causal attention over the full sequence (oracle prefill), and
the decode pool must end up holding exactly the K/V of every token at the receiver's placement."""
import numpy as np
import pytest
import torch

from paper_2401_11181_amd import synth, tetri
import gpu_common as gc

pytestmark = pytest.mark.gpu
DEV = gc.DEV


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 128), (3, 3, 64)])
def test_prefill_export_import_decode(oracle, hq, hkv, d):
    n_dec = 6
    full = synth.small("disagg", [150 + n_dec, 40 + n_dec, 7 + n_dec, 260 + n_dec], 64, hq, hkv, d, seed=400 + d)
    qs, ks, vs, tables = gc.workload_tensors(full)
    ref, _, _ = gc.oracle_prefill(oracle, full, qs, ks, vs, tables)
    lens = [n - n_dec for n in full.prompt_lens]
    B = len(lens)

    # prefill instance: the prompts without their last n_dec tokens
    pre = synth.small("disagg", lens, 64, hq, hkv, d, seed=400 + d)
    pre.num_pages = full.num_pages
    cut = lambda ts: [t[:n] for t, n in zip(ts, lens)]
    outs, pool_a, _, _ = gc.gpu_prefill(pre, cut(qs), cut(ks), cut(vs), tables, fused=True)
    gc.compare(outs, [r[:n] for r, n in zip(ref, lens)], label="disagg-prefill")

    # dispatcher: request-level export
    mb = max(len(t) for t in tables)
    bt_a = np.zeros((B, mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt_a[r, :len(t)] = t
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    h = tetri.Tetri(hq, hkv, d, 64, full.num_pages, mb, 8)
    d_cu = torch.from_numpy(cu).to(DEV)
    buf = torch.zeros(2 * hkv * d * int(cu[-1]), dtype=torch.bfloat16, device=DEV)
    h.tetri_kv_export(pool_a, torch.from_numpy(bt_a).to(DEV), d_cu, None, B, int(cu[-1]), buf)

    # decode instance: its own pool and placement (the same page ids mirrored)
    bt_b = (full.num_pages - 1 - bt_a).astype(np.int32)
    d_bt_b = torch.from_numpy(bt_b).to(DEV)
    pool_b = synth.pool_sentinel(tuple(pool_a.shape), device=DEV)
    h.tetri_kv_import(buf, d_bt_b, d_cu, None, B, int(cu[-1]), pool_b)
    got = [[] for _ in range(B)]
    for step in range(n_dec):
        pos = [n + step for n in lens]
        dq = torch.stack([qs[r][pos[r]] for r in range(B)]).to(DEV)
        dk = torch.stack([ks[r][pos[r]] for r in range(B)]).to(DEV)
        dv = torch.stack([vs[r][pos[r]] for r in range(B)]).to(DEV)
        out = torch.zeros_like(dq)
        h.tetri_decode_attn_append(dq, dk, dv, pool_b, d_bt_b, torch.tensor(pos, dtype=torch.int32, device=DEV), B,
                                   max(pos), full.scale, out)
        torch.cuda.synchronize()
        for r in range(B):
            got[r].append(out[r].cpu())
    print(gc.compare([torch.stack(g) for g in got], [ref[r][lens[r]:] for r in range(B)], label="disagg-decode"))

    # the decode pool: every token of every request where the receiver's table says, nothing else touched
    want = synth.pool_sentinel(tuple(pool_a.shape))
    for r in range(B):
        for j in range(full.prompt_lens[r]):
            want[bt_b[r, j // 16], 0, :, j % 16, :] = ks[r][j]
            want[bt_b[r, j // 16], 1, :, j % 16, :] = vs[r][j]
    assert torch.equal(pool_b.cpu().view(torch.int16), want.view(torch.int16))
    h.close()
