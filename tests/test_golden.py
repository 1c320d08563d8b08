"""Frozen oracle outputs (tests/golden/, written by tests/golden/make_golden.py from the oracle alone).

The paper prints no numeric example of this path; the stored values guard the pinned oracle against drift
(CPU test) and give the GPU path expected values that existed before it ran (GPU tests).
"""
import importlib.util
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = os.path.join(HERE, "golden")


def load_maker():
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(GOLD, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_oracle_still_computes_the_stored_values():
    mk = load_maker()
    assert np.allclose(mk.tiny_rows(), np.loadtxt(os.path.join(GOLD, "tiny_prefill_rows.txt")), rtol=0, atol=2e-7)
    rows, xfer = mk.packed_decode_rows()
    assert np.allclose(rows, np.loadtxt(os.path.join(GOLD, "ragged_decode_rows.txt")), rtol=0, atol=2e-7)
    assert np.allclose(xfer, np.loadtxt(os.path.join(GOLD, "ragged_export_sum.txt")), rtol=1e-8, atol=0)


@pytest.mark.gpu
def test_gpu_prefill_matches_the_stored_rows():
    import gpu_common as gc
    from paper_2401_11181_amd import synth
    mk = load_maker()
    w = synth.workload("tiny")
    qs, ks, vs, tables = gc.workload_tensors(w)
    outs, _, _, _ = gc.gpu_prefill(w, qs, ks, vs, tables, fused=True)
    got = np.stack([outs[0][r, h, :8].float().numpy() for r, h in mk.SAMPLES])
    want = np.loadtxt(os.path.join(GOLD, "tiny_prefill_rows.txt"))
    assert np.abs(got - want).max() <= 2e-2 and np.abs(got - want).mean() <= 2e-3


@pytest.mark.gpu
def test_gpu_decode_and_export_match_the_stored_values():
    import gpu_common as gc
    from paper_2401_11181_amd import synth, tetri
    w = synth.small("golden-decode", [37, 5, 64, 1, 23], 32, 4, 2, 64, seed=61)
    qs, ks, vs, tables = gc.workload_tensors(w)
    _, pool, _, _ = gc.gpu_prefill(w, qs, ks, vs, tables, fused=True)
    B = len(w.prompt_lens)
    mb = max(len(t) for t in tables)
    bt = np.zeros((B, mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt[r, :len(t)] = t
    ctx = np.array([n - 1 for n in w.prompt_lens], dtype=np.int32)
    dev = gc.DEV
    q = torch.stack([qs[r][ctx[r]] for r in range(B)]).to(dev)
    k = torch.stack([ks[r][ctx[r]] for r in range(B)]).to(dev)
    v = torch.stack([vs[r][ctx[r]] for r in range(B)]).to(dev)
    h = tetri.Tetri(w.num_q_heads, w.num_kv_heads, w.head_dim, 64, w.num_pages, mb, 8)
    out = torch.zeros_like(q)
    h.tetri_decode_attn(q, k, v, pool, torch.from_numpy(bt).to(dev), torch.from_numpy(ctx).to(dev), B, int(ctx.max()),
                        w.scale, out)
    cu = np.concatenate([[0], np.cumsum(w.prompt_lens)]).astype(np.int32)
    buf = torch.zeros(2 * w.num_kv_heads * w.head_dim * int(cu[-1]), dtype=torch.bfloat16, device=dev)
    h.tetri_kv_export(pool, torch.from_numpy(bt).to(dev), torch.from_numpy(cu).to(dev), None, B, int(cu[-1]), buf)
    torch.cuda.synchronize()
    got = out.cpu().float().numpy()[:, :, :8].reshape(-1, 8)
    want = np.loadtxt(os.path.join(GOLD, "ragged_decode_rows.txt"))
    assert np.abs(got - want).max() <= 2e-2 and np.abs(got - want).mean() <= 2e-3
    n, total = np.loadtxt(os.path.join(GOLD, "ragged_export_sum.txt"))
    assert buf.numel() == int(n)
    assert abs(float(buf.cpu().double().abs().sum()) - total) <= 1e-9 * total     # the copy is exact
    h.close()
