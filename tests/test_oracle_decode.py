"""Pins of the decode-iteration oracle against things other than itself (no GPU).

TetriInfer Sec. 2.1 defines the decode phase only in words (one token per iteration over the KV cache),
so the pins are: the whole-sequence causal definition computed by brute force (a decode step is its
last row), the separately written C oracle of the prefill path on one-token segments, and closed forms.
"""
import numpy as np
import pytest
import torch

from oracle import decode
from paper_2401_11181_amd import synth
from helpers import oracle_inputs, brute_force_attention


def paged(ks, vs, tables, num_pages, P):
    """Cache of whole requests, placed token by token (independent of the oracles' own append)."""
    hkv, d = ks[0].shape[1:]
    pool = np.full((num_pages, 2, hkv, P, d), 777.0, dtype=np.float32)
    for r, (k, v) in enumerate(zip(ks, vs)):
        for j in range(len(k)):
            pool[tables[r][j // P], 0, :, j % P, :] = k[j]
            pool[tables[r][j // P], 1, :, j % P, :] = v[j]
    return pool


def table_array(tables):
    mb = max(len(t) for t in tables)
    bt = np.zeros((len(tables), mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt[r, :len(t)] = t
    return bt


def test_decode_step_is_the_last_row_of_causal_attention():
    """Every prefix length of several requests (GQA 4:2, scattered pages): the decode output of the
    token at position n equals row n of brute-force causal attention over tokens 0..n."""
    w = synth.small("dec-pin", [37, 5, 64, 1], 32, 4, 2, 16, seed=51)
    qs, ks, vs, tables, _ = oracle_inputs(w, torch.float32)
    pool = paged(ks, vs, tables, w.num_pages, w.page_size)
    bt = table_array(tables)
    for r, n in enumerate(w.prompt_lens):
        full = brute_force_attention(qs[r], ks[r], vs[r], w.scale)
        for pos in sorted({0, n // 2, n - 1}):
            out = decode.decode_attn(qs[r][pos][None], ks[r][pos][None], vs[r][pos][None], pool,
                                     bt[r:r + 1], [pos], w.scale)
            assert np.abs(out[0] - full[pos]).max() <= 1e-12, (r, pos)


def test_batch_matches_the_prefill_oracle_on_one_token_segments(oracle):
    """The C oracle of the chunked-prefill path, fed a chunk of one-token segments, is a second,
    separately written statement of the same sum."""
    w = synth.small("dec-pin2", [50, 17, 33, 80, 2], 16, 6, 2, 32, seed=52)
    qs, ks, vs, tables, _ = oracle_inputs(w, torch.float32)
    pool = paged(ks, vs, tables, w.num_pages, w.page_size)
    bt = table_array(tables)
    B = len(w.prompt_lens)
    ctx = np.array([n - 1 for n in w.prompt_lens], dtype=np.int32)
    q = np.stack([qs[r][ctx[r]] for r in range(B)])
    k = np.stack([ks[r][ctx[r]] for r in range(B)])
    v = np.stack([vs[r][ctx[r]] for r in range(B)])
    out = decode.decode_attn(q, k, v, pool, bt, ctx, w.scale)
    ref = oracle.chunk_prefill_attn(q, k, v, pool, bt, np.arange(B + 1, dtype=np.int32), ctx, w.scale)
    assert np.abs(out - ref).max() <= 2e-6


def test_closed_forms():
    rng = np.random.default_rng(53)
    hq, hkv, d, P, L = 4, 2, 8, 16, 21
    pool = np.zeros((4, 2, hkv, P, d), dtype=np.float32)
    vals = rng.standard_normal((L + 1, hkv, d)).astype(np.float32)
    bt = np.array([[2, 0, 3]], dtype=np.int32)
    for j in range(L):
        pool[bt[0][j // P], 1, :, j % P, :] = vals[j]          # all cached keys are zero vectors
    q = rng.standard_normal((1, hq, d)).astype(np.float32)
    zero_k = np.zeros((1, hkv, d), dtype=np.float32)
    # equal scores: the output is the mean of the L + 1 values of the head's kv head
    out = decode.decode_attn(q, zero_k, vals[L][None], pool, bt, [L], 0.7)
    for h in range(hq):
        assert np.abs(out[0, h] - vals[:, h // 2, :].astype(np.float64).mean(axis=0)).max() <= 1e-12
    # empty cache: the token attends to itself only
    out = decode.decode_attn(q, rng.standard_normal((1, hkv, d)), vals[3][None], pool, bt, [0], 0.7)
    for h in range(hq):
        assert np.abs(out[0, h] - vals[3, h // 2]).max() <= 1e-12
    # one dominant key: its value comes out (weight of the rest below 1e-30)
    k_new = np.zeros((1, hkv, d), dtype=np.float32)
    k_new[0, :, 0] = 100.0
    q1 = np.zeros((1, hq, d), dtype=np.float32)
    q1[0, :, 0] = 1.0
    out = decode.decode_attn(q1, k_new, vals[L][None], pool, bt, [L], 1.0)
    for h in range(hq):
        assert np.abs(out[0, h] - vals[L, h // 2]).max() <= 1e-12
