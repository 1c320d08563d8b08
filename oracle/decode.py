"""Oracle of one decode iteration over the paged KV cache (test infrastructure only; plain numpy, float64).

TetriInfer Sec. 2.1: after prefill, the decode phase produces one token per iteration; the new token's
query attends to the request's cached keys and values (and to its own).  Sec. 3.4: the decode instance
batches the decode steps of many requests (continuous batching) over a paged KV cache (Sec. 5).
For request b with ctx_lens[b] cached tokens the new token sits at position ctx_lens[b]:
    out[b][h] = sum_{j=0..ctx_b} softmax_j(scale * q[b][h] . K_b[j]) * V_b[j]
with K_b[j], V_b[j] of kv head h / (Hq/Hkv) taken from the pages of request b for j < ctx_b and from
k_new[b] / v_new[b] for j = ctx_b.
"""
import numpy as np


def decode_attn(q, k_new, v_new, kv_pages, block_table, ctx_lens, scale):
    """q [B,Hq,D]; k_new, v_new [B,Hkv,D]; kv_pages [num_pages,2,Hkv,P,D]; block_table [B,max_blocks];
    ctx_lens [B].  Returns out [B,Hq,D] float64."""
    q = np.asarray(q, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    B, Hq, D = q.shape
    _, two, Hkv, P, D2 = kv_pages.shape
    assert two == 2 and D2 == D and Hq % Hkv == 0 and k_new.shape == (B, Hkv, D) == v_new.shape
    g = Hq // Hkv
    out = np.zeros((B, Hq, D), dtype=np.float64)
    for b in range(B):
        L = int(ctx_lens[b])
        keys = np.zeros((L + 1, Hkv, D), dtype=np.float64)
        vals = np.zeros((L + 1, Hkv, D), dtype=np.float64)
        for j in range(L):
            page = int(block_table[b][j // P])
            keys[j] = kv_pages[page, 0, :, j % P, :]
            vals[j] = kv_pages[page, 1, :, j % P, :]
        keys[L], vals[L] = k_new[b], v_new[b]
        for h in range(Hq):
            s = scale * (keys[:, h // g, :] @ q[b, h])
            w = np.exp(s - s.max())
            w /= w.sum()
            out[b, h] = w @ vals[:, h // g, :]
    return out


def decode_attn_fp8(q, k_new, v_new, kv_codes, block_table, ctx_lens, scale, k_scale, v_scale):
    """The same iteration over a cache of E4M3 codes (oracle/fp8.py): a cached K element is
    value(code) * k_scale, a cached V element value(code) * v_scale; the new token's K and V are taken as
    given (16-bit values, not quantised).  kv_codes [num_pages,2,Hkv,P,D] uint8."""
    from . import fp8
    pool = np.empty(kv_codes.shape, dtype=np.float64)
    pool[:, 0] = fp8.dequantize(kv_codes[:, 0], k_scale)
    pool[:, 1] = fp8.dequantize(kv_codes[:, 1], v_scale)
    # slots that no request uses may hold the NaN code; they are never read below
    return decode_attn(q, k_new, v_new, np.nan_to_num(pool, nan=0.0), block_table, ctx_lens, scale)


def decode_append_fp8(k_new, v_new, kv_codes, block_table, ctx_lens, k_scale, v_scale):
    """Caching the new tokens of a decode iteration in the E4M3 cache (in place): the codes of k_new[b] /
    v_new[b] go to slot ctx_b % P of page block_table[b][ctx_b / P]."""
    from . import fp8
    P = kv_codes.shape[3]
    for b in range(len(ctx_lens)):
        L = int(ctx_lens[b])
        page = int(block_table[b][L // P])
        kv_codes[page, 0, :, L % P, :] = fp8.quantize(np.asarray(k_new[b], dtype=np.float32), k_scale)
        kv_codes[page, 1, :, L % P, :] = fp8.quantize(np.asarray(v_new[b], dtype=np.float32), v_scale)
