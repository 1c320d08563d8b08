"""Oracle of chunked-prefill attention over a KV cache of FP8 E4M3 codes (test infrastructure only; plain
numpy, float64).

TetriInfer Sec. 3.3.3: a prompt is prefilled one fixed-size chunk at a time, several prompts may share a
chunk; Sec. 2.1: row t of a segment (position p = ctx + t of its request) attends to the request's
positions 0..p; Sec. 3.4: the earlier positions live in a paged cache.  The paper keeps that cache in the
model's 16-bit type; the cache of codes is this build's extension (oracle/fp8.py states the format).  The
reading taken, the same as for the decode iteration over such a cache (oracle/decode.py): a cached K element
is value(code) * k_scale, a cached V element value(code) * v_scale; the chunk's own rows k_new / v_new are
taken as given (16-bit values, not quantised), whether or not they are cached afterwards.
    out[t][h] = sum_{j=0..p} softmax_j(scale * q[t][h] . K[j]) * V[j]
with K[j], V[j] of kv head h / (Hq / Hkv) from the cache for j < ctx and from row cu[s] + (j - ctx) of
k_new / v_new for j >= ctx.  Rows of the chunk that belong to no segment are zero.
"""
import numpy as np

from . import fp8


def _segment_kv(k_new, v_new, k_vals, v_vals, row, L, a, b, kh, P):
    """Keys and values [L + n, D] (float64) of kv head kh that the rows a..b-1 of a segment may see: the L
    cached ones through the block-table row, then the chunk's own."""
    n, D = b - a, k_new.shape[2]
    keys = np.zeros((L + n, D), dtype=np.float64)
    vals = np.zeros((L + n, D), dtype=np.float64)
    for j in range(L):
        page = int(row[j // P])
        keys[j] = k_vals[page, kh, j % P, :]
        vals[j] = v_vals[page, kh, j % P, :]
    keys[L:] = k_new[a:b, kh, :]
    vals[L:] = v_new[a:b, kh, :]
    return keys, vals


def _one_row(qrow, keys, vals, visible, scale):
    s = scale * (keys[:visible] @ qrow)
    w = np.exp(s - s.max())
    w /= w.sum()
    return w @ vals[:visible]


def chunk_prefill_attn_fp8(q, k_new, v_new, kv_codes, block_table, cu, ctx, scale, k_scale, v_scale):
    """q [C,Hq,D]; k_new, v_new [C,Hkv,D]; kv_codes [num_pages,2,Hkv,P,D] uint8; block_table [S,max_blocks];
    cu [S+1]; ctx [S].  Returns out [C,Hq,D] float64."""
    q = np.asarray(q, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    C, Hq, D = q.shape
    _, two, Hkv, P, D2 = kv_codes.shape
    assert two == 2 and D2 == D and Hq % Hkv == 0 and k_new.shape == (C, Hkv, D) == v_new.shape
    g = Hq // Hkv
    k_vals = fp8.dequantize(kv_codes[:, 0], k_scale)
    v_vals = fp8.dequantize(kv_codes[:, 1], v_scale)
    out = np.zeros((C, Hq, D), dtype=np.float64)
    for s in range(len(ctx)):
        a, b, L = int(cu[s]), int(cu[s + 1]), int(ctx[s])
        for kh in range(Hkv):
            keys, vals = _segment_kv(k_new, v_new, k_vals, v_vals, block_table[s], L, a, b, kh, P)
            for h in range(kh * g, (kh + 1) * g):
                for t in range(b - a):
                    out[a + t, h] = _one_row(q[a + t, h], keys, vals, L + t + 1, scale)
    return out


def chunk_prefill_attn_fp8_samples(q, k_new, v_new, kv_codes, block_table, cu, ctx, scale, k_scale, v_scale,
                                   rows, heads):
    """The same for selected (chunk row, head) pairs only: [len(rows), D] float64.  Every row must belong to a
    segment."""
    q = np.asarray(q, dtype=np.float64)
    k_new = np.asarray(k_new, dtype=np.float64)
    v_new = np.asarray(v_new, dtype=np.float64)
    _, Hq, D = q.shape
    _, _, Hkv, P, _ = kv_codes.shape
    g = Hq // Hkv
    table = fp8.decode_table()
    ks, vs = np.float64(np.float32(k_scale)), np.float64(np.float32(v_scale))
    out = np.zeros((len(rows), D), dtype=np.float64)
    cache = {}
    for i, (r, h) in enumerate(zip(rows, heads)):
        r, h = int(r), int(h)
        s = max(x for x in range(len(ctx)) if int(cu[x]) <= r)
        a, b, L = int(cu[s]), int(cu[s + 1]), int(ctx[s])
        assert a <= r < b
        kh = h // g
        if (s, kh) not in cache:
            cache.clear()                              # one segment and head at a time: sort the samples to profit
            pages = np.asarray(block_table[s][:(L + P - 1) // P], dtype=np.int64)
            kc = kv_codes[pages, 0, kh].reshape(-1, D)[:L]
            vc = kv_codes[pages, 1, kh].reshape(-1, D)[:L]
            keys = np.concatenate([table[kc] * ks, k_new[a:b, kh, :]], axis=0)
            vals = np.concatenate([table[vc] * vs, v_new[a:b, kh, :]], axis=0)
            cache[(s, kh)] = (keys, vals)
        keys, vals = cache[(s, kh)]
        out[i] = _one_row(q[r, h], keys, vals, L + (r - a) + 1, scale)
    return out


def prefill_append_fp8(k_new, v_new, kv_codes, block_table, cu, ctx, k_scale, v_scale):
    """Caching a chunk's rows in the cache of codes (in place): row t of segment s goes, quantised under the
    tensor's scale (fp8.quantize), to slot (ctx + t) % P of page block_table[s][(ctx + t) / P]."""
    P = kv_codes.shape[3]
    for s in range(len(ctx)):
        a, b, L = int(cu[s]), int(cu[s + 1]), int(ctx[s])
        for t in range(b - a):
            pos = L + t
            page = int(block_table[s][pos // P])
            kv_codes[page, 0, :, pos % P, :] = fp8.quantize(np.asarray(k_new[a + t], dtype=np.float32), k_scale)
            kv_codes[page, 1, :, pos % P, :] = fp8.quantize(np.asarray(v_new[a + t], dtype=np.float32), v_scale)
