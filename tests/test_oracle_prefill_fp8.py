"""Pins of the oracle of chunked prefill over a cache of FP8 codes (oracle/prefill_fp8.py) against things other
than itself: scalar loops written out from the definition, the 16-bit C oracle on a pool of dequantised values
(scales that are powers of two make those exact in float32), closed forms, the decode-iteration and KV-transfer
oracles where the definitions coincide.  CPU only."""
import math

import numpy as np

import helpers
from oracle import decode, fp8, kv_transfer, prefill_fp8


def small_case(seed, segs=((5, 3), (0, 4), (17, 2)), hq=4, hkv=2, d=8, P=4, C=12, n_pages=16):
    """segs: (cached tokens, rows) per segment.  Returns q, k_new, v_new, codes, bt, cu, ctx; unused slots of the
    pool hold the NaN code."""
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((C, hq, d)).astype(np.float32)
    k_new = rng.standard_normal((C, hkv, d)).astype(np.float32)
    v_new = rng.standard_normal((C, hkv, d)).astype(np.float32)
    codes = np.full((n_pages, 2, hkv, P, d), 0x7F, dtype=np.uint8)
    perm = rng.permutation(n_pages)
    ctx = [L for L, _ in segs]
    cu = np.concatenate([[0], np.cumsum([n for _, n in segs])]).astype(np.int32)
    assert cu[-1] <= C
    max_blocks = max((L + n + P - 1) // P for L, n in segs)
    bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
    at = 0
    for s, (L, n) in enumerate(segs):
        nb = (L + n + P - 1) // P
        bt[s, :nb] = perm[at:at + nb]
        at += nb
        for j in range(L):
            codes[bt[s, j // P], :, :, j % P, :] = rng.integers(0, 0x7F, size=(2, hkv, d)) | (rng.integers(0, 2, size=(2, hkv, d)) << 7)
    assert at <= n_pages
    return q, k_new, v_new, codes, bt, cu, ctx


def test_scalar_loops_from_the_definition():
    q, k_new, v_new, codes, bt, cu, ctx = small_case(81)
    scale, k_scale, v_scale = 0.31, 0.0123, 0.07
    out = prefill_fp8.chunk_prefill_attn_fp8(q, k_new, v_new, codes, bt, cu, ctx, scale, k_scale, v_scale)
    t = fp8.decode_table()
    C, hq, d = q.shape
    hkv, P = k_new.shape[1], codes.shape[3]
    ks, vs = float(np.float32(k_scale)), float(np.float32(v_scale))
    want = np.zeros((C, hq, d))
    for s in range(len(ctx)):
        for row in range(cu[s], cu[s + 1]):
            p = ctx[s] + (row - cu[s])
            for h in range(hq):
                kh = h // (hq // hkv)
                scores, values = [], []
                for j in range(p + 1):
                    if j < ctx[s]:
                        page, slot = int(bt[s][j // P]), j % P
                        kj = [t[codes[page, 0, kh, slot, x]] * ks for x in range(d)]
                        vj = [t[codes[page, 1, kh, slot, x]] * vs for x in range(d)]
                    else:
                        kj = [float(k_new[cu[s] + j - ctx[s], kh, x]) for x in range(d)]
                        vj = [float(v_new[cu[s] + j - ctx[s], kh, x]) for x in range(d)]
                    scores.append(scale * sum(float(q[row, h, x]) * kj[x] for x in range(d)))
                    values.append(vj)
                mx = max(scores)
                w = [math.exp(x - mx) for x in scores]
                tot = sum(w)
                for x in range(d):
                    want[row, h, x] = sum(w[j] * values[j][x] for j in range(p + 1)) / tot
    assert np.abs(out - want).max() <= 1e-12
    assert not out[cu[-1]:].any()


def test_equals_the_16_bit_oracle_on_the_dequantised_pool(oracle):
    """With scales that are powers of two value(code) * scale is a float32 (a bf16, even): the cache of codes is
    then an ordinary pool and the C oracle applies."""
    q, k_new, v_new, codes, bt, cu, ctx = small_case(82, segs=((9, 5), (0, 2), (30, 6)), hq=6, hkv=2, d=16, P=16, C=16, n_pages=8)
    k_scale, v_scale = 2.0 ** -5, 2.0 ** -3
    pool = np.zeros(codes.shape, dtype=np.float32)
    t = np.nan_to_num(fp8.decode_table(), nan=0.0)       # unused slots: any number, never read
    pool[:, 0] = t[codes[:, 0]] * k_scale
    pool[:, 1] = t[codes[:, 1]] * v_scale
    want = oracle.chunk_prefill_attn(q, k_new, v_new, pool, bt, cu, ctx, 0.25)
    out = prefill_fp8.chunk_prefill_attn_fp8(q, k_new, v_new, codes, bt, cu, ctx, 0.25, k_scale, v_scale)
    assert np.abs(out - want).max() <= 2e-6               # the C oracle returns float32


def test_first_chunk_never_reads_the_cache():
    """No cached tokens: plain causal attention of the chunk's own rows, whatever the pool and the scales hold."""
    q, k_new, v_new, codes, bt, cu, ctx = small_case(83, segs=((0, 7),), C=8)
    assert (codes == 0x7F).all()
    out = prefill_fp8.chunk_prefill_attn_fp8(q, k_new, v_new, codes, bt, cu, ctx, 0.4, 123.0, 1e-3)
    want = helpers.brute_force_attention(q[:7], k_new[:7], v_new[:7], 0.4)
    assert np.abs(out[:7] - want).max() <= 1e-12 and not out[7:].any()


def test_zero_queries_average_the_visible_values():
    """q = 0: every visible position weighs the same, so row t is the mean of the dequantised cached values and
    of the chunk's values up to t, written out from the table."""
    q, k_new, v_new, codes, bt, cu, ctx = small_case(84)
    t = fp8.decode_table()
    out = prefill_fp8.chunk_prefill_attn_fp8(np.zeros_like(q), k_new, v_new, codes, bt, cu, ctx, 0.9, 3.0, 0.125)
    P, hq, hkv = codes.shape[3], q.shape[1], k_new.shape[1]
    for s in range(len(ctx)):
        for h in range(hq):
            kh = h // (hq // hkv)
            cached = sum(t[codes[bt[s][j // P], 1, kh, j % P, :]] for j in range(ctx[s])) * 0.125 if ctx[s] else 0.0
            for i in range(cu[s + 1] - cu[s]):
                want = (cached + v_new[cu[s]:cu[s] + i + 1, kh, :].astype(np.float64).sum(axis=0)) / (ctx[s] + i + 1)
                assert np.abs(out[cu[s] + i, h] - want).max() <= 1e-12


def test_the_k_scale_multiplies_cached_scores_only_and_the_v_scale_cached_values_only():
    """One cached key with code value 2 under k_scale 5, query e0: cached score 10.  The chunk's single row has
    key 3 * e0 (score 3, no scale) and value 7; the cached value is code 1.0 under v_scale 0.5."""
    hq = hkv = 1
    d, P = 4, 4
    codes = np.full((2, 2, hkv, P, d), 0x7F, dtype=np.uint8)
    codes[1, 0, 0, 0, :] = [0x40, 0, 0, 0]
    codes[1, 1, 0, 0, :] = 0x38
    q = np.zeros((1, hq, d), np.float32)
    q[0, 0, 0] = 1.0
    k = np.zeros((1, hkv, d), np.float32)
    k[0, 0, 0] = 3.0
    v = np.full((1, hkv, d), 7.0, np.float32)
    out = prefill_fp8.chunk_prefill_attn_fp8(q, k, v, codes, np.array([[1]], np.int32), [0, 1], [1], 1.0, 5.0, 0.5)
    w = math.exp(10.0) / (math.exp(10.0) + math.exp(3.0))
    assert np.abs(out[0, 0] - (w * 0.5 + (1 - w) * 7.0)).max() <= 1e-12


def test_samples_equal_full_rows():
    q, k_new, v_new, codes, bt, cu, ctx = small_case(85, segs=((21, 6), (3, 5)), hq=6, hkv=3, d=8, P=4, C=12)
    full = prefill_fp8.chunk_prefill_attn_fp8(q, k_new, v_new, codes, bt, cu, ctx, 0.3, 0.02, 0.05)
    rows = [0, 5, 3, 6, 10, 10, 7]
    heads = [0, 5, 2, 1, 4, 3, 0]
    got = prefill_fp8.chunk_prefill_attn_fp8_samples(q, k_new, v_new, codes, bt, cu, ctx, 0.3, 0.02, 0.05, rows, heads)
    for i, (r, h) in enumerate(zip(rows, heads)):
        assert np.abs(got[i] - full[r, h]).max() <= 1e-12


def test_append_places_the_codes():
    """Hand example: pages of 4 slots, one head, two elements.  Segment 0 has 3 cached tokens and 2 rows (positions
    3 and 4: page bt[0][0] slot 3, page bt[0][1] slot 0), segment 1 none and 1 row (page bt[1][0] slot 0)."""
    codes = np.full((4, 2, 1, 4, 2), 0x7F, dtype=np.uint8)
    bt = np.array([[2, 0], [3, 1]], dtype=np.int32)
    k = np.array([[[1.0, -2.0]], [[0.5, 448.0]], [[3.0, 0.0]], [[9.0, 9.0]]], dtype=np.float32)     # row 3: padding
    v = np.array([[[3.0, 0.25]], [[-1.0, 8.0]], [[100.0, 1.0]], [[9.0, 9.0]]], dtype=np.float32)
    prefill_fp8.prefill_append_fp8(k, v, codes, bt, [0, 2, 3], [3, 0], 1.0, 2.0)
    t = fp8.decode_table()
    assert t[codes[2, 0, 0, 3]].tolist() == [1.0, -2.0] and t[codes[2, 1, 0, 3]].tolist() == [1.5, 0.125]
    assert t[codes[0, 0, 0, 0]].tolist() == [0.5, 448.0] and t[codes[0, 1, 0, 0]].tolist() == [-0.5, 4.0]
    assert t[codes[3, 0, 0, 0]].tolist() == [3.0, 0.0] and t[codes[3, 1, 0, 0]].tolist() == [48.0, 0.5]
    assert (codes == 0x7F).sum() == codes.size - 12


def test_append_of_single_rows_is_the_decode_append():
    rng = np.random.default_rng(86)
    hkv, d, P = 2, 8, 4
    k = (rng.standard_normal((3, hkv, d)) * 2).astype(np.float32)
    v = (rng.standard_normal((3, hkv, d)) * 2).astype(np.float32)
    bt = np.array([[5, 1, 0], [2, 4, 0], [3, 6, 7]], dtype=np.int32)
    ctx = [6, 0, 11]
    a = np.full((8, 2, hkv, P, d), 0x7F, dtype=np.uint8)
    b = a.copy()
    prefill_fp8.prefill_append_fp8(k, v, a, bt, [0, 1, 2, 3], ctx, 0.03, 0.011)
    decode.decode_append_fp8(k, v, b, bt, ctx, 0.03, 0.011)
    assert np.array_equal(a, b) and (a != 0x7F).sum() >= 3 * 2 * hkv * d - 8


def test_append_equals_16_bit_append_followed_by_quantising_export(oracle):
    """Quantising on the way into the cache gives the codes that exporting the 16-bit cache under the same scales
    gives (the export oracle quantises what the pool holds)."""
    rng = np.random.default_rng(87)
    hkv, d, P, n = 2, 8, 16, 11
    k = rng.standard_normal((n, hkv, d)).astype(np.float32)
    v = rng.standard_normal((n, hkv, d)).astype(np.float32)
    bt = np.array([[3, 1]], dtype=np.int32)
    pool = np.zeros((4, 2, hkv, P, d), dtype=np.float32)
    oracle.kv_append(k, v, pool, bt, [0, n], [7])
    dense = kv_transfer.kv_export_fp8(pool, bt, [0, n], [7], 0.02, 0.05)           # [2][hkv][n][d]
    codes = np.full((4, 2, hkv, P, d), 0x7F, dtype=np.uint8)
    prefill_fp8.prefill_append_fp8(k, v, codes, bt, [0, n], [7], 0.02, 0.05)
    got = np.stack([codes[bt[0][(7 + i) // P], :, :, (7 + i) % P, :] for i in range(n)], axis=2)   # [2][hkv][n][d]
    assert np.array_equal(got.reshape(-1), np.asarray(dense).reshape(-1))


def test_two_chunks_in_a_row_equal_attention_over_the_quantised_first_chunk():
    """Chunk 1 appended as codes, then chunk 2: its rows see the quantised keys and values of chunk 1 and their own
    unquantised ones.  Checked against unpaged attention over the explicit concatenation."""
    rng = np.random.default_rng(88)
    hq, hkv, d, P, n1, n2 = 2, 1, 8, 4, 6, 5
    qs = rng.standard_normal((n1 + n2, hq, d)).astype(np.float32)
    ks = rng.standard_normal((n1 + n2, hkv, d)).astype(np.float32)
    vs = rng.standard_normal((n1 + n2, hkv, d)).astype(np.float32)
    bt = np.array([[2, 0, 3]], dtype=np.int32)
    codes = np.full((4, 2, hkv, P, d), 0x7F, dtype=np.uint8)
    k_scale, v_scale = 0.013, 0.017
    prefill_fp8.prefill_append_fp8(ks[:n1], vs[:n1], codes, bt, [0, n1], [0], k_scale, v_scale)
    out = prefill_fp8.chunk_prefill_attn_fp8(qs[n1:], ks[n1:], vs[n1:], codes, bt, [0, n2], [n1], 0.35, k_scale, v_scale)
    kq = fp8.dequantize(fp8.quantize(ks[:n1], k_scale), k_scale)
    vq = fp8.dequantize(fp8.quantize(vs[:n1], v_scale), v_scale)
    want = helpers.brute_force_attention(qs, np.concatenate([kq, ks[n1:]]), np.concatenate([vq, vs[n1:]]), 0.35)[n1:]
    assert np.abs(out - want).max() <= 1e-12
    assert np.abs(kq - ks[:n1]).max() <= 0.07 * np.abs(ks[:n1]).max()
