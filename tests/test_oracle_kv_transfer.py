"""Pins of the KV-transfer oracle against things other than itself (no GPU).

TetriInfer Sec. 3.3.4 gives the operation (the prefilled KV cache of a request, or of a chunk's slice of
it, travels to the decode instance) but prints no example, so the pins are: a case small enough to
write out by hand, the closed form "export of what the chunked prefill appended = the request's K
and V, transposed", brute-force indexing on the receiver, and the invariant that the two
granularities carry the same data.
"""
import numpy as np
import pytest

from oracle import kv_transfer, packer
from paper_2401_11181_amd import synth
from helpers import oracle_inputs


def coded_pool(num_pages, hkv, p, d):
    """Pool whose every element spells its own coordinates."""
    pool = np.zeros((num_pages, 2, hkv, p, d), dtype=np.float32)
    for page in range(num_pages):
        for kv in range(2):
            for h in range(hkv):
                for s in range(p):
                    for e in range(d):
                        pool[page, kv, h, s, e] = 10000 * page + 1000 * kv + 100 * h + 10 * s + e
    return pool


def test_hand_written_example():
    """Pages of 2 slots, one head, one element.  Request 0 = tokens 1..3 of a request living on pages
    (3, 1); request 1 = token 0 of a request on page 2.  Written out by hand:
    token 1 -> page 3 slot 1, token 2 -> page 1 slot 0, token 3 -> page 1 slot 1."""
    pool = coded_pool(4, 1, 2, 1)
    bt = np.array([[3, 1], [2, 0]], dtype=np.int32)
    buf = kv_transfer.kv_export(pool, bt, [0, 3, 4], [1, 0])
    #             K of request 0        V of request 0        K, V of request 1
    expect = [30010, 10000, 10010,  31010, 11000, 11010,  20000, 21000]
    assert buf.tolist() == expect


def test_hand_written_example_two_heads_two_elements():
    """Head-major inside K and inside V, tokens next, elements last."""
    pool = coded_pool(3, 2, 2, 2)
    bt = np.array([[2, 0]], dtype=np.int32)
    buf = kv_transfer.kv_export(pool, bt, [0, 2], [1])       # token 1 -> page 2 slot 1, token 2 -> page 0 slot 0
    expect = [20010, 20011, 0, 1,            # K head 0: token 1, token 2
              20110, 20111, 100, 101,        # K head 1
              21010, 21011, 1000, 1001,      # V head 0
              21110, 21111, 1100, 1101]      # V head 1
    assert buf.tolist() == expect


def test_export_of_prefilled_cache_is_the_requests_k_and_v(oracle):
    """Chunked prefill (C oracle, scattered pages, requests merged into chunks) followed by a
    request-level export gives K and V of each request as [Hkv][n][D]: the closed form."""
    w = synth.small("xfer", [37, 5, 64, 1, 23], 32, 4, 2, 16, seed=41)
    qs, ks, vs, tables, pool = oracle_inputs(w)
    oracle.prefill(qs, ks, vs, w.order, w.chunk_size, pool, tables, w.scale)
    mb = max(len(t) for t in tables)
    bt = np.zeros((len(tables), mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt[r, :len(t)] = t
    cu = np.concatenate([[0], np.cumsum(w.prompt_lens)])
    buf = kv_transfer.kv_export(pool, bt, cu)
    hkv, d = w.num_kv_heads, w.head_dim
    for r, n in enumerate(w.prompt_lens):
        block = buf[2 * hkv * d * cu[r]: 2 * hkv * d * cu[r + 1]].reshape(2, hkv, n, d)
        assert np.array_equal(block[0], ks[r].transpose(1, 0, 2))
        assert np.array_equal(block[1], vs[r].transpose(1, 0, 2))


def test_import_places_every_token_and_nothing_else():
    """Receiver with its own page placement: brute-force indexing finds every token where the
    receiver's block table says, and every other slot keeps its sentinel."""
    rng = np.random.default_rng(7)
    hkv, p, d = 3, 4, 2
    lens, first = [9, 1, 6], [0, 3, 5]
    cu = np.concatenate([[0], np.cumsum(lens)])
    buf = rng.standard_normal(2 * hkv * d * cu[-1]).astype(np.float32)
    pages = rng.permutation(16)
    bt = np.array([[pages[0], pages[1], pages[2]], [pages[3], 0, 0], [0, pages[4], pages[5]]], dtype=np.int32)
    pool = np.full((16, 2, hkv, p, d), 555.0, dtype=np.float32)
    kv_transfer.kv_import(buf, pool, bt, cu, first)
    touched = np.zeros(pool.shape, dtype=bool)
    for r, n in enumerate(lens):
        for t in range(n):
            pos = first[r] + t
            for kv in range(2):
                for h in range(hkv):
                    for e in range(d):
                        at = 2 * hkv * d * cu[r] + ((kv * hkv + h) * n + t) * d + e
                        assert pool[bt[r, pos // p], kv, h, pos % p, e] == buf[at]
                        touched[bt[r, pos // p], kv, h, pos % p, e] = True
    assert touched.sum() == buf.size
    assert (pool[~touched] == 555.0).all()


def test_import_inverts_export_across_different_placements():
    rng = np.random.default_rng(8)
    hkv, p, d = 2, 16, 8
    lens, first = [40, 17], [0, 0]
    cu = np.concatenate([[0], np.cumsum(lens)])
    src = rng.standard_normal((12, 2, hkv, p, d)).astype(np.float32)
    bt_src = np.array([[5, 1, 9], [7, 3, 0]], dtype=np.int32)
    bt_dst = np.array([[2, 11, 4], [0, 6, 0]], dtype=np.int32)
    buf = kv_transfer.kv_export(src, bt_src, cu, first)
    dst = np.zeros_like(src)
    kv_transfer.kv_import(buf, dst, bt_dst, cu, first)
    again = kv_transfer.kv_export(dst, bt_dst, cu, first)
    assert np.array_equal(buf, again)
    # a full page moved as a whole: logical page 1 of request 0
    assert np.array_equal(dst[11], src[1])


def test_chunk_level_slices_carry_the_same_data_as_request_level():
    """Sec. 3.3.4: chunk-level transfer sends each chunk's slice as it is produced, request-level the
    aggregate.  Importing the slices one by one fills the receiver exactly like one request-level import."""
    rng = np.random.default_rng(9)
    hkv, p, d, chunk = 2, 16, 4, 24
    lens = [50, 7, 31]
    plan = packer.pack_chunks(lens, list(range(len(lens))), chunk)
    src = rng.standard_normal((10, 2, hkv, p, d)).astype(np.float32)
    tables = np.array([[1, 4, 6, 8], [2, 0, 0, 0], [9, 3, 0, 0]], dtype=np.int32)
    cu_req = np.concatenate([[0], np.cumsum(lens)])
    whole = np.full_like(src, 3.0)
    kv_transfer.kv_import(kv_transfer.kv_export(src, tables, cu_req), whole, tables, cu_req)
    piecewise = np.full_like(src, 3.0)
    for segs in plan:
        cu, ctx = packer.chunk_arrays(segs)
        bt = tables[[req for req, _s, _n in segs]]
        kv_transfer.kv_import(kv_transfer.kv_export(src, bt, cu, ctx), piecewise, bt, cu, ctx)
    assert np.array_equal(whole, piecewise)


def test_empty_requests_and_empty_batch():
    pool = coded_pool(2, 1, 2, 1)
    bt = np.array([[1, 0], [0, 1]], dtype=np.int32)
    assert kv_transfer.kv_export(pool, bt, [0, 0, 0]).size == 0
    buf = kv_transfer.kv_export(pool, bt, [0, 0, 2], [0, 1])     # request 1: tokens 1, 2 -> page 0 slot 1, page 1 slot 0
    assert buf.tolist() == [10, 10000, 1010, 11000]
    before = pool.copy()
    kv_transfer.kv_import(np.zeros(0, dtype=np.float32), pool, bt, [0, 0, 0])
    assert np.array_equal(pool, before)
