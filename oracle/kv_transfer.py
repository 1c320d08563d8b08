"""Oracle of the KV transfer buffer (test infrastructure only; plain numpy, one token at a time).

TetriInfer Sec. 3.3.4 (Dispatcher): once a request is prefilled, its KV cache goes from the prefill
instance's accelerator memory to the chosen decode instance.  Two granularities are named there:
request-level (the whole request after its last chunk; the one the paper implements) and
chunk-level (each chunk's slice as soon as it exists).  Both are the same operation on a token
range [first, first + n) of a request; only the range differs.

The paper fixes no wire format.  The reading taken here: the buffer holds, request after request,
a dense block  [2 (K, V)][Hkv][n_r][D]  that does not depend on the page size or the page
placement of either side; request r's block starts at element 2 * Hkv * D * cu_tokens[r].
Sec. 3.4 / Sec. 5: both instances keep the cache in pages, so the receiver scatters the block into
pages of its own through its own block table.
"""
import numpy as np


def _ranges(cu_tokens, first_tokens):
    cu = np.asarray(cu_tokens, dtype=np.int64)
    R = len(cu) - 1
    first = np.zeros(R, dtype=np.int64) if first_tokens is None else np.asarray(first_tokens, dtype=np.int64)
    assert cu[0] == 0 and len(first) == R and (np.diff(cu) >= 0).all() and (first >= 0).all()
    return cu, first, R


def kv_export(kv_pages, block_table, cu_tokens, first_tokens=None):
    """Gather tokens [first_r, first_r + n_r) of every request r out of the paged pool.

    kv_pages [num_pages, 2, Hkv, P, D]; block_table [R, max_blocks]: logical page b of request r is
    physical page block_table[r][b]; cu_tokens [R+1]: prefix sums of n_r.  Returns the flat buffer.
    """
    cu, first, R = _ranges(cu_tokens, first_tokens)
    _, two, Hkv, P, D = kv_pages.shape
    assert two == 2
    buf = np.zeros(2 * Hkv * D * int(cu[R]), dtype=kv_pages.dtype)
    for r in range(R):
        n = int(cu[r + 1] - cu[r])
        block = buf[2 * Hkv * D * int(cu[r]): 2 * Hkv * D * int(cu[r + 1])].reshape(2, Hkv, n, D)
        for t in range(n):
            pos = int(first[r]) + t
            page = int(block_table[r][pos // P])
            block[:, :, t, :] = kv_pages[page, :, :, pos % P, :]
    return buf


def kv_import(buf, kv_pages, block_table, cu_tokens, first_tokens=None):
    """The inverse on the receiver: scatter every request's dense block into kv_pages (in place)
    through the receiver's block table.  Slots outside the token ranges keep their contents."""
    cu, first, R = _ranges(cu_tokens, first_tokens)
    _, two, Hkv, P, D = kv_pages.shape
    assert two == 2 and buf.size == 2 * Hkv * D * int(cu[R])
    for r in range(R):
        n = int(cu[r + 1] - cu[r])
        block = buf[2 * Hkv * D * int(cu[r]): 2 * Hkv * D * int(cu[r + 1])].reshape(2, Hkv, n, D)
        for t in range(n):
            pos = int(first[r]) + t
            page = int(block_table[r][pos // P])
            kv_pages[page, :, :, pos % P, :] = block[:, :, t, :]


def kv_export_fp8(kv_pages, block_table, cu_tokens, first_tokens, k_scale, v_scale):
    """Export with quantisation (oracle/fp8.py): the same dense blocks, one E4M3 code (uint8) per element;
    the K half of every request's block under k_scale, the V half under v_scale."""
    from . import fp8
    cu, _first, R = _ranges(cu_tokens, first_tokens)
    _, _two, Hkv, _P, D = kv_pages.shape
    dense = kv_export(np.asarray(kv_pages, dtype=np.float32), block_table, cu_tokens, first_tokens)
    codes = np.zeros(dense.shape, dtype=np.uint8)
    for r in range(R):
        lo, hi = 2 * Hkv * D * int(cu[r]), 2 * Hkv * D * int(cu[r + 1])
        half = (hi - lo) // 2
        codes[lo:lo + half] = fp8.quantize(dense[lo:lo + half], k_scale)
        codes[lo + half:hi] = fp8.quantize(dense[lo + half:hi], v_scale)
    return codes
