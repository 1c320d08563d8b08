"""ctypes front end of the C oracle (test infrastructure only).

Each function names the C routine it marshals for; the arithmetic lives in tetri_oracle.c.
Paper passages followed: TetriInfer Sec. 3.3.3 (chunked prefill, one chunk at a time, the
per-request progress variable), Sec. 2.1 (prefill generates the KV cache), Sec. 3.4 (paged KV).
"""
import ctypes
import os
import subprocess

import numpy as np

from . import packer

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tetri_oracle.c")
_LIB = os.path.join(_HERE, "libtetri_oracle.so")
_lib = None


def build(force=False, src=_SRC, out=_LIB):
    """Compile the C oracle with gcc (-O2 -fopenmp)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra",
                               "-o", out, src, "-lm"])
    return out


def load(path=None):
    """Load (building first if needed) the oracle library; ``path`` loads another build of it."""
    global _lib
    if path is not None:
        return _declare(ctypes.CDLL(path))
    if _lib is None:
        _lib = _declare(ctypes.CDLL(build()))
    return _lib


def _declare(lib):
    vp, i32p, c_int, c_float = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.oracle_kv_append.restype = c_int
    lib.oracle_kv_append.argtypes = [vp, vp, vp, i32p, i32p, i32p] + [c_int] * 6
    lib.oracle_chunk_prefill_attn.restype = c_int
    lib.oracle_chunk_prefill_attn.argtypes = [vp] * 4 + [i32p] * 3 + [c_int] * 7 + [c_float, vp]
    lib.oracle_chunk_prefill_attn_samples.restype = c_int
    lib.oracle_chunk_prefill_attn_samples.argtypes = (
        [vp] * 4 + [i32p] * 3 + [c_int] * 6 + [c_float, i32p, i32p, c_int, vp])
    lib.oracle_attn_row_probs.restype = c_int
    lib.oracle_attn_row_probs.argtypes = (
        [vp] * 4 + [i32p] * 3 + [c_int] * 6 + [c_float, c_int, c_int, vp])
    return lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def kv_append(k_new, v_new, kv_pages, block_table, cu, ctx, lib=None):
    """oracle_kv_append: in-place copy of the chunk's K/V rows into their page slots.

    k_new/v_new [C,Hkv,D], kv_pages [num_pages,2,Hkv,P,D]; dtype float32 or uint16 (bf16
    bits), all three the same.  kv_pages is modified in place.
    """
    lib = lib or load()
    assert kv_pages.flags["C_CONTIGUOUS"] and kv_pages.dtype == k_new.dtype == v_new.dtype
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    block_table, cu, ctx = _i32(block_table), _i32(cu), _i32(ctx)
    _, two, Hkv, P, D = kv_pages.shape
    assert two == 2 and k_new.shape[1:] == (Hkv, D) and block_table.ndim == 2
    S = len(ctx)
    assert len(cu) == S + 1 and block_table.shape[0] >= S
    rc = lib.oracle_kv_append(_p(k_new), _p(v_new), _p(kv_pages), _p(block_table), _p(cu), _p(ctx),
                              S, Hkv, D, P, block_table.shape[1], kv_pages.dtype.itemsize)
    if rc != 0:
        raise RuntimeError("oracle_kv_append failed (block table too short?)")


def _attn_args(q, k_new, v_new, kv_pages, block_table, cu, ctx):
    q, k_new, v_new = _f32(q), _f32(k_new), _f32(v_new)
    assert kv_pages.dtype == np.float32 and kv_pages.flags["C_CONTIGUOUS"]
    block_table, cu, ctx = _i32(block_table), _i32(cu), _i32(ctx)
    C, Hq, D = q.shape
    _, two, Hkv, P, D2 = kv_pages.shape
    assert two == 2 and D2 == D and k_new.shape == (C, Hkv, D) == v_new.shape
    S = len(ctx)
    assert len(cu) == S + 1 and cu[0] == 0 and cu[S] <= C and block_table.shape[0] >= S
    return q, k_new, v_new, block_table, cu, ctx, S, C, Hq, Hkv, D, P


def chunk_prefill_attn(q, k_new, v_new, kv_pages, block_table, cu, ctx, scale, lib=None):
    """oracle_chunk_prefill_attn: out [C,Hq,D] float32 for one chunk (padding rows zero)."""
    lib = lib or load()
    q, k_new, v_new, block_table, cu, ctx, S, C, Hq, Hkv, D, P = _attn_args(
        q, k_new, v_new, kv_pages, block_table, cu, ctx)
    out = np.empty((C, Hq, D), dtype=np.float32)
    rc = lib.oracle_chunk_prefill_attn(_p(q), _p(k_new), _p(v_new), _p(kv_pages), _p(block_table),
                                       _p(cu), _p(ctx), S, C, Hq, Hkv, D, P, block_table.shape[1],
                                       float(scale), _p(out))
    if rc != 0:
        raise RuntimeError("oracle_chunk_prefill_attn failed")
    return out


def chunk_prefill_attn_samples(q, k_new, v_new, kv_pages, block_table, cu, ctx, scale,
                               rows, heads, lib=None):
    """oracle_chunk_prefill_attn_samples: [n_samples, D] outputs of selected (row, head) pairs."""
    lib = lib or load()
    q, k_new, v_new, block_table, cu, ctx, S, C, Hq, Hkv, D, P = _attn_args(
        q, k_new, v_new, kv_pages, block_table, cu, ctx)
    rows, heads = _i32(rows), _i32(heads)
    assert len(rows) == len(heads) and (rows >= 0).all() and (rows < C).all()
    assert (heads >= 0).all() and (heads < Hq).all()
    out = np.empty((len(rows), D), dtype=np.float32)
    rc = lib.oracle_chunk_prefill_attn_samples(
        _p(q), _p(k_new), _p(v_new), _p(kv_pages), _p(block_table), _p(cu), _p(ctx),
        S, Hq, Hkv, D, P, block_table.shape[1], float(scale), _p(rows), _p(heads), len(rows), _p(out))
    if rc != 0:
        raise RuntimeError("oracle_chunk_prefill_attn_samples failed")
    return out


def attn_row_probs(q, k_new, v_new, kv_pages, block_table, cu, ctx, scale, row, head, lib=None):
    """oracle_attn_row_probs: the softmax weights (float64) of one (row, head)."""
    lib = lib or load()
    q, k_new, v_new, block_table, cu, ctx, S, C, Hq, Hkv, D, P = _attn_args(
        q, k_new, v_new, kv_pages, block_table, cu, ctx)
    cap = int(max(ctx[s] + cu[s + 1] - cu[s] for s in range(S)))
    probs = np.zeros(cap, dtype=np.float64)
    n = lib.oracle_attn_row_probs(_p(q), _p(k_new), _p(v_new), _p(kv_pages), _p(block_table),
                                  _p(cu), _p(ctx), S, Hq, Hkv, D, P, block_table.shape[1],
                                  float(scale), int(row), int(head), _p(probs))
    if n < 0:
        raise RuntimeError("oracle_attn_row_probs failed")
    return probs[:n]


def gather_chunk(per_req, segs, chunk_size):
    """Rows of a chunk: the token ranges of its segments laid end to end, zero padded.

    per_req[r] is an array [len_r, H, D]; returns [chunk_size, H, D] (Sec. 3.3.3: merge
    without reordering, pad the short last chunk with zeros).
    """
    first = per_req[segs[0][0]]
    rows = np.zeros((chunk_size,) + first.shape[1:], dtype=first.dtype)
    at = 0
    for req, start, n in segs:
        rows[at:at + n] = per_req[req][start:start + n]
        at += n
    return rows


def prefill(q_req, k_req, v_req, order, chunk_size, kv_pages, block_tables, scale, lib=None):
    """Chunked prefill of a scheduled batch, one chunk at a time (Sec. 3.3.3).

    q_req/k_req/v_req: per-request float32 arrays [len,H,D]; block_tables: per-request int32
    page lists; kv_pages float32 pool, updated in place.  Returns (outs, plan) with outs[r]
    [len_r,Hq,D] float32 and plan the list of chunks from the oracle packer.
    """
    lens = [len(x) for x in q_req]
    plan = packer.pack_chunks(lens, order, chunk_size)
    outs = [np.zeros_like(_f32(x)) for x in q_req]
    max_blocks = max(len(b) for b in block_tables)
    for segs in plan:
        cu, ctx = packer.chunk_arrays(segs)
        bt = np.zeros((len(segs), max_blocks), dtype=np.int32)
        for i, (req, _s, _n) in enumerate(segs):
            bt[i, :len(block_tables[req])] = block_tables[req]
        q = gather_chunk(q_req, segs, chunk_size)
        k = gather_chunk(k_req, segs, chunk_size)
        v = gather_chunk(v_req, segs, chunk_size)
        o = chunk_prefill_attn(q, k, v, kv_pages, bt, cu, ctx, scale, lib=lib)
        kv_append(_f32(k), _f32(v), kv_pages, bt, cu, ctx, lib=lib)
        for i, (req, start, n) in enumerate(segs):
            outs[req][start:start + n] = o[cu[i]:cu[i] + n]
    return outs, plan
