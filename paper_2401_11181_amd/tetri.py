"""Thin Python binding of libtetri (argument marshalling only).

Every function has the name of the C entry point it forwards to (see include/tetri.h).
PyTorch supplies device memory and streams; no step of the path runs in Python or on the CPU.
If the HIP library is missing this module fails to load it with an error: there is no fallback.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# TETRI_LIB selects another build of the same library (used when comparing kernel builds)
LIB_PATH = os.environ.get("TETRI_LIB") or os.path.join(_HERE, "libtetri.so")

TETRI_OK = 0
TETRI_ERR_INVALID_ARG = -1
TETRI_ERR_UNSUPPORTED = -2
TETRI_ERR_HIP = -3
TETRI_ERR_NOMEM = -4
TETRI_BF16 = 1


class TetriError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("tetri status %d: %s" % (status, message))
        self.status = status


class Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "num_q_heads", "num_kv_heads", "head_dim", "page_size", "chunk_size", "num_pages",
        "max_blocks_per_seq", "max_segs_per_chunk", "dtype")]


class Segment(ctypes.Structure):
    _fields_ = [("req", ctypes.c_int32), ("start", ctypes.c_int32), ("len", ctypes.c_int32)]


_lib = None


def lib():
    """The loaded C library (loads it on first use; raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libtetri.so is not built: run `python -m paper_2401_11181_amd.build` "
                              "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        L.tetri_abi_version.restype = i32
        L.tetri_abi_version.argtypes = []
        L.tetri_create.restype = i32
        L.tetri_create.argtypes = [ctypes.POINTER(Config), ctypes.POINTER(vp)]
        L.tetri_destroy.restype = None
        L.tetri_destroy.argtypes = [vp]
        L.tetri_last_error.restype = ctypes.c_char_p
        L.tetri_last_error.argtypes = [vp]
        L.tetri_pack_chunks.restype = i32
        L.tetri_pack_chunks.argtypes = [vp, i32, vp, i32, i32, vp, i32, vp, i32, ctypes.POINTER(i32)]
        L.tetri_schedule.restype = i32
        L.tetri_schedule.argtypes = [vp, i32, i32, i32, vp]
        L.tetri_chunk_metadata.restype = i32
        L.tetri_chunk_metadata.argtypes = [vp, i32, vp, i32, i32, vp, vp, vp]
        L.tetri_plan_metadata.restype = i32
        L.tetri_plan_metadata.argtypes = [vp, i32, vp, i32, i32, vp, i32, vp, ctypes.c_int64, vp, i32,
                                          ctypes.POINTER(ctypes.c_int64)]
        L.tetri_kv_append.restype = i32
        L.tetri_kv_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.tetri_chunk_prefill_attn.restype = i32
        L.tetri_chunk_prefill_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
        L.tetri_chunk_prefill_attn_append.restype = i32
        L.tetri_chunk_prefill_attn_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
        L.tetri_decode_attn.restype = i32
        L.tetri_decode_attn.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp]
        L.tetri_decode_attn_static.restype = i32
        L.tetri_decode_attn_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp]
        L.tetri_decode_attn_append.restype = i32
        L.tetri_decode_attn_append.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp]
        L.tetri_kv_export_fp8.restype = i32
        L.tetri_kv_export_fp8.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.c_int64, f32, f32, vp, vp]
        L.tetri_kv_import_fp8.restype = i32
        L.tetri_kv_import_fp8.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.c_int64, vp, vp]
        L.tetri_decode_attn_fp8.restype = i32
        L.tetri_decode_attn_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, f32, f32, i32, vp, vp]
        L.tetri_chunk_prefill_attn_fp8.restype = i32
        L.tetri_chunk_prefill_attn_fp8.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, f32, f32, i32, vp, vp]
        L.tetri_kv_export.restype = i32
        L.tetri_kv_export.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.c_int64, vp, vp]
        L.tetri_kv_import.restype = i32
        L.tetri_kv_import.argtypes = [vp, vp, vp, vp, vp, i32, ctypes.c_int64, vp, vp]
        L.tetri_validate_chunk.restype = i32
        L.tetri_validate_chunk.argtypes = [vp, vp, vp, vp, i32, vp]
        L.tetri_set_option.restype = i32
        L.tetri_set_option.argtypes = [vp, ctypes.c_char_p, i32]
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, torch.Tensor):
        return ctypes.c_void_p(t.data_ptr())
    if isinstance(t, np.ndarray):
        return t.ctypes.data_as(ctypes.c_void_p)
    return ctypes.c_void_p(int(t))


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def tetri_abi_version():
    return lib().tetri_abi_version()


def tetri_last_error(handle=None):
    return lib().tetri_last_error(handle.h if handle is not None else None).decode()


def tetri_pack_chunks(prompt_lens, order, chunk_size):
    """tetri_pack_chunks (host).  Returns (segs, offsets): segs int32 [n_segs,3] = (req,start,len),
    offsets int32 [n_chunks+1]."""
    L = lib()
    lens = np.ascontiguousarray(prompt_lens, dtype=np.int32)
    ordr = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
    n_order = len(lens) if ordr is None else len(ordr)
    n_segs = ctypes.c_int32(0)
    n_chunks = L.tetri_pack_chunks(_ptr(lens), len(lens), _ptr(ordr), n_order, int(chunk_size),
                                   None, 0, None, 0, ctypes.byref(n_segs))
    if n_chunks < 0:
        raise TetriError(n_chunks, tetri_last_error())
    segs = np.zeros((max(n_segs.value, 1), 3), dtype=np.int32)
    offsets = np.zeros(n_chunks + 1, dtype=np.int32)
    rc = L.tetri_pack_chunks(_ptr(lens), len(lens), _ptr(ordr), n_order, int(chunk_size),
                             _ptr(segs), n_segs.value, _ptr(offsets), n_chunks, ctypes.byref(n_segs))
    if rc < 0:
        raise TetriError(rc, tetri_last_error())
    return segs[:n_segs.value], offsets


TETRI_FCFS, TETRI_SJF, TETRI_LJF = 0, 1, 2


def tetri_schedule(prompt_lens, policy, sched_batch):
    """tetri_schedule (host).  Returns the scheduled order (int32 array)."""
    lens = np.ascontiguousarray(prompt_lens, dtype=np.int32)
    order = np.zeros(len(lens), dtype=np.int32)
    rc = lib().tetri_schedule(_ptr(lens), len(lens), int(policy), int(sched_batch), _ptr(order))
    if rc != TETRI_OK:
        raise TetriError(rc, tetri_last_error())
    return order


def tetri_chunk_metadata(segs, req_block_tables):
    """tetri_chunk_metadata (host).  segs int32 [S,3]; req_block_tables int32 [n_prompts,max_blocks].
    Returns host arrays (cu [S+1], ctx [S], block_table [S,max_blocks])."""
    segs = np.ascontiguousarray(segs, dtype=np.int32)
    rbt = np.ascontiguousarray(req_block_tables, dtype=np.int32)
    S, mb = len(segs), rbt.shape[1]
    cu = np.zeros(S + 1, dtype=np.int32)
    ctx = np.zeros(S, dtype=np.int32)
    bt = np.zeros((S, mb), dtype=np.int32)
    rc = lib().tetri_chunk_metadata(_ptr(segs), S, _ptr(rbt), rbt.shape[0], mb, _ptr(cu), _ptr(ctx), _ptr(bt))
    if rc != TETRI_OK:
        raise TetriError(rc, tetri_last_error())
    return cu, ctx, bt


def tetri_plan_metadata(prompt_lens, order, chunk_size, req_block_tables, meta_out=None, layout_out=None):
    """tetri_plan_metadata (host).  Without buffers: returns (n_chunks, meta_len).  With meta_out (int32
    array / pinned tensor) and layout_out (int32 [n_chunks,4]): fills them and returns n_chunks."""
    L = lib()
    lens = np.ascontiguousarray(prompt_lens, dtype=np.int32)
    ordr = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
    rbt = np.ascontiguousarray(req_block_tables, dtype=np.int32)
    n_order = len(lens) if ordr is None else len(ordr)
    meta_len = ctypes.c_int64(0)
    if meta_out is None:
        n = L.tetri_plan_metadata(_ptr(lens), len(lens), _ptr(ordr), n_order, int(chunk_size), _ptr(rbt),
                                  rbt.shape[1], None, 0, None, 0, ctypes.byref(meta_len))
        if n < 0:
            raise TetriError(n, tetri_last_error())
        return n, meta_len.value
    n = L.tetri_plan_metadata(_ptr(lens), len(lens), _ptr(ordr), n_order, int(chunk_size), _ptr(rbt),
                              rbt.shape[1], _ptr(meta_out), meta_out.numel() if isinstance(meta_out, torch.Tensor)
                              else meta_out.size, _ptr(layout_out), layout_out.shape[0], ctypes.byref(meta_len))
    if n < 0:
        raise TetriError(n, tetri_last_error())
    return n


class Tetri:
    """A tetri_ctx handle (tetri_create / tetri_destroy)."""

    def __init__(self, num_q_heads, num_kv_heads, head_dim, chunk_size, num_pages, max_blocks_per_seq,
                 max_segs_per_chunk, page_size=16, dtype=TETRI_BF16):
        self.h = None
        self.cfg = Config(num_q_heads, num_kv_heads, head_dim, page_size, chunk_size, num_pages,
                          max_blocks_per_seq, max_segs_per_chunk, dtype)
        h = ctypes.c_void_p()
        rc = lib().tetri_create(ctypes.byref(self.cfg), ctypes.byref(h))
        if rc != TETRI_OK:
            raise TetriError(rc, tetri_last_error())
        self.h = h

    def close(self):
        if self.h is not None:
            lib().tetri_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != TETRI_OK:
            raise TetriError(rc, tetri_last_error(self))

    def tetri_set_option(self, key, value):
        self._check(lib().tetri_set_option(self.h, key.encode(), int(value)))

    def tetri_kv_append(self, k_new, v_new, kv_pages, block_table, cu_chunk_q_lens, ctx_lens, num_segs,
                        stream=None):
        self._check(lib().tetri_kv_append(self.h, _ptr(k_new), _ptr(v_new), _ptr(kv_pages), _ptr(block_table),
                                          _ptr(cu_chunk_q_lens), _ptr(ctx_lens), int(num_segs), _stream(stream)))

    def tetri_chunk_prefill_attn(self, q, k_new, v_new, kv_pages, block_table, cu_chunk_q_lens, ctx_lens,
                                 num_segs, scale, out, stream=None):
        self._check(lib().tetri_chunk_prefill_attn(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages),
                                                   _ptr(block_table), _ptr(cu_chunk_q_lens), _ptr(ctx_lens),
                                                   int(num_segs), float(scale), _ptr(out), _stream(stream)))

    def tetri_chunk_prefill_attn_append(self, q, k_new, v_new, kv_pages, block_table, cu_chunk_q_lens, ctx_lens,
                                        num_segs, scale, out, stream=None):
        self._check(lib().tetri_chunk_prefill_attn_append(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages),
                                                          _ptr(block_table), _ptr(cu_chunk_q_lens), _ptr(ctx_lens),
                                                          int(num_segs), float(scale), _ptr(out), _stream(stream)))

    def tetri_decode_attn(self, q, k_new, v_new, kv_pages, block_table, ctx_lens, num_reqs, max_ctx_len, scale, out,
                          stream=None):
        self._check(lib().tetri_decode_attn(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages),
                                            _ptr(block_table), _ptr(ctx_lens), int(num_reqs), int(max_ctx_len),
                                            float(scale), _ptr(out), _stream(stream)))

    def tetri_decode_attn_static(self, q, k_new, v_new, kv_pages, block_table, ctx_lens, num_reqs, max_ctx_len, scale, out,
                                 stream=None):
        self._check(lib().tetri_decode_attn_static(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages),
                                                   _ptr(block_table), _ptr(ctx_lens), int(num_reqs), int(max_ctx_len),
                                                   float(scale), _ptr(out), _stream(stream)))

    def tetri_decode_attn_append(self, q, k_new, v_new, kv_pages, block_table, ctx_lens, num_reqs, max_ctx_len, scale,
                                 out, stream=None):
        self._check(lib().tetri_decode_attn_append(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages),
                                                   _ptr(block_table), _ptr(ctx_lens), int(num_reqs), int(max_ctx_len),
                                                   float(scale), _ptr(out), _stream(stream)))

    def tetri_kv_export_fp8(self, kv_pages, block_table, cu_tokens, first_tokens, num_reqs, total_tokens, k_scale,
                            v_scale, buf, stream=None):
        self._check(lib().tetri_kv_export_fp8(self.h, _ptr(kv_pages), _ptr(block_table), _ptr(cu_tokens),
                                              _ptr(first_tokens), int(num_reqs), int(total_tokens), float(k_scale),
                                              float(v_scale), _ptr(buf), _stream(stream)))

    def tetri_kv_import_fp8(self, buf, block_table, cu_tokens, first_tokens, num_reqs, total_tokens, kv_pages_fp8,
                            stream=None):
        self._check(lib().tetri_kv_import_fp8(self.h, _ptr(buf), _ptr(block_table), _ptr(cu_tokens),
                                              _ptr(first_tokens), int(num_reqs), int(total_tokens), _ptr(kv_pages_fp8),
                                              _stream(stream)))

    def tetri_decode_attn_fp8(self, q, k_new, v_new, kv_pages_fp8, block_table, ctx_lens, num_reqs, max_ctx_len, scale,
                              k_scale, v_scale, append, out, stream=None):
        self._check(lib().tetri_decode_attn_fp8(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages_fp8),
                                                _ptr(block_table), _ptr(ctx_lens), int(num_reqs), int(max_ctx_len),
                                                float(scale), float(k_scale), float(v_scale), int(append), _ptr(out),
                                                _stream(stream)))

    def tetri_chunk_prefill_attn_fp8(self, q, k_new, v_new, kv_pages_fp8, block_table, cu_chunk_q_lens, ctx_lens, num_segs,
                                     scale, k_scale, v_scale, append, out, stream=None):
        self._check(lib().tetri_chunk_prefill_attn_fp8(self.h, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kv_pages_fp8),
                                                       _ptr(block_table), _ptr(cu_chunk_q_lens), _ptr(ctx_lens),
                                                       int(num_segs), float(scale), float(k_scale), float(v_scale),
                                                       int(append), _ptr(out), _stream(stream)))

    def tetri_kv_export(self, kv_pages, block_table, cu_tokens, first_tokens, num_reqs, total_tokens, buf,
                        stream=None):
        self._check(lib().tetri_kv_export(self.h, _ptr(kv_pages), _ptr(block_table), _ptr(cu_tokens),
                                          _ptr(first_tokens), int(num_reqs), int(total_tokens), _ptr(buf),
                                          _stream(stream)))

    def tetri_kv_import(self, buf, block_table, cu_tokens, first_tokens, num_reqs, total_tokens, kv_pages,
                        stream=None):
        self._check(lib().tetri_kv_import(self.h, _ptr(buf), _ptr(block_table), _ptr(cu_tokens),
                                          _ptr(first_tokens), int(num_reqs), int(total_tokens), _ptr(kv_pages),
                                          _stream(stream)))

    def tetri_validate_chunk(self, block_table, cu_chunk_q_lens, ctx_lens, num_segs, stream=None):
        self._check(lib().tetri_validate_chunk(self.h, _ptr(block_table), _ptr(cu_chunk_q_lens), _ptr(ctx_lens),
                                               int(num_segs), _stream(stream)))
