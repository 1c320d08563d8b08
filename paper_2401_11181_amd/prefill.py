"""Driving the C library over a scheduled batch: plan, per-chunk metadata, launches.

Plumbing only (tensor slicing, host-to-device copies of the small int32 arrays, launches through
the binding).  The arithmetic is in the HIP kernels; packing is tetri_pack_chunks in the C library.
Follows TetriInfer Sec. 3.3.3: prefill runs one fixed-size chunk at a time and the per-request
progress variable advances after each chunk.
"""
import numpy as np
import torch

from . import tetri


class ChunkedPrefill:
    """Plan + device-resident metadata of one scheduled batch, and its per-chunk launches."""

    def __init__(self, prompt_lens, order, chunk_size, num_q_heads, num_kv_heads, head_dim, num_pages,
                 req_block_tables, device="cuda:0", page_size=16):
        self.device = torch.device(device)
        self.C, self.Hq, self.Hkv, self.D = chunk_size, num_q_heads, num_kv_heads, head_dim
        self.prompt_lens = [int(x) for x in prompt_lens]
        max_blocks = max(1, max(len(t) for t in req_block_tables))
        self.max_blocks = max_blocks
        self.req_bt = np.zeros((len(req_block_tables), max_blocks), dtype=np.int32)
        for r, t in enumerate(req_block_tables):
            self.req_bt[r, :len(t)] = t
        # a1: chunk packing (C library, host)
        self.segs, self.offsets = tetri.tetri_pack_chunks(self.prompt_lens, order, chunk_size)
        self.n_chunks = len(self.offsets) - 1
        max_segs = max([1] + [int(self.offsets[i + 1] - self.offsets[i]) for i in range(self.n_chunks)])
        self.handle = tetri.Tetri(num_q_heads, num_kv_heads, head_dim, chunk_size, num_pages, max_blocks,
                                  max_segs, page_size=page_size)
        # per-chunk metadata, built on the host by the C library and uploaded once
        self.meta = []
        cus, ctxs, bts = [], [], []
        for c in range(self.n_chunks):
            segs = self.segs[self.offsets[c]:self.offsets[c + 1]]
            cu, ctx, bt = tetri.tetri_chunk_metadata(segs, self.req_bt)
            cus.append(cu), ctxs.append(ctx), bts.append(bt.reshape(-1))
        # keep every sub-array 16-byte aligned inside one upload
        parts, at = [], 0
        layout = []
        for group in (cus, ctxs, bts):
            for a in group:
                pad = (-at) % 4
                at += pad
                parts.append(np.zeros(pad, np.int32))
                parts.append(a)
                layout.append((at, len(a)))
                at += len(a)
        host = np.concatenate(parts) if parts else np.zeros(1, np.int32)
        self.meta_dev = torch.from_numpy(host).to(self.device)
        n = self.n_chunks
        for c in range(n):
            views = []
            for k in range(3):
                off, ln = layout[k * n + c]
                views.append(self.meta_dev[off:off + ln])
            self.meta.append((views[0], views[1], views[2], len(ctxs[c])))

    def chunk_segments(self, c):
        return [tuple(int(v) for v in s) for s in self.segs[self.offsets[c]:self.offsets[c + 1]]]

    def gather_chunk(self, per_req, c):
        """[C, H, D] rows of chunk c from per-request tensors (zero padded); device tensors."""
        first = per_req[self.segs[self.offsets[c]][0]]
        rows = torch.zeros((self.C,) + tuple(first.shape[1:]), dtype=first.dtype, device=self.device)
        at = 0
        for req, start, n in self.chunk_segments(c):
            rows[at:at + n] = per_req[req][start:start + n]
            at += n
        return rows

    def attn(self, c, q, k_new, v_new, kv_pages, scale, out, stream=None):
        cu, ctx, bt, S = self.meta[c]
        self.handle.tetri_chunk_prefill_attn(q, k_new, v_new, kv_pages, bt, cu, ctx, S, scale, out, stream)

    def append(self, c, k_new, v_new, kv_pages, stream=None):
        cu, ctx, bt, S = self.meta[c]
        self.handle.tetri_kv_append(k_new, v_new, kv_pages, bt, cu, ctx, S, stream)

    def attn_append(self, c, q, k_new, v_new, kv_pages, scale, out, stream=None):
        cu, ctx, bt, S = self.meta[c]
        self.handle.tetri_chunk_prefill_attn_append(q, k_new, v_new, kv_pages, bt, cu, ctx, S, scale, out, stream)

    def attn_fp8(self, c, q, k_new, v_new, kv_pages_fp8, scale, k_scale, v_scale, append, out, stream=None):
        cu, ctx, bt, S = self.meta[c]
        self.handle.tetri_chunk_prefill_attn_fp8(q, k_new, v_new, kv_pages_fp8, bt, cu, ctx, S, scale, k_scale, v_scale,
                                                 append, out, stream)

    def validate(self, c):
        cu, ctx, bt, S = self.meta[c]
        self.handle.tetri_validate_chunk(bt, cu, ctx, S)


class PrefillPipeline:
    """The whole hot path of one scheduled batch as a repeatable step, for measurement.

    step() = pack the batch into chunks and build every chunk's metadata on the host
    (tetri_plan_metadata, one C call) into pinned memory, one asynchronous upload, then for every
    chunk in order one launch that does attention and append (or two launches with fused=False;
    Sec. 3.3.3: one chunk at a time; the
    progress variable of each request is the `start` field of its next segment).
    Inputs (per-chunk q, k_new, v_new) and the page pool are resident in HBM before a step.
    With use_graph the launches of a step are replayed from a HIP graph; packing, metadata and the
    upload still run every step.
    """

    RING = 4    # pinned staging buffers in flight

    def __init__(self, prompt_lens, order, chunk_size, num_q_heads, num_kv_heads, head_dim, num_pages,
                 req_block_tables, scale, device="cuda:0", page_size=16, use_graph=False, fused=True, export=None, handle=None):
        self.device = torch.device(device)
        self.C, self.Hq, self.Hkv, self.D = chunk_size, num_q_heads, num_kv_heads, head_dim
        self.scale = float(scale)
        self.fused = fused          # one launch per chunk (attention + append) instead of two
        # KV transfer granularity of the step (Sec. 3.3.4): None = no export, "request" = one export of every
        # request after the last chunk, "chunk" = each chunk's slice exported on a second stream while the next
        # chunk is prefilled
        self.export = export
        if export not in (None, "request", "chunk"):
            raise ValueError("export must be None, 'request' or 'chunk'")
        if export and use_graph:
            raise ValueError("the export modes are launched eagerly")
        self.lens = np.ascontiguousarray(prompt_lens, dtype=np.int32)
        self.order = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
        self.max_blocks = max(1, max(len(t) for t in req_block_tables))
        self.req_bt = np.zeros((len(req_block_tables), self.max_blocks), dtype=np.int32)
        for r, t in enumerate(req_block_tables):
            self.req_bt[r, :len(t)] = t
        self.plan_segs, self.plan_offsets = tetri.tetri_pack_chunks(self.lens, self.order, chunk_size)
        self.n_chunks, self.meta_len = tetri.tetri_plan_metadata(self.lens, self.order, chunk_size, self.req_bt)
        self.meta_len = max(int(self.meta_len), 4)
        self.stage = [torch.zeros(self.meta_len, dtype=torch.int32, pin_memory=True) for _ in range(self.RING)]
        self.layout_np = np.zeros((max(self.n_chunks, 1), 4), dtype=np.int32)
        self.meta_dev = torch.zeros(self.meta_len, dtype=torch.int32, device=self.device)
        self.host_plan(0)
        self.layout = [tuple(int(x) for x in row) for row in self.layout_np[:self.n_chunks]]
        max_segs = max([1] + [l[3] for l in self.layout])
        # (several pipelines of one shape may share a handle, as long as their launches do not overlap)
        self.handle = handle or tetri.Tetri(num_q_heads, num_kv_heads, head_dim, chunk_size, num_pages, self.max_blocks,
                                            max_segs, page_size=page_size)
        self.events = [torch.cuda.Event() for _ in range(self.RING)]
        self.used = [False] * self.RING
        self.graph = None
        self.use_graph = use_graph
        self.turn = 0

    # --- inputs -------------------------------------------------------------------------------
    def bind(self, q_chunks, k_chunks, v_chunks, kv_pages, out_chunks):
        """Device tensors: q/out [n_chunks,C,Hq,D], k/v [n_chunks,C,Hkv,D], the page pool."""
        self.q, self.k, self.v, self.pool, self.out = q_chunks, k_chunks, v_chunks, kv_pages, out_chunks
        self.graph = None
        self._bind_args()
        if self.export:
            total = int(self.lens.sum())
            self.xbuf = torch.zeros(2 * self.Hkv * self.D * max(total, 1), dtype=self.pool.dtype, device=self.device)
            self.req_bt_dev = torch.from_numpy(self.req_bt).to(self.device)
            self.req_cu_dev = torch.from_numpy(np.concatenate([[0], np.cumsum(self.lens)]).astype(np.int32)).to(self.device)
            self.side = torch.cuda.Stream(device=self.device)      # default priority
            self.chunk_done = [torch.cuda.Event() for _ in range(self.n_chunks)]
            self.side_done = torch.cuda.Event()
            # a chunk's slice goes behind the slices of the chunks before it
            self.chunk_tokens = [sum(n for _r, _s, n in self.chunk_segments(c)) for c in range(self.n_chunks)]
            self.chunk_at = [2 * self.Hkv * self.D * sum(self.chunk_tokens[:c]) for c in range(self.n_chunks)]
            import ctypes
            vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
            base, esz = self.meta_dev.data_ptr(), self.xbuf.element_size()
            self._side_stream = vp(self.side.cuda_stream)
            self._chunk_export_args = []
            for c in range(self.n_chunks):
                o_cu, o_ctx, o_bt, S = self.layout[c]
                self._chunk_export_args.append((self.handle.h, vp(self.pool.data_ptr()), vp(base + 4 * o_bt), vp(base + 4 * o_cu),
                                                vp(base + 4 * o_ctx), i32(S), i64(self.chunk_tokens[c]),
                                                vp(self.xbuf.data_ptr() + esz * self.chunk_at[c]), self._side_stream))
            self._request_export_args = (self.handle.h, vp(self.pool.data_ptr()), vp(self.req_bt_dev.data_ptr()),
                                         vp(self.req_cu_dev.data_ptr()), None, i32(len(self.lens)), i64(total),
                                         vp(self.xbuf.data_ptr()))

    # --- host part of a step --------------------------------------------------------------------
    def host_plan(self, slot):
        """a1: pack, and every chunk's cu / ctx / block table into staging buffer `slot`."""
        n = tetri.tetri_plan_metadata(self.lens, self.order, self.C, self.req_bt, self.stage[slot], self.layout_np)
        if n != self.n_chunks:
            raise RuntimeError("plan changed between steps")

    # --- device part of a step ------------------------------------------------------------------
    def _bind_args(self):
        """Marshal the arguments of every launch once (ctypes objects), so that a launch is one foreign call."""
        import ctypes
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        base = self.meta_dev.data_ptr()
        self._attn_args, self._app_args = [], []
        for c in range(self.n_chunks):
            o_cu, o_ctx, o_bt, S = self.layout[c]
            q, k, v, o = (vp(t[c].data_ptr()) for t in (self.q, self.k, self.v, self.out))
            pool = vp(self.pool.data_ptr())
            bt, cu, ctx = vp(base + 4 * o_bt), vp(base + 4 * o_cu), vp(base + 4 * o_ctx)
            self._attn_args.append((self.handle.h, q, k, v, pool, bt, cu, ctx, i32(S), f32(self.scale), o))
            self._app_args.append((self.handle.h, k, v, pool, bt, cu, ctx, i32(S)))
        self._lib = tetri.lib()

    def launch_attn(self, c, stream=None):
        """One attention launch of chunk c with the metadata currently on the device."""
        rc = self._lib.tetri_chunk_prefill_attn(*self._attn_args[c], stream or tetri._stream(None))
        if rc != tetri.TETRI_OK:
            raise tetri.TetriError(rc, tetri.tetri_last_error(self.handle))

    def launch_fused(self, c, stream=None):
        """Attention and append of chunk c in one launch."""
        rc = self._lib.tetri_chunk_prefill_attn_append(*self._attn_args[c], stream or tetri._stream(None))
        if rc != tetri.TETRI_OK:
            raise tetri.TetriError(rc, tetri.tetri_last_error(self.handle))

    def launch_fused_fp8(self, c, kv_pages_fp8, k_scale, v_scale, append=1, stream=None):
        """Chunk c over a pool of FP8 codes: attention and, with append, the quantising append, in one launch."""
        import ctypes
        h, q, k, v, _pool, bt, cu, ctx, S, scale, o = self._attn_args[c]
        rc = self._lib.tetri_chunk_prefill_attn_fp8(h, q, k, v, ctypes.c_void_p(kv_pages_fp8.data_ptr()), bt, cu, ctx, S, scale,
                                                    ctypes.c_float(k_scale), ctypes.c_float(v_scale), ctypes.c_int32(append), o,
                                                    stream or tetri._stream(None))
        if rc != tetri.TETRI_OK:
            raise tetri.TetriError(rc, tetri.tetri_last_error(self.handle))

    def launch_append(self, c, stream=None):
        rc = self._lib.tetri_kv_append(*self._app_args[c], stream or tetri._stream(None))
        if rc != tetri.TETRI_OK:
            raise tetri.TetriError(rc, tetri.tetri_last_error(self.handle))

    def _launch_all(self):
        stream = tetri._stream(None)                # the current stream, looked up once per step
        for c in range(self.n_chunks):
            if self.fused:
                self.launch_fused(c, stream)
            else:
                self.launch_attn(c, stream)
                self.launch_append(c, stream)
            if self.export == "chunk":
                # the slice this chunk cached, named by the chunk's own metadata arrays
                self.chunk_done[c].record()
                self.side.wait_event(self.chunk_done[c])
                rc = self._lib.tetri_kv_export(*self._chunk_export_args[c])
                if rc != tetri.TETRI_OK:
                    raise tetri.TetriError(rc, tetri.tetri_last_error(self.handle))
        if self.export == "chunk":
            self.side_done.record(self.side)
            torch.cuda.current_stream().wait_event(self.side_done)
        elif self.export == "request":
            rc = self._lib.tetri_kv_export(*self._request_export_args, stream)
            if rc != tetri.TETRI_OK:
                raise tetri.TetriError(rc, tetri.tetri_last_error(self.handle))

    def step(self):
        slot = self.turn % self.RING
        self.turn += 1
        if self.used[slot]:
            self.events[slot].synchronize()         # the upload that last used this buffer is done
        self.host_plan(slot)
        self.meta_dev.copy_(self.stage[slot], non_blocking=True)
        self.events[slot].record()
        self.used[slot] = True
        if self.use_graph:
            if self.graph is None:                  # one graph: the launches read meta_dev, whose address is fixed
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    self._launch_all()
                self.graph = g
            self.graph.replay()
        else:
            self._launch_all()

    # --- the plan -------------------------------------------------------------------------------
    def chunk_segments(self, c):
        return [tuple(int(v) for v in s) for s in self.plan_segs[self.plan_offsets[c]:self.plan_offsets[c + 1]]]
