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

    def validate(self, c):
        cu, ctx, bt, S = self.meta[c]
        self.handle.tetri_validate_chunk(bt, cu, ctx, S)

    def pairs(self, c):
        """Unmasked (query, key) pairs per query head of chunk c: sum n*L + n(n+1)/2."""
        return sum(n * start + n * (n + 1) // 2 for _req, start, n in self.chunk_segments(c))

    def flops(self, c):
        """Algorithmic attention flops of chunk c: 4 * D * Hq * pairs (QK^T and PV, masked pairs count zero)."""
        return 4 * self.D * self.Hq * self.pairs(c)


class PrefillPipeline:
    """The whole hot path of one scheduled batch as a repeatable step, for measurement.

    step() = pack the batch into chunks on the host (tetri_pack_chunks), build every chunk's
    metadata (tetri_chunk_metadata) into pinned host memory, one asynchronous upload, then for
    every chunk in order one attention launch and one append launch (Sec. 3.3.3: one chunk at a
    time; the progress variable of each request is the `start` field of its next segment).
    Inputs (per-chunk q, k_new, v_new) and the page pool are resident in HBM before a step.
    With use_graph the upload and the launches of a step are replayed from a HIP graph; packing
    and metadata still run on the host every step.
    """

    RING = 4    # staging buffers in flight

    def __init__(self, prompt_lens, order, chunk_size, num_q_heads, num_kv_heads, head_dim, num_pages,
                 req_block_tables, scale, device="cuda:0", page_size=16, use_graph=False):
        self.device = torch.device(device)
        self.C, self.Hq, self.Hkv, self.D = chunk_size, num_q_heads, num_kv_heads, head_dim
        self.scale = float(scale)
        self.lens = np.ascontiguousarray(prompt_lens, dtype=np.int32)
        self.order = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
        self.max_blocks = max(1, max(len(t) for t in req_block_tables))
        self.req_bt = np.zeros((len(req_block_tables), self.max_blocks), dtype=np.int32)
        for r, t in enumerate(req_block_tables):
            self.req_bt[r, :len(t)] = t
        segs, offsets = tetri.tetri_pack_chunks(self.lens, self.order, chunk_size)
        self.n_chunks = len(offsets) - 1
        self.seg_counts = [int(offsets[c + 1] - offsets[c]) for c in range(self.n_chunks)]
        self.max_segs = max([1] + self.seg_counts)
        self.segs_buf = np.zeros((len(segs) + 1, 3), dtype=np.int32)
        self.offs_buf = np.zeros(self.n_chunks + 1, dtype=np.int32)
        self.plan_segs = segs.copy()
        self.plan_offsets = offsets.copy()
        self.handle = tetri.Tetri(num_q_heads, num_kv_heads, head_dim, chunk_size, num_pages, self.max_blocks,
                                  self.max_segs, page_size=page_size)
        # fixed layout of the metadata block: per chunk cu | ctx | block_table, each 16-byte aligned
        def up4(x):
            return (x + 3) // 4 * 4
        self.layout, at = [], 0
        for c in range(self.n_chunks):
            S = self.seg_counts[c]
            o_cu, at = at, at + up4(S + 1)
            o_ctx, at = at, at + up4(S)
            o_bt, at = at, at + up4(S * self.max_blocks)
            self.layout.append((o_cu, o_ctx, o_bt, S))
        self.meta_len = max(at, 4)
        self.stage = [torch.zeros(self.meta_len, dtype=torch.int32, pin_memory=True) for _ in range(self.RING)]
        self.stage_np = [t.numpy() for t in self.stage]
        self.meta_dev = torch.zeros(self.meta_len, dtype=torch.int32, device=self.device)
        self.events = [None] * self.RING
        self.graphs = [None] * self.RING
        self.use_graph = use_graph
        self.turn = 0
        self._lib = tetri.lib()
        self._ptrs = None

    # --- inputs -------------------------------------------------------------------------------
    def bind(self, q_chunks, k_chunks, v_chunks, kv_pages, out_chunks):
        """Device tensors: q/out [n_chunks,C,Hq,D], k/v [n_chunks,C,Hkv,D], the page pool."""
        self.q, self.k, self.v, self.pool, self.out = q_chunks, k_chunks, v_chunks, kv_pages, out_chunks
        self.graphs = [None] * self.RING

    # --- host part of a step --------------------------------------------------------------------
    def host_plan(self, slot):
        """a1: pack; then every chunk's cu / ctx / block table into staging buffer `slot`."""
        import ctypes
        L = self._lib
        n_segs = ctypes.c_int32(0)
        n_order = len(self.lens) if self.order is None else len(self.order)
        n = L.tetri_pack_chunks(tetri._ptr(self.lens), len(self.lens), tetri._ptr(self.order), n_order, self.C,
                                tetri._ptr(self.segs_buf), len(self.segs_buf), tetri._ptr(self.offs_buf),
                                self.n_chunks, ctypes.byref(n_segs))
        if n != self.n_chunks:
            raise tetri.TetriError(n, tetri.tetri_last_error())
        base = self.stage[slot].data_ptr()
        segs_ptr = self.segs_buf.ctypes.data
        rbt = tetri._ptr(self.req_bt)
        for c in range(self.n_chunks):
            o_cu, o_ctx, o_bt, S = self.layout[c]
            rc = L.tetri_chunk_metadata(ctypes.c_void_p(segs_ptr + 12 * int(self.offs_buf[c])), S, rbt,
                                        self.req_bt.shape[0], self.max_blocks,
                                        ctypes.c_void_p(base + 4 * o_cu), ctypes.c_void_p(base + 4 * o_ctx),
                                        ctypes.c_void_p(base + 4 * o_bt))
            if rc != tetri.TETRI_OK:
                raise tetri.TetriError(rc, tetri.tetri_last_error())

    # --- device part of a step ------------------------------------------------------------------
    def _launch_all(self, slot, timing=None):
        self.meta_dev.copy_(self.stage[slot], non_blocking=True)
        base = self.meta_dev.data_ptr()
        h = self.handle
        for c in range(self.n_chunks):
            o_cu, o_ctx, o_bt, S = self.layout[c]
            cu, ctx, bt = base + 4 * o_cu, base + 4 * o_ctx, base + 4 * o_bt
            if timing is not None:
                timing[c][0].record()
            h.tetri_chunk_prefill_attn(self.q[c], self.k[c], self.v[c], self.pool, bt, cu, ctx, S, self.scale,
                                       self.out[c])
            if timing is not None:
                timing[c][1].record()
            h.tetri_kv_append(self.k[c], self.v[c], self.pool, bt, cu, ctx, S)
            if timing is not None:
                timing[c][2].record()

    def step(self, timing=None):
        slot = self.turn % self.RING
        self.turn += 1
        if self.events[slot] is not None:
            self.events[slot].synchronize()         # the upload that last used this buffer is done
        self.host_plan(slot)
        if self.use_graph and timing is None:
            if self.graphs[slot] is None:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    self._launch_all(slot)
                self.graphs[slot] = g
            self.graphs[slot].replay()
        else:
            self._launch_all(slot, timing)
        ev = torch.cuda.Event()
        ev.record()
        self.events[slot] = ev

    # --- bookkeeping ----------------------------------------------------------------------------
    def chunk_segments(self, c):
        return [tuple(int(v) for v in s) for s in self.plan_segs[self.plan_offsets[c]:self.plan_offsets[c + 1]]]

    def pairs(self, c):
        return sum(n * start + n * (n + 1) // 2 for _req, start, n in self.chunk_segments(c))

    def flops(self, c):
        return 4 * self.D * self.Hq * self.pairs(c)

    def attn_bytes(self, c):
        """Algorithmic HBM bytes of one attention launch: Q in + out, K and V once, block table."""
        segs = self.chunk_segments(c)
        n = sum(x[2] for x in segs)
        kv = sum((start + ln) * self.Hkv * self.D * 2 * 2 for _r, start, ln in segs)
        bt = sum(-(-start // 16) * 4 for _r, start, _ln in segs)
        return 2 * n * self.Hq * self.D * 2 + kv + bt

    def append_bytes(self, c):
        n = sum(x[2] for x in self.chunk_segments(c))
        return 2 * 2 * n * self.Hkv * self.D * 2
