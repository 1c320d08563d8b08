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
