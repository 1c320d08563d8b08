"""Writes tests/golden/*.txt from the CPU oracle alone (run from the repository root:
`python tests/golden/make_golden.py`).

The paper prints no numeric example of this path, so these are not the paper's values: they freeze what the
pinned oracle computes today for small seeded inputs, so that a later change of the oracle's arithmetic
cannot pass unnoticed (tests/test_golden.py), and they give the GPU tests expected values that were
stored before the GPU ran.  Nothing here calls the HIP library.
"""
import os
import sys

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

from oracle import decode, kv_transfer, tetri_oracle  # noqa: E402
from paper_2401_11181_amd import synth  # noqa: E402
from helpers import oracle_inputs  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
# (row, head) pairs of the tiny configuration whose outputs are stored: first and last token, chunk
# boundaries (63 | 64), a mid-page position
SAMPLES = [(0, 0), (1, 3), (15, 1), (16, 2), (63, 0), (64, 3), (100, 1), (191, 2), (192, 0), (255, 3)]


def tiny_rows():
    """Config 'tiny' (256 tokens, 4 chunks of 64, 4 heads x 64, seed 1001), inputs rounded to bf16."""
    w = synth.workload("tiny")
    qs, ks, vs, tables, pool = oracle_inputs(w, torch.bfloat16)
    outs, _ = tetri_oracle.prefill(qs, ks, vs, w.order, w.chunk_size, pool, tables, w.scale)
    return np.stack([outs[0][r, h, :8] for r, h in SAMPLES])


def packed_decode_rows():
    """A ragged GQA batch (seed 61): decode outputs of every request's last token, first 8 elements."""
    w = synth.small("golden-decode", [37, 5, 64, 1, 23], 32, 4, 2, 64, seed=61)
    qs, ks, vs, tables, pool = oracle_inputs(w, torch.bfloat16)
    tetri_oracle.prefill(qs, ks, vs, w.order, w.chunk_size, pool, tables, w.scale)
    mb = max(len(t) for t in tables)
    bt = np.zeros((len(tables), mb), dtype=np.int32)
    for r, t in enumerate(tables):
        bt[r, :len(t)] = t
    ctx = np.array([n - 1 for n in w.prompt_lens])
    q = np.stack([qs[r][ctx[r]] for r in range(len(ctx))])
    k = np.stack([ks[r][ctx[r]] for r in range(len(ctx))])
    v = np.stack([vs[r][ctx[r]] for r in range(len(ctx))])
    out = decode.decode_attn(q, k, v, pool, bt, ctx, w.scale)
    cu = np.concatenate([[0], np.cumsum(w.prompt_lens)])
    buf = kv_transfer.kv_export(pool, bt, cu)
    return out[:, :, :8].reshape(-1, 8), np.array([buf.size, float(np.abs(buf.astype(np.float64)).sum())])


def main():
    np.savetxt(os.path.join(HERE, "tiny_prefill_rows.txt"), tiny_rows(), fmt="%.9e",
               header="oracle prefill outputs out[row][head][0:8] of config tiny for (row, head) in " + repr(SAMPLES))
    rows, xfer = packed_decode_rows()
    np.savetxt(os.path.join(HERE, "ragged_decode_rows.txt"), rows, fmt="%.9e",
               header="oracle decode outputs out[request][head][0:8], workload golden-decode (lengths 37 5 64 1 23, seed 61)")
    np.savetxt(os.path.join(HERE, "ragged_export_sum.txt"), xfer[None], fmt="%.9e",
               header="request-level export of the same cache: number of elements, sum of absolute values")


if __name__ == "__main__":
    main()
