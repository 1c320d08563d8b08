"""Shared test plumbing: turning a synthetic workload into oracle inputs (no method arithmetic)."""
import numpy as np
import torch

from paper_2401_11181_amd import synth


def oracle_inputs(w, dtype=torch.bfloat16):
    """Per-request float32 Q/K/V (rounded once to dtype), block tables and an empty float32 pool."""
    qs, ks, vs = [], [], []
    for r in range(len(w.prompt_lens)):
        q, k, v = synth.request_qkv(w, r, dtype)
        qs.append(q.float().numpy())
        ks.append(k.float().numpy())
        vs.append(v.float().numpy())
    tables = synth.place_pages(w)
    pool = np.full((w.num_pages, 2, w.num_kv_heads, w.page_size, w.head_dim), 777.0, dtype=np.float32)
    return qs, ks, vs, tables, pool


def brute_force_attention(q, k, v, scale):
    """Unchunked, unpaged causal attention of one request in float64 with the full score matrix.

    q [n,Hq,D], k/v [n,Hkv,D].  An independent statement of the definition, written with
    matrix primitives rather than the oracle's scalar loops.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    n, hq, _ = q.shape
    g = hq // k.shape[1]
    out = np.zeros_like(q)
    future = np.triu(np.ones((n, n), dtype=bool), 1)
    for h in range(hq):
        s = scale * (q[:, h, :] @ k[:, h // g, :].T)
        s[future] = -np.inf
        w = np.exp(s - s.max(axis=1, keepdims=True))
        w /= w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ v[:, h // g, :]
    return out
