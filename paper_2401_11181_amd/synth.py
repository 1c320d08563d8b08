"""Seeded synthetic workloads for chunked-prefill attention (inputs only).

This module holds no arithmetic of the method: it only draws random prompts, Q/K/V values
and page placements.  Both the GPU path and the CPU oracle are fed from here.

The workloads stand in for the ShareGPT-derived traffic of TetriInfer's evaluation (Sec. 5),
which is not available offline: only its shape is kept (light prefills of tens of tokens,
heavy prefills of hundreds to thousands of tokens, lengths spread over orders of magnitude;
Sec. 2.2 and Fig. 1), with ChunkSize 512 for the OPT-13B shape (Sec. 3.3.3).
"""
from dataclasses import dataclass, field, replace
import math

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    prompt_lens: list
    chunk_size: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    std: float            # standard deviation of Q, K and V entries
    scale: float          # softmax scale
    seed: int
    order: list = field(default_factory=list)   # scheduled order of the requests (FCFS)

    def __post_init__(self):
        if not self.order:
            self.order = list(range(len(self.prompt_lens)))

    @property
    def pages_needed(self):
        return sum(-(-n // self.page_size) for n in self.prompt_lens)


def _lognormal_lens(rng, total_tokens):
    """Prompt lengths clamp(rint(exp(N(4.5, 0.8))), 16, 512), drawn until total_tokens would overflow."""
    lens, tot = [], 0
    while True:
        n = int(min(512, max(16, np.rint(np.exp(rng.normal(4.5, 0.8))))))
        if tot + n > total_tokens:
            break
        lens.append(n)
        tot += n
    return lens


def workload(name):
    """The five benchmark configurations (seeds 1001..1005)."""
    if name == "tiny":
        return Workload("tiny", [256], 64, 4, 4, 64, 16, 32, 1.0, 1.0 / 8.0, 1001)
    if name == "opt13b":
        return Workload("opt13b", [2048], 512, 40, 40, 128, 16, 1024,
                        1.0 / math.sqrt(128), 1.0 / math.sqrt(128), 1002)
    if name == "packed":
        rng = np.random.default_rng(1003)
        lens = _lognormal_lens(rng, 64 * 512)
        w = Workload("packed", lens, 512, 40, 40, 128, 16, 0,
                     1.0 / math.sqrt(128), 1.0 / math.sqrt(128), 1003)
        w.num_pages = w.pages_needed + 64
        return w
    if name == "heavy":
        return Workload("heavy", [16384], 512, 40, 40, 128, 16, 32768,
                        1.0 / math.sqrt(128), 1.0 / math.sqrt(128), 1004)
    if name == "gqa":
        rng = np.random.default_rng(1005)
        lens = [int(x) for x in rng.integers(4096, 32768, size=8, endpoint=True)]
        w = Workload("gqa", lens, 2048, 32, 8, 128, 16, 0,
                     1.0 / math.sqrt(128), 1.0 / math.sqrt(128), 1005)
        w.num_pages = w.pages_needed
        return w
    raise KeyError(name)


def sharp(w, **kw):
    """Parity-only variant: Q, K, V ~ N(0,1) so that scores are O(1) and softmax is peaked."""
    return replace(w, name=w.name + "-sharp", std=1.0, scale=1.0 / math.sqrt(w.head_dim), **kw)


def small(name, prompt_lens, chunk_size, hq, hkv, d, seed, page_size=16, slack_pages=7, std=1.0,
          scale=None, order=None):
    """An ad-hoc small workload for parity and edge-case tests."""
    w = Workload(name, list(prompt_lens), chunk_size, hq, hkv, d, page_size, 0, std,
                 scale if scale is not None else 1.0 / math.sqrt(d), seed, list(order or []))
    w.num_pages = w.pages_needed + slack_pages
    return w


def request_qkv(w, req, dtype=torch.bfloat16):
    """Q [n,Hq,D], K and V [n,Hkv,D] of one request: N(0, std^2) in float32, rounded once to dtype."""
    rng = np.random.default_rng([w.seed, 7, req])
    n = w.prompt_lens[req]
    out = []
    for heads in (w.num_q_heads, w.num_kv_heads, w.num_kv_heads):
        a = rng.standard_normal((n, heads, w.head_dim), dtype=np.float32)
        a *= np.float32(w.std)
        out.append(torch.from_numpy(a).to(dtype))
    return tuple(out)


def place_pages(w):
    """Random placement without repeats: per-request int32 arrays of physical page ids."""
    rng = np.random.default_rng([w.seed, 11])
    if w.pages_needed > w.num_pages:
        raise ValueError("pool too small")
    perm = rng.permutation(w.num_pages)[:w.pages_needed].astype(np.int32)
    tables, at = [], 0
    for n in w.prompt_lens:
        k = -(-n // w.page_size)
        tables.append(perm[at:at + k].copy())
        at += k
    return tables


def pool_sentinel(shape, dtype=torch.bfloat16, device="cpu"):
    """A page pool prefilled with a fixed finite bit pattern (to detect stray writes)."""
    t = torch.empty(shape, dtype=torch.int16, device=device)
    t.fill_(0x3B5A)                       # bf16 0x3B5A ~ 3.3e-3, finite
    return t.view(dtype) if dtype != torch.int16 else t


def random_kv_codes(shape, seed, k_scale, v_scale, std=1.0):
    """A pool [num_pages,2,Hkv,P,D] of FP8 E4M3 codes (uint8) whose values times the tensor's scale are about
    N(0, std^2): normal draws divided by the scale, turned into codes by torch's float8_e4m3fn conversion (an
    input generator: both sides read the codes, neither the draws)."""
    g = torch.Generator().manual_seed(int(seed))
    x = torch.randn(shape, generator=g, dtype=torch.float32) * std
    x[:, 0] /= k_scale
    x[:, 1] /= v_scale
    return x.clamp_(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
