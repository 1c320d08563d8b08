"""Host-side checks of the C ABI that need no GPU: exported symbols, the packer, error conventions."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import packer as opacker
from paper_2401_11181_amd import synth, tetri

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tetri.h")).read()
    return sorted(set(re.findall(r"TETRI_API[^;(]*?\b(tetri_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 10 and "tetri_chunk_prefill_attn" in names and "tetri_kv_append" in names
    lib = tetri.lib()
    for n in names:
        assert hasattr(lib, n), "libtetri.so does not export " + n
    assert tetri.tetri_abi_version() == 1


def test_library_exports_nothing_else():
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", tetri.LIB_PATH], capture_output=True, text=True).stdout
    exported = sorted(l.split()[-1] for l in out.splitlines() if " T " in l)
    assert exported == declared_functions()


def lib_plan(lens, order, C):
    segs, offs = tetri.tetri_pack_chunks(lens, order, C)
    return [[tuple(int(x) for x in s) for s in segs[offs[c]:offs[c + 1]]] for c in range(len(offs) - 1)]


def test_packer_hand_example():
    assert lib_plan([3, 5, 2], None, 4) == [[(0, 0, 3), (1, 0, 1)], [(1, 1, 4)], [(2, 0, 2)]]
    assert lib_plan([3, 5, 2], [2, 0, 1], 4) == [[(2, 0, 2), (0, 0, 2)], [(0, 2, 1), (1, 0, 3)], [(1, 3, 2)]]
    assert lib_plan([0, 0], None, 4) == []
    assert lib_plan([], None, 4) == []


def test_packer_matches_oracle_packer_on_random_batches():
    rng = np.random.default_rng(42)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        lens = [int(x) for x in rng.integers(0, 70, size=n)]
        order = [int(x) for x in rng.permutation(n)[: int(rng.integers(1, n + 1))]]
        C = int(rng.integers(1, 40))
        assert lib_plan(lens, order, C) == [list(c) for c in opacker.pack_chunks(lens, order, C)]
    for name in ("packed", "gqa", "heavy"):
        w = synth.workload(name)
        assert lib_plan(w.prompt_lens, w.order, w.chunk_size) == \
            [list(c) for c in opacker.pack_chunks(w.prompt_lens, w.order, w.chunk_size)]


def test_packer_errors():
    for lens, order, C, code in [([3, -1], None, 4, tetri.TETRI_ERR_INVALID_ARG),
                                 ([3, 2], [0, 0], 4, tetri.TETRI_ERR_INVALID_ARG),
                                 ([3, 2], [0, 2], 4, tetri.TETRI_ERR_INVALID_ARG),
                                 ([3, 2], None, 0, tetri.TETRI_ERR_INVALID_ARG)]:
        with pytest.raises(tetri.TetriError) as e:
            tetri.tetri_pack_chunks(lens, order, C)
        assert e.value.status == code and "tetri_pack_chunks" in str(e.value)
    # capacity too small
    L = tetri.lib()
    lens = np.array([10, 10], dtype=np.int32)
    segs = np.zeros((1, 3), dtype=np.int32)
    offs = np.zeros(8, dtype=np.int32)
    rc = L.tetri_pack_chunks(tetri._ptr(lens), 2, None, 2, 4, tetri._ptr(segs), 1, tetri._ptr(offs), 7, None)
    assert rc == tetri.TETRI_ERR_NOMEM
    rc = L.tetri_pack_chunks(tetri._ptr(lens), 2, None, 2, 4, tetri._ptr(segs), 1, None, 7, None)
    assert rc == tetri.TETRI_ERR_INVALID_ARG           # one output array without the other


def test_chunk_and_plan_metadata_agree():
    w = synth.small("meta", [21, 50, 9, 33], 32, 2, 2, 64, seed=3)
    tables = synth.place_pages(w)
    mb = max(len(t) for t in tables)
    rbt = np.zeros((4, mb), dtype=np.int32)
    for r, t in enumerate(tables):
        rbt[r, :len(t)] = t
    segs, offs = tetri.tetri_pack_chunks(w.prompt_lens, None, 32)
    n, meta_len = tetri.tetri_plan_metadata(w.prompt_lens, None, 32, rbt)
    assert n == len(offs) - 1
    meta = np.full(meta_len, -7, dtype=np.int32)
    layout = np.zeros((n, 4), dtype=np.int32)
    assert tetri.tetri_plan_metadata(w.prompt_lens, None, 32, rbt, meta, layout) == n
    for c in range(n):
        cu, ctx, bt = tetri.tetri_chunk_metadata(segs[offs[c]:offs[c + 1]], rbt)
        o_cu, o_ctx, o_bt, S = (int(x) for x in layout[c])
        assert S == len(ctx) and o_cu % 4 == 0 and o_ctx % 4 == 0 and o_bt % 4 == 0
        assert np.array_equal(meta[o_cu:o_cu + S + 1], cu)
        assert np.array_equal(meta[o_ctx:o_ctx + S], ctx)
        assert np.array_equal(meta[o_bt:o_bt + S * mb].reshape(S, mb), bt)
        # the arrays say what the oracle packer says
        ocu, octx = opacker.chunk_arrays(opacker.pack_chunks(w.prompt_lens, w.order, 32)[c])
        assert list(cu) == ocu and list(ctx) == octx


def test_create_rejects_bad_configurations_before_touching_the_device():
    bad = [dict(num_q_heads=6, num_kv_heads=4), dict(head_dim=96), dict(page_size=32), dict(dtype=7),
           dict(chunk_size=0), dict(max_segs_per_chunk=1000)]
    codes = [tetri.TETRI_ERR_INVALID_ARG, tetri.TETRI_ERR_UNSUPPORTED, tetri.TETRI_ERR_UNSUPPORTED,
             tetri.TETRI_ERR_UNSUPPORTED, tetri.TETRI_ERR_INVALID_ARG, tetri.TETRI_ERR_INVALID_ARG]
    base = dict(num_q_heads=4, num_kv_heads=4, head_dim=64, chunk_size=64, num_pages=32, max_blocks_per_seq=16,
                max_segs_per_chunk=4, page_size=16, dtype=tetri.TETRI_BF16)
    for kw, code in zip(bad, codes):
        with pytest.raises(tetri.TetriError) as e:
            tetri.Tetri(**{**base, **kw})
        assert e.value.status == code, kw


def test_launching_entry_points_reject_a_null_handle():
    L = tetri.lib()
    assert L.tetri_kv_append(None, None, None, None, None, None, None, 1, None) == tetri.TETRI_ERR_INVALID_ARG
    assert L.tetri_chunk_prefill_attn(None, None, None, None, None, None, None, None, 1, 1.0, None, None) \
        == tetri.TETRI_ERR_INVALID_ARG
    assert L.tetri_validate_chunk(None, None, None, None, 1, None) == tetri.TETRI_ERR_INVALID_ARG
    assert L.tetri_set_option(None, b"attn_variant", 0) == tetri.TETRI_ERR_INVALID_ARG
    assert isinstance(tetri.tetri_last_error(), str)


# ---------------------------------------------------------------- prefill scheduler (Sec. 3.3.2)

def test_scheduler_paper_example_twenty_requests_batch_ten():
    """The text's example: twenty queued requests, PrefillSchedBatch 10: two groups, each sorted on its own."""
    rng = np.random.default_rng(7)
    lens = [int(x) for x in rng.integers(1, 600, size=20)]
    for policy, name in ((tetri.TETRI_SJF, "sjf"), (tetri.TETRI_LJF, "ljf"), (tetri.TETRI_FCFS, "fcfs")):
        order = [int(x) for x in tetri.tetri_schedule(lens, policy, 10)]
        assert order == opacker.schedule(lens, name, 10)
        assert sorted(order[:10]) == list(range(10)) and sorted(order[10:]) == list(range(10, 20))
        first = [lens[i] for i in order[:10]]
        second = [lens[i] for i in order[10:]]
        if name == "sjf":
            assert first == sorted(first) and second == sorted(second)
        if name == "ljf":
            assert first == sorted(first, reverse=True) and second == sorted(second, reverse=True)
        if name == "fcfs":
            assert order == list(range(20))


def test_scheduler_is_stable_and_ljf_is_not_reversed_sjf():
    lens = [5, 3, 5, 3, 9]
    assert list(tetri.tetri_schedule(lens, tetri.TETRI_SJF, 0)) == [1, 3, 0, 2, 4]
    assert list(tetri.tetri_schedule(lens, tetri.TETRI_LJF, 0)) == [4, 0, 2, 1, 3]      # ties keep arrival order
    assert list(tetri.tetri_schedule(lens, tetri.TETRI_SJF, 2)) == [1, 0, 3, 2, 4]
    assert list(tetri.tetri_schedule([], tetri.TETRI_SJF, 4)) == []
    with pytest.raises(tetri.TetriError):
        tetri.tetri_schedule(lens, 9, 4)
    with pytest.raises(tetri.TetriError):
        tetri.tetri_schedule([1, -2], tetri.TETRI_SJF, 4)


def test_scheduler_random_batches_match_python_sort_and_feed_the_packer():
    rng = np.random.default_rng(8)
    for _ in range(100):
        n = int(rng.integers(1, 40))
        lens = [int(x) for x in rng.integers(0, 50, size=n)]
        batch = int(rng.integers(0, 12))
        for policy, name in ((tetri.TETRI_SJF, "sjf"), (tetri.TETRI_LJF, "ljf")):
            order = [int(x) for x in tetri.tetri_schedule(lens, policy, batch)]
            assert order == opacker.schedule(lens, name, batch)
            assert lib_plan(lens, order, 16) == [list(c) for c in opacker.pack_chunks(lens, order, 16)]
