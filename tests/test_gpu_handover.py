"""GPU tests of the state that launches with divided tiles keep on a handle (partial results and arrival counters
in the handle's scratch memory): one handle used across every way of handing out the work, two handles on two
streams at once, and the refusal of a launch that would overlap the handle's previous one on another stream.

Every kernel here runs to its normal end: the overlap is detected on the host, before anything is launched.
"""
import numpy as np
import pytest
import torch

from paper_2401_11181_amd import synth, tetri
import gpu_common as gc

pytestmark = pytest.mark.gpu
DEV = gc.DEV

# (label, options set before the launch); options keep their value until set again
MODES = [
    ("tails", {"split_keys": 1, "stream_wgs": 0, "split_min_stages": 2, "split_bias_stages": 0}),
    ("stream5", {"stream_wgs": 5}),
    ("whole", {"stream_wgs": 0, "split_keys": 0}),
    ("tails", {"split_keys": 1}),
    ("stream3", {"stream_wgs": 3}),
    ("stream200", {"stream_wgs": 200}),
    ("tails", {"stream_wgs": 0}),
    ("stream5", {"stream_wgs": 5}),
    ("whole", {"stream_wgs": 0, "split_keys": 0}),
]


def prefilled(oracle, name, seed):
    """A 1024-token prompt prefilled in 4 chunks of 256 (8 heads x 128): session, device inputs of the last chunk,
    the pool, and the oracle's output rows of that chunk."""
    w = synth.small(name, [1024], 256, 8, 8, 128, seed=seed)
    qs, ks, vs, tables = gc.workload_tensors(w)
    outs, pool, sess, _ = gc.gpu_prefill(w, qs, ks, vs, tables, fused=True)
    ref, _, _ = gc.oracle_prefill(oracle, w, qs, ks, vs, tables)
    gc.compare(outs, ref, label=name)
    c = sess.n_chunks - 1
    dq, dk, dv = [t.to(DEV) for t in qs], [t.to(DEV) for t in ks], [t.to(DEV) for t in vs]
    q, k, v = sess.gather_chunk(dq, c), sess.gather_chunk(dk, c), sess.gather_chunk(dv, c)
    return w, sess, c, (q, k, v), pool, np.asarray(ref[0])[768:1024]


def check(out, ref_rows, label):
    got = out.float().cpu().numpy()
    err = np.abs(got - ref_rows)
    rel = np.linalg.norm(got - ref_rows) / np.linalg.norm(ref_rows)
    assert err.max() <= 2e-2 and err.mean() <= 2e-3 and rel <= 1e-2, (label, err.max(), err.mean(), rel)


def test_one_handle_across_modes(oracle):
    """The same chunk on one handle with the work handed out in every way in turn, two rounds: every result meets
    the oracle, and a way of handing out gives the same bits whatever ran on the handle before it."""
    w, sess, c, (q, k, v), pool, ref_rows = prefilled(oracle, "modes", 141)
    seen = {}
    for _round in range(2):
        for label, opts in MODES:
            for key, value in opts.items():
                sess.handle.tetri_set_option(key, value)
            out = torch.full((w.chunk_size, w.num_q_heads, w.head_dim), 7.0, dtype=torch.bfloat16, device=DEV)
            sess.attn(c, q, k, v, pool, w.scale, out)
            torch.cuda.synchronize()
            check(out, ref_rows, label)
            bits = out.view(torch.int16).cpu()
            if label in seen:
                assert torch.equal(bits, seen[label]), label + ": result depends on what ran on the handle before"
            seen[label] = bits


def test_two_handles_on_two_streams(oracle):
    """Two handles, each with its own scratch memory, launching divided tiles on two streams at once: allowed, and
    each gives the bits it gives alone."""
    w, sess_a, c, (q, k, v), pool, ref_rows = prefilled(oracle, "two-handles", 142)
    qs, ks, vs, tables = gc.workload_tensors(w)
    from paper_2401_11181_amd.prefill import ChunkedPrefill
    sess_b = ChunkedPrefill(w.prompt_lens, w.order, w.chunk_size, w.num_q_heads, w.num_kv_heads, w.head_dim,
                            w.num_pages, tables, device=DEV, page_size=w.page_size)
    for s in (sess_a, sess_b):
        s.handle.tetri_set_option("split_min_stages", 2)
        s.handle.tetri_set_option("split_bias_stages", 0)
    sess_b.handle.tetri_set_option("stream_wgs", 5)
    alone = []
    for s in (sess_a, sess_b):
        out = torch.zeros((w.chunk_size, w.num_q_heads, w.head_dim), dtype=torch.bfloat16, device=DEV)
        s.attn(c, q, k, v, pool, w.scale, out)
        torch.cuda.synchronize()
        check(out, ref_rows, "alone")
        alone.append(out.view(torch.int16).cpu())
    st_a, st_b = torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)
    outs_a = [torch.zeros_like(q) for _ in range(20)]
    outs_b = [torch.zeros_like(q) for _ in range(20)]
    torch.cuda.synchronize()
    for i in range(20):
        sess_a.attn(c, q, k, v, pool, w.scale, outs_a[i], stream=st_a)
        sess_b.attn(c, q, k, v, pool, w.scale, outs_b[i], stream=st_b)
    torch.cuda.synchronize()
    for i in range(20):
        assert torch.equal(outs_a[i].view(torch.int16).cpu(), alone[0]), ("tails", i)
        assert torch.equal(outs_b[i].view(torch.int16).cpu(), alone[1]), ("stream", i)


def test_overlapping_launches_on_one_handle_are_refused(oracle):
    """A launch that divides tiles while the handle's previous such launch may still run on another stream is an
    error (the two would share scratch memory); launches that divide nothing are not held to this; once the first
    stream has drained, the other stream may use the handle."""
    w, sess, c, (q, k, v), pool, ref_rows = prefilled(oracle, "overlap", 143)
    sess.handle.tetri_set_option("split_min_stages", 2)
    sess.handle.tetri_set_option("split_bias_stages", 0)
    st_a, st_b = torch.cuda.Stream(device=DEV), torch.cuda.Stream(device=DEV)
    out_a, out_b = torch.zeros_like(q), torch.zeros_like(q)
    big = torch.randn(8192, 8192, device=DEV).to(torch.bfloat16)
    acc = torch.empty_like(big)
    torch.matmul(big, big, out=acc)
    torch.cuda.synchronize()
    for mode_opts in ({"stream_wgs": 0}, {"stream_wgs": 5}):
        for key, value in mode_opts.items():
            sess.handle.tetri_set_option(key, value)
        with torch.cuda.stream(st_a):
            for _ in range(80):                             # some hundred milliseconds of work ahead of the launch
                torch.matmul(big, big, out=acc)
        sess.attn(c, q, k, v, pool, w.scale, out_a, stream=st_a)
        assert not st_a.query(), "stream A should still be busy"
        with pytest.raises(tetri.TetriError) as info:
            sess.attn(c, q, k, v, pool, w.scale, out_b, stream=st_b)
        assert info.value.status == tetri.TETRI_ERR_INVALID_ARG
        assert "overlap" in str(info.value)
        # a launch of whole tiles uses no scratch memory: allowed on the other stream meanwhile
        sess.handle.tetri_set_option("split_keys", 0)
        sess.handle.tetri_set_option("stream_wgs", 0)
        sess.attn(c, q, k, v, pool, w.scale, out_b, stream=st_b)
        sess.handle.tetri_set_option("split_keys", 1)
        for key, value in mode_opts.items():
            sess.handle.tetri_set_option(key, value)
        torch.cuda.synchronize()
        check(out_a, ref_rows, "first stream")
        check(out_b, ref_rows, "whole tiles on the second stream")
        # the first stream has drained: the second one may now divide tiles on this handle
        out_b.zero_()
        torch.cuda.synchronize()                            # (the fill runs on the default stream)
        sess.attn(c, q, k, v, pool, w.scale, out_b, stream=st_b)
        torch.cuda.synchronize()
        check(out_b, ref_rows, "second stream, after the first has drained")
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))


@pytest.mark.parametrize("fp8", [False, True], ids=["16-bit-pool", "fp8-pool"])
def test_graph_replays_between_eager_launches(oracle, fp8):
    """A HIP graph that holds an odd number of launches that divide tiles, replayed several times with eager launches of
    the same kind and synchronisations in between: every replay gives the bits of the eager launch.  (A replay uses the
    arrival counters it was captured with, whatever the handle has handed out since: every launch leaves the counters
    it used at zero.)"""
    if fp8:
        w = synth.small("graph-fp8", [1024], 256, 8, 8, 128, seed=145)
        qs, ks, vs, tables = gc.workload_tensors(w)
        _outs, pool, sess = gc.gpu_prefill_fp8(w, qs, ks, vs, tables, 0.0137, 0.0171)
        c = sess.n_chunks - 1
        dq, dk, dv = [t.to(DEV) for t in qs], [t.to(DEV) for t in ks], [t.to(DEV) for t in vs]
        q, k, v = sess.gather_chunk(dq, c), sess.gather_chunk(dk, c), sess.gather_chunk(dv, c)
        launch = lambda out: sess.attn_fp8(c, q, k, v, pool, w.scale, 0.0137, 0.0171, 0, out)
    else:
        w, sess, c, (q, k, v), pool, _ref_rows = prefilled(oracle, "graph", 144)
        launch = lambda out: sess.attn(c, q, k, v, pool, w.scale, out)
    for mode_opts in ({"stream_wgs": 0, "split_min_stages": 2, "split_bias_stages": 0}, {"stream_wgs": 5}, {"stream_wgs": 3}):
        for key, value in mode_opts.items():
            sess.handle.tetri_set_option(key, value)
        eager = torch.zeros_like(q)
        launch(eager)
        torch.cuda.synchronize()
        want = eager.view(torch.int16).clone()
        outs = [torch.zeros_like(q) for _ in range(3)]
        tmp = torch.zeros_like(q)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for o in outs:
                launch(o)
        for rep in range(4):
            for o in outs:
                o.fill_(7.0)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for i, o in enumerate(outs):
                assert torch.equal(o.view(torch.int16), want), (mode_opts, "replay", rep, "launch", i)
            for _ in range(rep % 2 + 1):                 # one or two eager launches: the handle's own alternation moves on
                tmp.fill_(7.0)
                launch(tmp)
            torch.cuda.synchronize()
            assert torch.equal(tmp.view(torch.int16), want), (mode_opts, "eager after replay", rep)
