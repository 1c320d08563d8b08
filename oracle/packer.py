"""Oracle chunk packer (test infrastructure only).

Follows TetriInfer Sec. 3.3.3 "Chunked Prefill" and the caption of the prefill-scheduler
figure: the scheduled prompts' tokens are laid end to end in scheduled order and cut every
ChunkSize tokens, so a prompt may be sliced across chunks and a chunk may merge several
prompts; only the last chunk may be short (it is then padded to ChunkSize).  A per-request
counter remembers how many tokens were already prefilled.

Written the slow, literal way on purpose: it materialises the token stream.
"""


def pack_chunks(prompt_lens, order, chunk_size):
    """Return a list of chunks; each chunk is a list of segments (req, start, n).

    ``start`` is the number of the request's tokens prefilled before this chunk (the value of
    the per-request progress variable when the chunk runs) and ``n`` the number of its tokens
    in this chunk.  Requests with zero tokens contribute nothing.
    """
    if chunk_size < 1:
        raise ValueError("chunk_size must be positive")
    stream = []                                  # one entry per prompt token, in order
    for req in order:
        for pos in range(int(prompt_lens[req])):
            stream.append((req, pos))
    chunks = []
    for base in range(0, len(stream), chunk_size):
        piece = stream[base:base + chunk_size]   # the last piece may be short
        segs = []
        for req, pos in piece:
            if segs and segs[-1][0] == req and segs[-1][1] + segs[-1][2] == pos:
                segs[-1][2] += 1
            else:
                segs.append([req, pos, 1])
        chunks.append([tuple(s) for s in segs])
    return chunks


def chunk_arrays(segs):
    """cu (prefix sums of segment lengths, cu[0] = 0) and ctx (tokens cached before) of a chunk."""
    cu = [0]
    ctx = []
    for _req, start, n in segs:
        cu.append(cu[-1] + n)
        ctx.append(start)
    return cu, ctx


def schedule(prompt_lens, policy, sched_batch):
    """Scheduled order of the raw queue (Sec. 3.3.2 "Prefill Scheduler").

    The raw queue holds requests 0..n-1 in arrival order.  They are scheduled PrefillSchedBatch at a
    time; each group is sorted by prompt token count with Python's native (stable) sort: "fcfs" keeps
    arrival order, "sjf" ascending, "ljf" descending.  Groups are not interleaved (non-preemptive).
    """
    n = len(prompt_lens)
    group = sched_batch if sched_batch and sched_batch > 0 else max(n, 1)
    order = []
    for b in range(0, n, group):
        ids = list(range(b, min(b + group, n)))
        if policy == "sjf":
            ids.sort(key=lambda i: prompt_lens[i])
        elif policy == "ljf":
            ids.sort(key=lambda i: -prompt_lens[i])
        elif policy != "fcfs":
            raise ValueError(policy)
        order.extend(ids)
    return order
