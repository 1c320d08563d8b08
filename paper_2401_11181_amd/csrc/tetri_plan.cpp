// Chunk packer, prefill scheduler and per-chunk metadata of libtetri: plain host code, no HIP, so
// that it also builds with an ordinary C++ compiler (the sanitizer build of the tests does).
// TetriInfer Sec. 3.3.3 "Chunked Prefill" is the source of the packing rule, Sec. 3.3.2 "Prefill
// Scheduler" of the ordering policies.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "tetri_plan.h"

namespace {

thread_local std::string g_thread_err;

tetri_status fail(void *, tetri_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_thread_err = buf;
    return st;
}

}  // namespace

void tetri_set_thread_error(const char *msg) { g_thread_err = msg ? msg : ""; }
const char *tetri_thread_error() { return g_thread_err.c_str(); }

extern "C" {

int32_t tetri_pack_chunks(const int32_t *prompt_lens, int32_t n_prompts, const int32_t *order, int32_t n_order,
                          int32_t chunk_size, tetri_segment *segs, int32_t seg_capacity,
                          int32_t *chunk_seg_offsets, int32_t chunk_capacity, int32_t *n_segs_out)
{
    if (!prompt_lens || n_prompts < 0 || n_order < 0)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: null prompt_lens or negative count");
    if (chunk_size < 1) return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: chunk_size=%d", chunk_size);
    if (!order && n_order > n_prompts)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: n_order=%d exceeds n_prompts=%d", n_order, n_prompts);
    const bool query = (segs == nullptr && chunk_seg_offsets == nullptr);
    if (!query && (!segs || !chunk_seg_offsets))
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: segs and chunk_seg_offsets must both be given or both be null");
    std::vector<char> seen(order ? (size_t)n_prompts : 0, 0);
    int64_t n_chunks = 0, n_segs = 0;
    int32_t room = 0;                      // free rows left in the chunk being filled
    for (int32_t i = 0; i < n_order; ++i) {
        const int32_t req = order ? order[i] : i;
        if (req < 0 || req >= n_prompts)
            return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: order[%d]=%d out of range", i, req);
        if (order) {
            if (seen[req]) return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: request %d scheduled twice", req);
            seen[req] = 1;
        }
        const int32_t len = prompt_lens[req];
        if (len < 0) return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: prompt_lens[%d]=%d", req, len);
        int32_t done = 0;
        while (done < len) {
            if (room == 0) {               // open the next chunk
                if (!query) {
                    if (n_chunks >= chunk_capacity)
                        return fail(nullptr, TETRI_ERR_NOMEM, "tetri_pack_chunks: chunk_capacity=%d too small", chunk_capacity);
                    chunk_seg_offsets[n_chunks] = (int32_t)n_segs;
                }
                ++n_chunks;
                room = chunk_size;
            }
            const int32_t take = (len - done < room) ? len - done : room;
            if (!query) {
                if (n_segs >= seg_capacity)
                    return fail(nullptr, TETRI_ERR_NOMEM, "tetri_pack_chunks: seg_capacity=%d too small", seg_capacity);
                segs[n_segs].req = req;
                segs[n_segs].start = done;
                segs[n_segs].len = take;
            }
            ++n_segs;
            done += take;
            room -= take;
        }
    }
    if (n_chunks > INT32_MAX || n_segs > INT32_MAX)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_pack_chunks: plan too large");
    if (!query) chunk_seg_offsets[n_chunks] = (int32_t)n_segs;
    if (n_segs_out) *n_segs_out = (int32_t)n_segs;
    return (int32_t)n_chunks;
}

tetri_status tetri_schedule(const int32_t *prompt_lens, int32_t n, int32_t policy, int32_t sched_batch, int32_t *order_out)
{
    if (!prompt_lens || !order_out || n < 0)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_schedule: null pointer or negative count");
    if (policy != TETRI_FCFS && policy != TETRI_SJF && policy != TETRI_LJF)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_schedule: unknown policy %d", policy);
    for (int32_t i = 0; i < n; ++i) {
        if (prompt_lens[i] < 0) return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_schedule: prompt_lens[%d]=%d", i, prompt_lens[i]);
        order_out[i] = i;
    }
    if (policy == TETRI_FCFS) return TETRI_OK;
    const int32_t group = sched_batch > 0 ? sched_batch : (n > 0 ? n : 1);
    for (int32_t b = 0; b < n; b += group) {
        int32_t *first = order_out + b, *last = order_out + (b + group < n ? b + group : n);
        if (policy == TETRI_SJF)
            std::stable_sort(first, last, [&](int32_t x, int32_t y) { return prompt_lens[x] < prompt_lens[y]; });
        else
            std::stable_sort(first, last, [&](int32_t x, int32_t y) { return prompt_lens[x] > prompt_lens[y]; });
    }
    return TETRI_OK;
}

tetri_status tetri_chunk_metadata(const tetri_segment *segs, int32_t num_segs, const int32_t *req_block_tables,
                                  int32_t n_prompts, int32_t max_blocks_per_seq,
                                  int32_t *cu_out, int32_t *ctx_out, int32_t *block_table_out)
{
    if (!segs || !req_block_tables || !cu_out || !ctx_out || !block_table_out || num_segs < 1 || max_blocks_per_seq < 1)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_chunk_metadata: null argument or empty chunk");
    cu_out[0] = 0;
    for (int32_t s = 0; s < num_segs; ++s) {
        if (segs[s].req < 0 || segs[s].req >= n_prompts || segs[s].len <= 0 || segs[s].start < 0)
            return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_chunk_metadata: segment %d is malformed", s);
        cu_out[s + 1] = cu_out[s] + segs[s].len;
        ctx_out[s] = segs[s].start;
        std::memcpy(block_table_out + (size_t)s * max_blocks_per_seq,
                    req_block_tables + (size_t)segs[s].req * max_blocks_per_seq,
                    sizeof(int32_t) * (size_t)max_blocks_per_seq);
    }
    return TETRI_OK;
}

int32_t tetri_plan_metadata(const int32_t *prompt_lens, int32_t n_prompts, const int32_t *order, int32_t n_order,
                            int32_t chunk_size, const int32_t *req_block_tables, int32_t max_blocks,
                            int32_t *meta_out, int64_t meta_capacity, int32_t *layout_out, int32_t chunk_capacity,
                            int64_t *meta_len_out)
{
    if (!req_block_tables || max_blocks < 1)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_plan_metadata: null block tables or max_blocks_per_seq < 1");
    const bool query = (meta_out == nullptr && layout_out == nullptr);
    if (!query && (!meta_out || !layout_out))
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_plan_metadata: meta_out and layout_out must both be given or both be null");
    int32_t n_segs = 0;
    const int32_t n_chunks = tetri_pack_chunks(prompt_lens, n_prompts, order, n_order, chunk_size, nullptr, 0, nullptr, 0, &n_segs);
    if (n_chunks < 0) return n_chunks;
    thread_local std::vector<tetri_segment> segs;
    thread_local std::vector<int32_t> offs;
    segs.resize((size_t)n_segs + 1);
    offs.resize((size_t)n_chunks + 1);
    int32_t rc = tetri_pack_chunks(prompt_lens, n_prompts, order, n_order, chunk_size, segs.data(), n_segs, offs.data(), n_chunks, nullptr);
    if (rc < 0) return rc;
    if (!query && n_chunks > chunk_capacity)
        return fail(nullptr, TETRI_ERR_NOMEM, "tetri_plan_metadata: chunk_capacity=%d too small for %d chunks", chunk_capacity, n_chunks);
    auto up4 = [](int64_t x) { return (x + 3) / 4 * 4; };
    int64_t at = 0;
    for (int32_t c = 0; c < n_chunks; ++c) {
        const int32_t S = offs[c + 1] - offs[c];
        const int64_t o_cu = at, o_ctx = o_cu + up4(S + 1), o_bt = o_ctx + up4(S);
        at = o_bt + up4((int64_t)S * max_blocks);
        if (query) continue;
        if (at > meta_capacity || at > INT32_MAX)
            return fail(nullptr, TETRI_ERR_NOMEM, "tetri_plan_metadata: meta_capacity=%lld too small", (long long)meta_capacity);
        layout_out[4 * c + 0] = (int32_t)o_cu;
        layout_out[4 * c + 1] = (int32_t)o_ctx;
        layout_out[4 * c + 2] = (int32_t)o_bt;
        layout_out[4 * c + 3] = S;
        tetri_status st = tetri_chunk_metadata(segs.data() + offs[c], S, req_block_tables, n_prompts, max_blocks,
                                               meta_out + o_cu, meta_out + o_ctx, meta_out + o_bt);
        if (st != TETRI_OK) return st;
    }
    if (meta_len_out) *meta_len_out = at;
    return n_chunks;
}

}  // extern "C"
