/*
 * tetri.h -- C ABI of the MI355X (gfx950) chunked-prefill attention library.
 *
 * The library implements the data-parallel hot path of the prefill instance of TetriInfer
 * (arxiv 2401.11181):
 *   - Sec. 3.3.3 "Chunked Prefill": the scheduled prompts are sliced and merged, in order,
 *     into fixed-size chunks of ChunkSize tokens, the last chunk of a batch is padded, the
 *     model runs prefill one chunk at a time and a per-request variable records how far each
 *     request has been prefilled;
 *   - Sec. 2.1: prefill of a causal LLM produces the KV cache, so each chunk attends to all
 *     earlier tokens of its own request(s) and to itself;
 *   - Sec. 3.4 / Sec. 5: the KV cache is managed in pages.
 * and the steps that follow it on the same pages: the prefill scheduler's ordering (Sec. 3.3.2), the export /
 * import of a request's KV cache between the instances (Sec. 3.3.4), the decode instance's attention
 * iteration (Sec. 2.1, Sec. 3.4), and an FP8 variant of the decode-side cache (an extension of this build).
 *
 * Conventions shared by every entry point
 *   - Plain C, no exceptions, no aborts: every call returns a tetri_status (or a count that
 *     is negative on error); a message is kept in the handle (tetri_last_error).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory owned by the caller.  The library never frees or reallocates
 *     caller memory and allocates nothing per call.
 *   - Launching entry points are asynchronous on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and never synchronise it.
 *   - Host-checkable violations (null pointer, counts out of range, unsupported shape,
 *     pointers not 16-byte aligned) are rejected with no kernel launched.  The contents of
 *     device-resident metadata cannot be checked without a synchronisation; use
 *     tetri_validate_chunk for that in tests.
 *
 * Tensor layouts (contiguous, row-major, bf16 unless stated)
 *   q, out         [chunk_size][num_q_heads][head_dim]
 *   k_new, v_new   [chunk_size][num_kv_heads][head_dim]
 *   kv_pages       [num_pages][2 (0 = K, 1 = V)][num_kv_heads][page_size][head_dim]
 *   block_table    [num_segs][max_blocks_per_seq] int32: physical page of logical page b of the
 *                  request of segment s; must cover ceil((ctx_lens[s] + n_s) / page_size) pages
 *   cu_chunk_q_lens[num_segs + 1] int32: prefix sums of the segment lengths n_s inside the
 *                  chunk, cu[0] = 0, cu[num_segs] <= chunk_size; rows [cu[num_segs], chunk_size)
 *                  are padding and belong to no request
 *   ctx_lens       [num_segs] int32: tokens of the segment's request already in the cache
 *                  before this chunk (the per-request progress variable of Sec. 3.3.3)
 */
#ifndef TETRI_H
#define TETRI_H

#include <stdint.h>

#if defined(TETRI_BUILDING)
#define TETRI_API __attribute__((visibility("default")))
#else
#define TETRI_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tetri_ctx tetri_ctx;

typedef enum {
    TETRI_OK = 0,
    TETRI_ERR_INVALID_ARG = -1,   /* null/misaligned pointer, count out of range, bad metadata */
    TETRI_ERR_UNSUPPORTED = -2,   /* shape or dtype this build has no kernel for */
    TETRI_ERR_HIP = -3,           /* the HIP runtime reported an error (launch, copy, no device) */
    TETRI_ERR_NOMEM = -4          /* host allocation failed or a caller-sized array is too small */
} tetri_status;

enum { TETRI_BF16 = 1 };

typedef struct {
    int32_t num_q_heads;          /* Hq                                                     */
    int32_t num_kv_heads;         /* Hkv, Hq % Hkv == 0 (Hq / Hkv query heads share a KV head) */
    int32_t head_dim;             /* 64 or 128                                              */
    int32_t page_size;            /* 16                                                     */
    int32_t chunk_size;           /* ChunkSize: rows of q / k_new / v_new / out             */
    int32_t num_pages;            /* pages in kv_pages                                      */
    int32_t max_blocks_per_seq;   /* row length of block_table                              */
    int32_t max_segs_per_chunk;   /* upper bound of num_segs                                */
    int32_t dtype;                /* TETRI_BF16                                             */
} tetri_config;

/* One slice of a request inside a chunk (Sec. 3.3.3: slicing and merging). */
typedef struct {
    int32_t req;                  /* index into prompt_lens                                 */
    int32_t start;                /* tokens of this request prefilled before this chunk     */
    int32_t len;                  /* tokens of this request in this chunk (> 0)             */
} tetri_segment;

/*
 * Create / destroy a handle carrying the static shape.  The handle owns a fixed amount of device
 * scratch memory (about 34 MB on a 256-CU device, allocated here, freed by tetri_destroy) on the
 * device that is current at creation; launching calls must be made with that device current.
 * tetri_chunk_prefill_attn / _attn_append (launches small enough to be divided over the compute units by
 * stages rather than by row tiles) and tetri_decode_attn keep partial results there: such launches on one
 * handle must not overlap in time; use one handle per stream that runs concurrently.  The attention calls
 * return TETRI_ERR_INVALID_ARG when the handle's previous such launch went to another stream and that stream
 * still has work pending (synchronise the two streams, or use a handle each).  No state survives from one
 * launch to the next: a launch sets the arrival counters it used back to zero, and they are zeroed once more
 * for each launch by the launch before it (and by tetri_create).  The calls may be captured into a HIP graph
 * (a stream that is capturing is not asked whether it has work pending); replays of such a graph and launches
 * outside it may follow each other in any order on one handle, as long as they do not overlap in time.
 * tetri_create checks the configuration (TETRI_ERR_UNSUPPORTED / TETRI_ERR_INVALID_ARG) and
 * that a HIP device is usable (TETRI_ERR_HIP) and stores the handle in *out.
 * A handle must not be used by two threads at once.
 */
TETRI_API tetri_status tetri_create(const tetri_config *config, tetri_ctx **out);
TETRI_API void tetri_destroy(tetri_ctx *ctx);

/* Message of the last error on this handle ("" if none).  With ctx == NULL: the message of the
 * calling thread's last failed tetri_create / tetri_pack_chunks.  Never NULL. */
TETRI_API const char *tetri_last_error(const tetri_ctx *ctx);

/*
 * Chunk packing, host only (Sec. 3.3.3 and the prefill-scheduler figure): lay the tokens of
 * prompts order[0], order[1], ... end to end and cut every chunk_size tokens.  A prompt may be
 * sliced over several chunks, a chunk may merge several prompts, each request is one contiguous
 * row range of a chunk; only the last chunk may be short (its remaining rows are padding).
 *
 *   prompt_lens [n_prompts] host: token count of each prompt (>= 0; empty prompts are skipped)
 *   order       [n_order]   host: scheduled order, indices into prompt_lens, no repeats;
 *                           NULL means 0, 1, ..., n_order - 1 (then n_order <= n_prompts)
 *   segs        [seg_capacity]           host, out: segments of all chunks, chunk after chunk
 *   chunk_seg_offsets [chunk_capacity+1] host, out: chunk c owns segs[offsets[c] .. offsets[c+1])
 *   n_segs_out  host, out (may be NULL): total number of segments
 * Query mode: with segs == NULL and chunk_seg_offsets == NULL nothing is written except
 * *n_segs_out; the return value is the number of chunks either way.
 * Returns the number of chunks (>= 0), or a negative tetri_status: TETRI_ERR_INVALID_ARG
 * (null prompt_lens, chunk_size < 1, negative length, order entry out of range or repeated),
 * TETRI_ERR_NOMEM (a capacity is too small; nothing useful is written).
 */
TETRI_API int32_t tetri_pack_chunks(const int32_t *prompt_lens, int32_t n_prompts,
                          const int32_t *order, int32_t n_order, int32_t chunk_size,
                          tetri_segment *segs, int32_t seg_capacity,
                          int32_t *chunk_seg_offsets, int32_t chunk_capacity,
                          int32_t *n_segs_out);

/*
 * Prefill scheduler, host only (Sec. 3.3.2 "Prefill Scheduler"): turns the raw request queue (arrival
 * order 0..n-1) into the scheduled order that tetri_pack_chunks takes.  Requests are scheduled
 * sched_batch (PrefillSchedBatch) at a time; inside each group of sched_batch consecutive arrivals
 * the policy sorts by prompt token count: TETRI_FCFS keeps arrival order, TETRI_SJF ascending,
 * TETRI_LJF descending.  The sort is stable (ties keep arrival order; the paper uses Python's native
 * sort).  Non-preemptive: groups are never interleaved.  sched_batch <= 0 means one group of all n.
 *   prompt_lens [n] host, in; order_out [n] host, out.
 * Returns TETRI_OK or TETRI_ERR_INVALID_ARG (null pointer, n < 0, unknown policy, negative length).
 */
enum { TETRI_FCFS = 0, TETRI_SJF = 1, TETRI_LJF = 2 };
TETRI_API tetri_status tetri_schedule(const int32_t *prompt_lens, int32_t n, int32_t policy,
                                      int32_t sched_batch, int32_t *order_out);

/*
 * Per-chunk metadata, host only: turn the segments of one chunk into the three int32 arrays
 * the launching entry points take (the caller then copies them to the device).
 *   segs [num_segs] host; req_block_tables [n_prompts][max_blocks_per_seq] host: page list of
 *   every request; cu_out [num_segs+1], ctx_out [num_segs],
 *   block_table_out [num_segs][max_blocks_per_seq] host, out.
 * Returns TETRI_OK or TETRI_ERR_INVALID_ARG (null pointer, req out of range, len <= 0).
 */
TETRI_API tetri_status tetri_chunk_metadata(const tetri_segment *segs, int32_t num_segs,
                                  const int32_t *req_block_tables, int32_t n_prompts,
                                  int32_t max_blocks_per_seq,
                                  int32_t *cu_out, int32_t *ctx_out, int32_t *block_table_out);

/*
 * Packing and metadata of a whole scheduled batch in one host call: tetri_pack_chunks followed by
 * tetri_chunk_metadata for every chunk, written back to back into one caller buffer that can be
 * uploaded with a single copy.
 *   meta_out [meta_capacity] host, out: for chunk c, cu at layout_out[4c+0], ctx_lens at
 *            layout_out[4c+1], block_table at layout_out[4c+2] (offsets in int32 units, each a
 *            multiple of 4 so that every array stays 16-byte aligned); layout_out[4c+3] = num_segs
 *   layout_out [4 * chunk_capacity] host, out
 * Query mode: meta_out == NULL and layout_out == NULL: nothing is written except *meta_len_out.
 * *meta_len_out (may be NULL) receives the number of int32 the metadata needs.
 * Returns the number of chunks or a negative tetri_status (as tetri_pack_chunks; TETRI_ERR_NOMEM if
 * a capacity is too small).
 */
TETRI_API int32_t tetri_plan_metadata(const int32_t *prompt_lens, int32_t n_prompts,
                                      const int32_t *order, int32_t n_order, int32_t chunk_size,
                                      const int32_t *req_block_tables, int32_t max_blocks_per_seq,
                                      int32_t *meta_out, int64_t meta_capacity,
                                      int32_t *layout_out, int32_t chunk_capacity, int64_t *meta_len_out);

/*
 * KV append (Sec. 2.1: prefill generates the KV cache; Sec. 3.4: kept in pages).
 * For every segment s, local token t < n_s and kv head: copy k_new / v_new[cu[s] + t][head][:]
 * bit for bit into slot (ctx_lens[s] + t) % page_size of page
 * block_table[s][(ctx_lens[s] + t) / page_size].  Writes exactly those slots and nothing else;
 * padding rows are not cached.
 *   k_new, v_new: device, in.  kv_pages: device, in/out.  block_table, cu_chunk_q_lens,
 *   ctx_lens: device, in.  num_segs: host scalar, 1..max_segs_per_chunk.
 */
TETRI_API tetri_status tetri_kv_append(tetri_ctx *ctx, const void *k_new, const void *v_new, void *kv_pages,
                             const int32_t *block_table, const int32_t *cu_chunk_q_lens,
                             const int32_t *ctx_lens, int32_t num_segs, void *stream);

/*
 * Chunked-prefill attention for one chunk (Sec. 3.3.3: prefill forward one chunk at a time).
 * Row t of segment s (absolute position p = ctx_lens[s] + t) and query head h produce
 *     out[cu[s]+t][h][:] = sum_{j=0..p} softmax_j(scale * q[cu[s]+t][h] . K_s[j]) * V_s[j]
 * where K_s[j], V_s[j] of kv head h / (Hq/Hkv) come from kv_pages through block_table[s] for
 * j < ctx_lens[s] and from k_new / v_new[cu[s] + j - ctx_lens[s]] otherwise (so the result does
 * not depend on whether tetri_kv_append has already run for this chunk).  Requests merged into
 * one chunk never attend to each other; padding rows of `out` are written as +0 and padding
 * rows of q / k_new / v_new are never read.  Page slots at positions >= ctx_lens[s] are never
 * read.  Arithmetic: bf16 inputs, fp32 accumulation (bf16 MFMA), online softmax in fp32, the
 * softmax weights are rounded to bf16 before the PV product, output rounded to bf16 (nearest
 * even).  Results are deterministic run to run.
 *   q, k_new, v_new, kv_pages, block_table, cu_chunk_q_lens, ctx_lens: device, in.
 *   out: device, out.  num_segs, scale: host scalars.
 */
TETRI_API tetri_status tetri_chunk_prefill_attn(tetri_ctx *ctx, const void *q, const void *k_new,
                                      const void *v_new, const void *kv_pages,
                                      const int32_t *block_table, const int32_t *cu_chunk_q_lens,
                                      const int32_t *ctx_lens, int32_t num_segs, float scale,
                                      void *out, void *stream);

/*
 * Attention and KV append of one chunk in ONE launch (the two steps of Sec. 3.3.3's per-chunk
 * forward that touch the KV cache).  Same results, bit for bit, as tetri_chunk_prefill_attn followed
 * by tetri_kv_append with the same arguments: attention reads only positions < ctx_lens[s] from
 * the pool, the append writes only positions >= ctx_lens[s], so the two do not interfere.
 * Arguments as tetri_chunk_prefill_attn, except that kv_pages is in/out.
 */
TETRI_API tetri_status tetri_chunk_prefill_attn_append(tetri_ctx *ctx, const void *q, const void *k_new,
                                                       const void *v_new, void *kv_pages,
                                                       const int32_t *block_table, const int32_t *cu_chunk_q_lens,
                                                       const int32_t *ctx_lens, int32_t num_segs, float scale,
                                                       void *out, void *stream);

/*
 * KV export and import: the data plane of the dispatcher (Sec. 3.3.4 "Dispatcher": a prefilled
 * request's KV cache is sent from the prefill instance's accelerator memory to the chosen decode
 * instance, either request-level, i.e. the whole request after its last chunk, or chunk-level, i.e.
 * each chunk's slice as soon as it is produced; both instances keep the cache in pages, Sec. 3.4).
 * Both granularities are the same call with other token ranges.
 *
 * For request r = 0..num_reqs-1 the calls move tokens [first_r, first_r + n_r) with
 * n_r = cu_tokens[r+1] - cu_tokens[r] and first_r = first_tokens[r] (0 if first_tokens is NULL),
 * found in slot (pos % page_size) of page block_table[r][pos / page_size].  The transfer buffer is
 * independent of page size and page placement: request after request a dense bf16 block
 *     [2 (0 = K, 1 = V)][num_kv_heads][n_r][head_dim]
 * starting at element 2 * num_kv_heads * head_dim * cu_tokens[r]; so each request's block is one
 * contiguous message and the whole buffer has 2 * num_kv_heads * head_dim * total_tokens elements.
 * tetri_kv_export reads the pool and writes every element of the buffer; tetri_kv_import reads the
 * buffer and writes exactly the page slots of the token ranges (bit for bit, nothing else).
 * With a chunk's cu_chunk_q_lens / ctx_lens / block_table as cu_tokens / first_tokens / block_table
 * the calls move exactly what tetri_kv_append cached for that chunk.
 *   kv_pages, buf: device (export: in, out; import: out, in).  block_table [num_reqs][max_blocks_per_seq],
 *   cu_tokens [num_reqs + 1] (cu_tokens[0] = 0, non-decreasing), first_tokens [num_reqs] or NULL: device, in.
 *   num_reqs: host scalar >= 1.  total_tokens: host scalar, must equal cu_tokens[num_reqs]
 *   (it sizes the launch; 0 is allowed and launches nothing).
 * Neither call uses the handle's scratch memory: they may overlap other launches of the same handle on
 * another stream (chunk-level export while the next chunk is prefilled), as long as the host calls
 * themselves come from one thread at a time.
 * Token ranges of one import must not overlap in the pool.  The device arrays are trusted like those of
 * the other launching calls.  TETRI_ERR_INVALID_ARG for null / misaligned pointers and counts out of
 * range (total_tokens above num_reqs * max_blocks_per_seq * page_size).
 */
TETRI_API tetri_status tetri_kv_export(tetri_ctx *ctx, const void *kv_pages, const int32_t *block_table,
                                       const int32_t *cu_tokens, const int32_t *first_tokens, int32_t num_reqs,
                                       int64_t total_tokens, void *buf, void *stream);
TETRI_API tetri_status tetri_kv_import(tetri_ctx *ctx, const void *buf, const int32_t *block_table,
                                       const int32_t *cu_tokens, const int32_t *first_tokens, int32_t num_reqs,
                                       int64_t total_tokens, void *kv_pages, void *stream);

/*
 * One decode iteration of a batch of requests over the paged cache: the decode instance's counterpart
 * of tetri_chunk_prefill_attn (Sec. 2.1: after prefill, each iteration produces one token whose query
 * attends to the request's KV cache; Sec. 3.4: the decode instance runs the steps of many requests
 * as one batch over a paged cache).  For request b with ctx_lens[b] cached tokens and query head h
 *     out[b][h][:] = sum_{j=0..ctx_b} softmax_j(scale * q[b][h] . K_b[j]) * V_b[j]
 * where K_b[j], V_b[j] of kv head h / (Hq/Hkv) come from kv_pages through block_table[b] for
 * j < ctx_lens[b] and from k_new[b] / v_new[b] for j = ctx_lens[b] (the new token attends to itself;
 * cache it with tetri_kv_append and cu_chunk_q_lens = 0, 1, ..., num_reqs, before or after).  The same
 * function as tetri_chunk_prefill_attn on a chunk of one-token segments, computed by a kernel made
 * for it: it reads every cached byte once, for all query heads of a kv head together.
 * Arithmetic as tetri_chunk_prefill_attn; page slots at positions >= ctx_lens[b] are never read.
 *   q, out [num_reqs][num_q_heads][head_dim]; k_new, v_new [num_reqs][num_kv_heads][head_dim];
 *   block_table [num_reqs][max_blocks_per_seq]; ctx_lens [num_reqs] (>= 0): device.
 *   num_reqs >= 1 (not bound by chunk_size or max_segs_per_chunk); max_ctx_len: host scalar, an upper
 *   bound of ctx_lens that only sizes the launch (how far the keys of a request are split over
 *   workgroups when there are few requests); results do not depend on it.
 * Uses the handle's scratch memory when it splits: launches on one handle must not overlap in time.
 * Results are deterministic run to run.  TETRI_ERR_UNSUPPORTED for more than 32 query heads per kv head.
 */
TETRI_API tetri_status tetri_decode_attn(tetri_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                                         const void *kv_pages, const int32_t *block_table, const int32_t *ctx_lens,
                                         int32_t num_reqs, int32_t max_ctx_len, float scale, void *out, void *stream);

/*
 * tetri_decode_attn for callers that cannot allocate device memory or hold an allocation: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same function and
 * same kernels as tetri_decode_attn; the only difference is where the parts of split requests are kept: not
 * in memory the handle allocated but in a static device array of the library, 8 MiB on every device the
 * library runs on, held until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine); the array's address on the handle's device was looked up by tetri_create.
 * Limit: num_reqs * num_q_heads * (head_dim + 2) * 4 bytes * 2 must fit the array (two parts per request and
 * head; 8066 (request, head) pairs at head_dim 128), else TETRI_ERR_INVALID_ARG and nothing is launched;
 * within the limit the keys of a request are split as far as the array reaches, so the split (and with it
 * the rounding, not the function) may differ from tetri_decode_attn's; with the same "decode_parts" the
 * two calls give the same bits.
 * Every call on a device shares that device's array, which keeps the last call's contents (every part is
 * written before it is read, nothing has to start at zero): calls that overlap in time on one device, on
 * any handles or streams, race.
 */
TETRI_API tetri_status tetri_decode_attn_static(tetri_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                                                const void *kv_pages, const int32_t *block_table, const int32_t *ctx_lens,
                                                int32_t num_reqs, int32_t max_ctx_len, float scale, void *out, void *stream);

/*
 * The decode iteration and the caching of its new tokens in ONE launch (Sec. 2.1: every decode
 * iteration extends the KV cache by one token).  Same `out`, bit for bit, as tetri_decode_attn, and the
 * same pool as tetri_kv_append with cu_chunk_q_lens = 0, 1, ..., num_reqs afterwards: k_new[b] / v_new[b]
 * are written to slot ctx_lens[b] % page_size of page block_table[b][ctx_lens[b] / page_size], and
 * nothing else is written.  block_table must therefore cover position ctx_lens[b]
 * (max_ctx_len <= max_blocks_per_seq * page_size - 1).  Arguments as tetri_decode_attn, kv_pages in/out.
 */
TETRI_API tetri_status tetri_decode_attn_append(tetri_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                                                void *kv_pages, const int32_t *block_table, const int32_t *ctx_lens,
                                                int32_t num_reqs, int32_t max_ctx_len, float scale, void *out,
                                                void *stream);

/*
 * FP8 KV cache on the decode side (an extension of this build, not of the paper: the paper keeps the cache
 * in the model's 16-bit type; Sec. 3.3.4 names the link between the instances as the scarce resource and
 * Sec. 3.4 the decode instance's memory, and an 8-bit cache halves the bytes of both).
 * Format: one OCP FP8 E4M3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, no infinities,
 * largest finite value 448) per element, pool layout as kv_pages with one byte per element, and one
 * positive finite scale per tensor: a value x is stored as the code of fl32(x * fl32(1 / scale)) clamped
 * to [-448, 448] and rounded to nearest, ties to even; a code stands for value(code) * scale.
 *
 * tetri_kv_export_fp8: as tetri_kv_export from the 16-bit pool, but the dense buffer holds codes
 *   ([2][num_kv_heads][n_r][head_dim] bytes per request, request r at byte 2 * num_kv_heads * head_dim *
 *   cu_tokens[r]); the K half of every block under k_scale, the V half under v_scale.
 * tetri_kv_import_fp8: scatters such a buffer of codes into an FP8 pool (bytes, bit for bit).
 * tetri_decode_attn_fp8: tetri_decode_attn over an FP8 pool: cached K and V are value(code) * k_scale and
 *   value(code) * v_scale, the new token's k_new / v_new (bf16) enter unquantised; with append = 1 the
 *   codes of k_new[b] / v_new[b] are also written to slot ctx_lens[b] of the pool (then kv_pages_fp8 is
 *   in/out and block_table must cover that position), with append = 0 the pool is only read.
 * Other arguments, errors and the scratch-memory rule as for the 16-bit calls; TETRI_ERR_INVALID_ARG for
 * scales that are not positive and finite.
 */
TETRI_API tetri_status tetri_kv_export_fp8(tetri_ctx *ctx, const void *kv_pages, const int32_t *block_table,
                                           const int32_t *cu_tokens, const int32_t *first_tokens, int32_t num_reqs,
                                           int64_t total_tokens, float k_scale, float v_scale, void *buf, void *stream);
TETRI_API tetri_status tetri_kv_import_fp8(tetri_ctx *ctx, const void *buf, const int32_t *block_table,
                                           const int32_t *cu_tokens, const int32_t *first_tokens, int32_t num_reqs,
                                           int64_t total_tokens, void *kv_pages_fp8, void *stream);
TETRI_API tetri_status tetri_decode_attn_fp8(tetri_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                                             void *kv_pages_fp8, const int32_t *block_table, const int32_t *ctx_lens,
                                             int32_t num_reqs, int32_t max_ctx_len, float scale, float k_scale,
                                             float v_scale, int32_t append, void *out, void *stream);

/*
 * Chunked prefill over the FP8 cache (the same extension on the prefill side: an instance that keeps its cache in
 * codes, e.g. a decode instance that takes over a prefill, Sec. 3.3.4 / 3.4, reads it without a 16-bit copy).
 * tetri_chunk_prefill_attn over a pool of E4M3 codes in the format above: the cached K and V of a segment are
 * value(code) * k_scale and value(code) * v_scale, the chunk's own rows k_new / v_new (bf16) enter unquantised.
 * With append = 1 the codes of the chunk's rows (fl32(x * fl32(1 / scale)), clamped, rounded to nearest even) are
 * also written to their slots of the pool, as tetri_chunk_prefill_attn_append does with the 16-bit values (the
 * launch reads none of the slots it writes); with append = 0 the pool is only read.
 *   kv_pages_fp8 device [num_pages][2][num_kv_heads][page_size][head_dim] bytes, 16-byte aligned; in/out with append = 1
 * Every other argument, the scratch-memory rule and the errors as for tetri_chunk_prefill_attn;
 * TETRI_ERR_INVALID_ARG also for scales that are not positive and finite and for append other than 0 / 1.
 */
TETRI_API tetri_status tetri_chunk_prefill_attn_fp8(tetri_ctx *ctx, const void *q, const void *k_new, const void *v_new,
                                                    void *kv_pages_fp8, const int32_t *block_table,
                                                    const int32_t *cu_chunk_q_lens, const int32_t *ctx_lens,
                                                    int32_t num_segs, float scale, float k_scale, float v_scale,
                                                    int32_t append, void *out, void *stream);

/*
 * Debug check of device-resident chunk metadata.  Synchronises `stream`, copies the arrays to
 * the host and checks: cu[0] == 0, cu strictly increasing, cu[num_segs] <= chunk_size,
 * ctx_lens >= 0, every needed block-table entry in [0, num_pages), enough logical pages
 * (ceil((ctx+n)/page_size) <= max_blocks_per_seq), and no physical page written by two
 * segments.  Returns TETRI_OK, TETRI_ERR_INVALID_ARG (message says what), or TETRI_ERR_HIP.
 */
TETRI_API tetri_status tetri_validate_chunk(tetri_ctx *ctx, const int32_t *block_table,
                                  const int32_t *cu_chunk_q_lens, const int32_t *ctx_lens,
                                  int32_t num_segs, void *stream);

/*
 * Kernel-variant selection for measurements and tests.  Known keys:
 *   "attn_variant"      0 = the library chooses the workgroup size (8 wavefronts; 4, two workgroups to a
 *                       compute unit, when a full chunk alone gives five row tiles per four compute units or
 *                       more), 1 / 2 = 4- / 8-wavefront workgroups;
 *   "split_keys"        1 (default) = a launch with fewer than five row tiles per four compute units divides the key
 *                       ranges of its tiles among more workgroups than it has tiles.  If the tiles and one helper
 *                       workgroup per two tiles fit the compute units, every tile with a long key range hands the
 *                       tail of it to its helper; otherwise (and only for chunks whose segments have 256 rows or
 *                       more on average, and at most 64 segments) the stages (64 or 128 keys each) of all row
 *                       tiles of a head group are laid end to end and every workgroup of the group gets an equal
 *                       range of them.  Tiles shared by several workgroups are finished from partial results in
 *                       the handle's scratch memory (see tetri_create).  0 = always one workgroup per row tile;
 *   "split_min_stages"  tails: key ranges of fewer stages than this are not divided (default 8; at least 2);
 *   "split_bias_stages" tails: stages a tile keeps before the rest is shared (default 6; not negative);
 *   "split_share_q8"    tails: share of that rest the helper takes, in 1/256 (default 85; 1..128);
 *   "stream_wgs"        workgroups per head group when the stages are laid end to end (default 0: as many as
 *                       the device has compute units for); a value of 1..255 also forces that division for
 *                       launches of any size with at most 64 segments;
 *   "decode_parts"      workgroups that share the keys of one (request, kv head) in tetri_decode_attn
 *                       (default 0: chosen from num_reqs and max_ctx_len);
 *   "transfer_slabs"    (K / V, head) slabs one workgroup of tetri_kv_export / tetri_kv_import moves
 *                       (default 0: chosen from the size of the transfer).
 * Unknown keys or values give TETRI_ERR_INVALID_ARG.  Every setting computes the same
 * function to the same tolerance.
 */
TETRI_API tetri_status tetri_set_option(tetri_ctx *ctx, const char *key, int32_t value);

/* Version of this ABI (bumped on incompatible change). */
TETRI_API int32_t tetri_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TETRI_H */
