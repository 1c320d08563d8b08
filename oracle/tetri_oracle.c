/*
 * tetri_oracle.c -- CPU oracle for chunked-prefill attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, obviously-correct statement of
 * what the GPU path must compute.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may build or call it; the product library never does, and the two
 * share no code.
 *
 * What it follows (TetriInfer, arxiv 2401.11181):
 *   - Sec. 3.3.3 "Chunked Prefill": scheduled prompts are sliced and merged, in order, into
 *     fixed-size chunks of ChunkSize tokens; the last chunk is padded; the model runs
 *     prefill one chunk at a time; a per-request variable remembers how far the request
 *     has been prefilled (here ctx_lens[s], the number of tokens already cached).
 *   - Sec. 2.1: the prefill phase of a causal LLM produces the KV cache, so a chunk's
 *     forward has to see every earlier token of its own request plus itself.
 *   - Sec. 3.4 / Sec. 5: the KV cache is kept in pages (the engine is vLLM-derived).
 * The paper gives no kernel; the arithmetic below is the textbook definition of causal
 * scaled-dot-product attention, restricted per request (block-diagonal causal mask),
 * with keys/values read through the page table for cached positions and from the chunk's
 * own k_new/v_new for new positions.
 *
 * Precision: inputs and outputs are float32 arrays (tests feed bf16-representable values
 * widened to float32); every sum, the max, the exponential and the division are done in
 * double.  Softmax is the two-pass textbook form (max, then exp and sum).  No tiling, no
 * online rescaling, no reordering.
 *
 * Layouts (all contiguous, row-major):
 *   q, out          [C][Hq][D]
 *   k_new, v_new    [C][Hkv][D]
 *   kv_pages        [num_pages][2 (0=K,1=V)][Hkv][P][D]
 *   block_table     [S][max_blocks]   physical page id of logical page b of segment s
 *   cu              [S+1]             prefix sums of segment lengths inside the chunk, cu[0]=0
 *   ctx             [S]               tokens of the segment's request already in the cache
 * Rows [cu[S], C) of the chunk are padding: they belong to no request.
 *
 * Pins: every exported function here is pinned by tests/test_oracle_pins.py (brute force,
 * closed forms, invariants, a library routine on the unchunked special case) and by
 * tests/test_oracle_mutants.py (planted mistakes must be caught by those pins).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_MAX_D 1024   /* largest head dimension the oracle accepts */

/* Address of element 0 of the D-vector of (page, which, head, slot) in the pool. */
static size_t pool_offset(int32_t page, int which, int head, int slot,
                          int Hkv, int P, int D)
{
    return ((((size_t)page * 2 + (size_t)which) * (size_t)Hkv + (size_t)head) * (size_t)P
            + (size_t)slot) * (size_t)D;
}

/*
 * KV append (Sec. 2.1: prefill generates the KV cache; Sec. 3.4: in pages).
 * For every segment s and local token t < n_s, position p = ctx[s] + t: copy the K and V
 * vectors of every kv head into slot p % P of page block_table[s][p / P].  Pure copy of
 * elem_size-byte elements (2 for bf16 bit patterns, 4 for float32), nothing else is touched.
 * Returns 0, or -1 if a logical page index exceeds max_blocks.
 */
int oracle_kv_append(const void *k_new, const void *v_new, void *kv_pages,
                     const int32_t *block_table, const int32_t *cu, const int32_t *ctx,
                     int S, int Hkv, int D, int P, int max_blocks, int elem_size)
{
    const char *src[2] = { (const char *)k_new, (const char *)v_new };
    char *pool = (char *)kv_pages;
    size_t vec_bytes = (size_t)D * (size_t)elem_size;
    for (int s = 0; s < S; ++s) {
        int n = cu[s + 1] - cu[s];
        for (int t = 0; t < n; ++t) {
            int p = ctx[s] + t;
            int b = p / P;
            if (b >= max_blocks) return -1;
            int32_t page = block_table[(size_t)s * max_blocks + b];
            int slot = p % P;
            int row = cu[s] + t;
            for (int which = 0; which < 2; ++which)
                for (int kh = 0; kh < Hkv; ++kh) {
                    size_t so = ((size_t)row * Hkv + kh) * vec_bytes;
                    size_t dof = pool_offset(page, which, kh, slot, Hkv, P, D) * (size_t)elem_size;
                    memcpy(pool + dof, src[which] + so, vec_bytes);
                }
        }
    }
    return 0;
}

/* Pointer to the K (which=0) or V (which=1) vector that segment s sees at position j. */
static const float *kv_vector(int which, int s, int j, int kh,
                              const float *k_new, const float *v_new, const float *kv_pages,
                              const int32_t *block_table, const int32_t *cu, const int32_t *ctx,
                              int Hkv, int D, int P, int max_blocks)
{
    if (j < ctx[s]) {                      /* cached earlier: through the page table */
        int32_t page = block_table[(size_t)s * max_blocks + j / P];
        return kv_pages + pool_offset(page, which, kh, j % P, Hkv, P, D);
    }
    /* produced by this chunk: row cu[s] + (j - ctx[s]) of k_new / v_new */
    const float *src = which ? v_new : k_new;
    return src + ((size_t)(cu[s] + (j - ctx[s])) * Hkv + kh) * (size_t)D;
}

/*
 * One output row: segment s, local token t, query head h.  Absolute position p = ctx[s]+t
 * attends to positions 0..p of its own request.  If probs != NULL it receives the p+1
 * softmax weights.  scratch must hold p+1 doubles.
 */
static void attn_one_row(int s, int t, int h,
                         const float *q, const float *k_new, const float *v_new,
                         const float *kv_pages, const int32_t *block_table,
                         const int32_t *cu, const int32_t *ctx,
                         int Hq, int Hkv, int D, int P, int max_blocks, double scale,
                         float *out_vec, double *probs, double *scratch)
{
    int p = ctx[s] + t;
    int kh = h / (Hq / Hkv);               /* query heads share kv heads in groups */
    const float *qv = q + ((size_t)(cu[s] + t) * Hq + h) * (size_t)D;
    double m = -INFINITY;
    for (int j = 0; j <= p; ++j) {
        const float *kv = kv_vector(0, s, j, kh, k_new, v_new, kv_pages, block_table, cu, ctx,
                                    Hkv, D, P, max_blocks);
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += (double)qv[d] * (double)kv[d];
        scratch[j] = scale * dot;
        if (scratch[j] > m) m = scratch[j];
    }
    double l = 0.0;
    for (int j = 0; j <= p; ++j) {
        scratch[j] = exp(scratch[j] - m);
        l += scratch[j];
    }
    double acc[ORACLE_MAX_D];
    for (int d = 0; d < D; ++d) acc[d] = 0.0;
    for (int j = 0; j <= p; ++j) {
        const float *vv = kv_vector(1, s, j, kh, k_new, v_new, kv_pages, block_table, cu, ctx,
                                    Hkv, D, P, max_blocks);
        for (int d = 0; d < D; ++d) acc[d] += scratch[j] * (double)vv[d];
    }
    for (int d = 0; d < D; ++d) out_vec[d] = (float)(acc[d] / l);
    if (probs)
        for (int j = 0; j <= p; ++j) probs[j] = scratch[j] / l;
}

static int max_position(const int32_t *cu, const int32_t *ctx, int S)
{
    int mx = 0;
    for (int s = 0; s < S; ++s) {
        int e = ctx[s] + (cu[s + 1] - cu[s]);
        if (e > mx) mx = e;
    }
    return mx;
}

/*
 * Attention for one whole chunk (Sec. 3.3.3: "one chunk at a time").  Every real row of
 * every segment and every query head gets its output; padding rows [cu[S], C) get zeros.
 * Returns 0, -1 on allocation failure.
 */
int oracle_chunk_prefill_attn(const float *q, const float *k_new, const float *v_new,
                              const float *kv_pages, const int32_t *block_table,
                              const int32_t *cu, const int32_t *ctx,
                              int S, int C, int Hq, int Hkv, int D, int P, int max_blocks,
                              float scale, float *out)
{
    if (D > ORACLE_MAX_D || Hkv <= 0 || Hq % Hkv != 0) return -1;
    int n_real = cu[S];
    int maxp = max_position(cu, ctx, S);
    int failed = 0;
    /* rows of the chunk -> (segment, local token) */
    int *seg_of = (int *)malloc(sizeof(int) * (size_t)(n_real > 0 ? n_real : 1));
    if (!seg_of) return -1;
    for (int s = 0; s < S; ++s)
        for (int r = cu[s]; r < cu[s + 1]; ++r) seg_of[r] = s;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(maxp + 1));
        if (!scratch) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 4)
        for (int r = 0; r < n_real; ++r)
            for (int h = 0; h < Hq; ++h) {
                if (!scratch) continue;
                int s = seg_of[r];
                attn_one_row(s, r - cu[s], h, q, k_new, v_new, kv_pages, block_table, cu, ctx,
                             Hq, Hkv, D, P, max_blocks, (double)scale,
                             out + ((size_t)r * Hq + h) * (size_t)D, NULL, scratch);
            }
        free(scratch);
    }
    free(seg_of);
    for (size_t i = (size_t)n_real * Hq * D; i < (size_t)C * Hq * D; ++i) out[i] = 0.0f;
    return failed ? -1 : 0;
}

/*
 * The same arithmetic for a list of sampled (chunk row, query head) pairs only, for
 * full-size workloads where computing every row on the CPU would take too long.
 * out_samples is [n_samples][D].  A sampled padding row yields zeros.
 */
int oracle_chunk_prefill_attn_samples(const float *q, const float *k_new, const float *v_new,
                                      const float *kv_pages, const int32_t *block_table,
                                      const int32_t *cu, const int32_t *ctx,
                                      int S, int Hq, int Hkv, int D, int P, int max_blocks,
                                      float scale, const int32_t *rows, const int32_t *heads,
                                      int n_samples, float *out_samples)
{
    if (D > ORACLE_MAX_D || Hkv <= 0 || Hq % Hkv != 0) return -1;
    int maxp = max_position(cu, ctx, S);
    int failed = 0;
#pragma omp parallel
    {
        double *scratch = (double *)malloc(sizeof(double) * (size_t)(maxp + 1));
        if (!scratch) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int i = 0; i < n_samples; ++i) {
            if (!scratch) continue;
            int r = rows[i], s = -1;
            for (int k = 0; k < S; ++k)
                if (r >= cu[k] && r < cu[k + 1]) s = k;
            float *o = out_samples + (size_t)i * D;
            if (s < 0) { for (int d = 0; d < D; ++d) o[d] = 0.0f; continue; }
            attn_one_row(s, r - cu[s], heads[i], q, k_new, v_new, kv_pages, block_table, cu, ctx,
                         Hq, Hkv, D, P, max_blocks, (double)scale, o, NULL, scratch);
        }
        free(scratch);
    }
    return failed ? -1 : 0;
}

/*
 * Softmax weights of one row (chunk row r, query head h): probs[0..p] with p = ctx[s]+t.
 * Returns p+1 (the number of weights written), 0 for a padding row, -1 on failure.
 * probs must hold at least ctx[s] + n_s doubles.
 */
int oracle_attn_row_probs(const float *q, const float *k_new, const float *v_new,
                          const float *kv_pages, const int32_t *block_table,
                          const int32_t *cu, const int32_t *ctx,
                          int S, int Hq, int Hkv, int D, int P, int max_blocks,
                          float scale, int r, int h, double *probs)
{
    int s = -1;
    for (int k = 0; k < S; ++k)
        if (r >= cu[k] && r < cu[k + 1]) s = k;
    if (s < 0) return 0;
    if (D > ORACLE_MAX_D || Hkv <= 0 || Hq % Hkv != 0) return -1;
    int p = ctx[s] + (r - cu[s]);
    double *scratch = (double *)malloc(sizeof(double) * (size_t)(p + 1));
    float *tmp = (float *)malloc(sizeof(float) * (size_t)D);
    if (!scratch || !tmp) { free(scratch); free(tmp); return -1; }
    attn_one_row(s, r - cu[s], h, q, k_new, v_new, kv_pages, block_table, cu, ctx,
                 Hq, Hkv, D, P, max_blocks, (double)scale, tmp, probs, scratch);
    free(scratch);
    free(tmp);
    return p + 1;
}
