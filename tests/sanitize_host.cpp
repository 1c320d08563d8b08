// Driver of the sanitizer leg (built and run by tests/test_sanitizers.py with
// -fsanitize=address,undefined): the HIP-free host layer of the library (chunk packer, scheduler,
// per-chunk metadata: tetri_plan.cpp) and the C oracle (oracle/tetri_oracle.c) are compiled into
// this one program and driven with exactly-sized heap buffers, so that any read or write past a
// capacity, a bad offset or an integer overflow in their index arithmetic aborts the run.
// Results are also checked: the packer against a token-stream re-derivation written here, the
// oracle against closed forms (first token returns its own V; zero keys give the prefix mean; the
// append puts every row where the page table says and nowhere else).
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "tetri.h"

extern "C" {
int oracle_kv_append(const void *k_new, const void *v_new, void *kv_pages, const int32_t *block_table, const int32_t *cu,
                     const int32_t *ctx, int S, int Hkv, int D, int P, int max_blocks, int elem_size);
int oracle_chunk_prefill_attn(const float *q, const float *k_new, const float *v_new, const float *kv_pages,
                              const int32_t *block_table, const int32_t *cu, const int32_t *ctx, int S, int C, int Hq, int Hkv,
                              int D, int P, int max_blocks, float scale, float *out);
int oracle_chunk_prefill_attn_samples(const float *q, const float *k_new, const float *v_new, const float *kv_pages,
                                      const int32_t *block_table, const int32_t *cu, const int32_t *ctx, int S, int Hq, int Hkv,
                                      int D, int P, int max_blocks, float scale, const int32_t *rows, const int32_t *heads,
                                      int n_samples, float *out_samples);
int oracle_attn_row_probs(const float *q, const float *k_new, const float *v_new, const float *kv_pages,
                          const int32_t *block_table, const int32_t *cu, const int32_t *ctx, int S, int Hq, int Hkv, int D, int P,
                          int max_blocks, float scale, int r, int h, double *probs);
}

static int g_failed = 0;
#define CHECK(cond)                                                                   \
    do {                                                                              \
        if (!(cond)) {                                                                \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            ++g_failed;                                                               \
        }                                                                             \
    } while (0)

// Heap arrays of exactly n elements (no slack: the sanitizer sees the first byte past the end).
template <class T> struct Exact {
    T *p;
    size_t n;
    explicit Exact(size_t n_) : p(static_cast<T *>(std::malloc(n_ ? n_ * sizeof(T) : 1))), n(n_) {}
    ~Exact() { std::free(p); }
    T &operator[](size_t i) { return p[i]; }
    Exact(const Exact &) = delete;
};

static void packer_against_token_stream(std::mt19937 &rng)
{
    for (int round = 0; round < 200; ++round) {
        const int n = 1 + rng() % 12, C = 1 + rng() % 40;
        std::vector<int32_t> lens(n), order(n);
        for (int i = 0; i < n; ++i) { lens[i] = rng() % 70; order[i] = i; }
        for (int i = n - 1; i > 0; --i) std::swap(order[i], order[rng() % (i + 1)]);
        // the token stream of the scheduled prompts, cut every C tokens
        std::vector<int32_t> owner, pos;
        for (int i = 0; i < n; ++i)
            for (int t = 0; t < lens[order[i]]; ++t) { owner.push_back(order[i]); pos.push_back(t); }
        std::vector<tetri_segment> want;
        std::vector<int32_t> want_off;
        for (size_t at = 0; at < owner.size(); ++at) {
            if (at % C == 0) want_off.push_back((int32_t)want.size());
            if (at % C == 0 || owner[at] != owner[at - 1]) want.push_back({owner[at], pos[at], 0});
            ++want.back().len;
        }
        want_off.push_back((int32_t)want.size());
        int32_t n_segs = -1;
        const int32_t n_chunks = tetri_pack_chunks(lens.data(), n, order.data(), n, C, nullptr, 0, nullptr, 0, &n_segs);
        CHECK(n_chunks == (int32_t)want_off.size() - 1 && n_segs == (int32_t)want.size());
        Exact<tetri_segment> segs(n_segs);
        Exact<int32_t> offs(n_chunks + 1);
        CHECK(tetri_pack_chunks(lens.data(), n, order.data(), n, C, segs.p, n_segs, offs.p, n_chunks, nullptr) == n_chunks);
        for (int i = 0; i < n_segs; ++i)
            CHECK(segs[i].req == want[i].req && segs[i].start == want[i].start && segs[i].len == want[i].len);
        for (int c = 0; c <= n_chunks; ++c) CHECK(offs[c] == want_off[c]);
        // a capacity one too small is an error, never an overrun
        if (n_segs > 0) {
            Exact<tetri_segment> small(n_segs - 1);
            CHECK(tetri_pack_chunks(lens.data(), n, order.data(), n, C, small.p, n_segs - 1, offs.p, n_chunks, nullptr) == TETRI_ERR_NOMEM);
        }
        if (n_chunks > 0) {
            Exact<int32_t> small(n_chunks);
            CHECK(tetri_pack_chunks(lens.data(), n, order.data(), n, C, segs.p, n_segs, small.p, n_chunks - 1, nullptr) == TETRI_ERR_NOMEM);
        }
        // the whole batch's metadata in one buffer of exactly the queried length
        const int max_blocks = 1 + (70 + 15) / 16;
        std::vector<int32_t> tables((size_t)n * max_blocks);
        for (auto &x : tables) x = (int32_t)(rng() % 1000);
        int64_t meta_len = -1;
        CHECK(tetri_plan_metadata(lens.data(), n, order.data(), n, C, tables.data(), max_blocks, nullptr, 0, nullptr, 0, &meta_len) == n_chunks);
        Exact<int32_t> meta((size_t)meta_len);
        Exact<int32_t> layout((size_t)4 * n_chunks);
        CHECK(tetri_plan_metadata(lens.data(), n, order.data(), n, C, tables.data(), max_blocks, meta.p, meta_len, layout.p, n_chunks, nullptr) == n_chunks);
        for (int c = 0; c < n_chunks; ++c) {
            const int S = layout[4 * c + 3];
            CHECK(S == want_off[c + 1] - want_off[c]);
            const int32_t *cu = meta.p + layout[4 * c], *ctx = meta.p + layout[4 * c + 1], *bt = meta.p + layout[4 * c + 2];
            CHECK(cu[0] == 0 && layout[4 * c] % 4 == 0 && layout[4 * c + 1] % 4 == 0 && layout[4 * c + 2] % 4 == 0);
            for (int s = 0; s < S; ++s) {
                const tetri_segment &g = want[want_off[c] + s];
                CHECK(cu[s + 1] - cu[s] == g.len && ctx[s] == g.start);
                CHECK(std::memcmp(bt + (size_t)s * max_blocks, tables.data() + (size_t)g.req * max_blocks, sizeof(int32_t) * max_blocks) == 0);
            }
        }
        if (meta_len > 0) {
            Exact<int32_t> small((size_t)meta_len - 1);
            CHECK(tetri_plan_metadata(lens.data(), n, order.data(), n, C, tables.data(), max_blocks, small.p, meta_len - 1, layout.p, n_chunks, nullptr) == TETRI_ERR_NOMEM);
        }
        if (n_chunks > 0)
            CHECK(tetri_plan_metadata(lens.data(), n, order.data(), n, C, tables.data(), max_blocks, meta.p, meta_len, layout.p, n_chunks - 1, nullptr) == TETRI_ERR_NOMEM);
    }
    // the hand example: lengths 3, 5, 2 with ChunkSize 4
    const int32_t lens[3] = {3, 5, 2};
    tetri_segment segs[4];
    int32_t offs[4];
    CHECK(tetri_pack_chunks(lens, 3, nullptr, 3, 4, segs, 4, offs, 3, nullptr) == 3);
    const tetri_segment want[4] = {{0, 0, 3}, {1, 0, 1}, {1, 1, 4}, {2, 0, 2}};
    for (int i = 0; i < 4; ++i) CHECK(segs[i].req == want[i].req && segs[i].start == want[i].start && segs[i].len == want[i].len);
    CHECK(offs[0] == 0 && offs[1] == 2 && offs[2] == 3 && offs[3] == 4);
    // rejected inputs
    const int32_t twice[2] = {1, 1};
    CHECK(tetri_pack_chunks(lens, 3, twice, 2, 4, nullptr, 0, nullptr, 0, nullptr) == TETRI_ERR_INVALID_ARG);
    const int32_t outside[1] = {3};
    CHECK(tetri_pack_chunks(lens, 3, outside, 1, 4, nullptr, 0, nullptr, 0, nullptr) == TETRI_ERR_INVALID_ARG);
    CHECK(tetri_pack_chunks(lens, 3, nullptr, 3, 0, nullptr, 0, nullptr, 0, nullptr) == TETRI_ERR_INVALID_ARG);
    CHECK(tetri_pack_chunks(nullptr, 3, nullptr, 3, 4, nullptr, 0, nullptr, 0, nullptr) == TETRI_ERR_INVALID_ARG);
}

static void scheduler(std::mt19937 &rng)
{
    for (int round = 0; round < 100; ++round) {
        const int n = rng() % 40, batch = rng() % 12;
        Exact<int32_t> lens(n), order(n);
        for (int i = 0; i < n; ++i) lens[i] = rng() % 6;
        for (int policy = TETRI_FCFS; policy <= TETRI_LJF; ++policy) {
            CHECK(tetri_schedule(lens.p, n, policy, batch, order.p) == TETRI_OK);
            const int group = batch > 0 ? batch : (n > 0 ? n : 1);
            std::vector<char> seen(n, 0);
            for (int i = 0; i < n; ++i) {
                CHECK(order[i] >= 0 && order[i] < n && !seen[order[i]]);
                seen[order[i]] = 1;
                CHECK(order[i] / group == i / group);                  // groups are never interleaved
                if (i % group == 0) continue;
                const int a = order[i - 1], b = order[i];
                if (policy == TETRI_FCFS) CHECK(a < b);
                if (policy == TETRI_SJF) CHECK(lens[a] < lens[b] || (lens[a] == lens[b] && a < b));
                if (policy == TETRI_LJF) CHECK(lens[a] > lens[b] || (lens[a] == lens[b] && a < b));
            }
        }
    }
    int32_t one = 1, out = 0;
    CHECK(tetri_schedule(&one, 1, 7, 0, &out) == TETRI_ERR_INVALID_ARG);
    CHECK(tetri_schedule(nullptr, 1, TETRI_SJF, 0, &out) == TETRI_ERR_INVALID_ARG);
}

static void oracle_on_exact_buffers(std::mt19937 &rng)
{
    std::normal_distribution<float> gauss(0.f, 1.f);
    for (int round = 0; round < 12; ++round) {
        const int P = round % 3 == 0 ? 1 : 16, D = round % 2 ? 64 : 128, Hkv = 1 + rng() % 3, g = 1 + rng() % 3, Hq = Hkv * g;
        const int S = 1 + rng() % 3, C = 40;
        Exact<int32_t> cu(S + 1), ctx(S);
        cu[0] = 0;
        int pages_needed = 0, max_blocks = 0;
        for (int s = 0; s < S; ++s) {
            const int n = 1 + rng() % (C / S);
            cu[s + 1] = cu[s] + n;
            ctx[s] = rng() % 50;
            const int blocks = (ctx[s] + n + P - 1) / P;
            pages_needed += blocks;
            max_blocks = blocks > max_blocks ? blocks : max_blocks;
        }
        const int num_pages = pages_needed;                        // every page is used: no spare page to overrun into
        Exact<int32_t> bt((size_t)S * max_blocks);
        std::vector<int32_t> perm(num_pages);
        for (int i = 0; i < num_pages; ++i) perm[i] = i;
        for (int i = num_pages - 1; i > 0; --i) std::swap(perm[i], perm[rng() % (i + 1)]);
        int at = 0;
        for (int s = 0; s < S; ++s)
            for (int b = 0; b < max_blocks; ++b)
                bt[(size_t)s * max_blocks + b] = b < (ctx[s] + cu[s + 1] - cu[s] + P - 1) / P ? perm[at++] : 0;
        const size_t pool_n = (size_t)num_pages * 2 * Hkv * P * D;
        Exact<float> q((size_t)C * Hq * D), k((size_t)C * Hkv * D), v((size_t)C * Hkv * D), pool(pool_n), out((size_t)C * Hq * D);
        for (size_t i = 0; i < q.n; ++i) q[i] = gauss(rng);
        for (size_t i = 0; i < k.n; ++i) { k[i] = round % 4 == 1 ? 0.f : gauss(rng); v[i] = gauss(rng); }
        for (size_t i = 0; i < pool_n; ++i) pool[i] = round % 4 == 1 ? 0.f : gauss(rng);
        const float scale = 1.0f / std::sqrt((float)D);
        CHECK(oracle_chunk_prefill_attn(q.p, k.p, v.p, pool.p, bt.p, cu.p, ctx.p, S, C, Hq, Hkv, D, P, max_blocks, scale, out.p) == 0);
        for (int s = 0; s < S; ++s) {
            const int n = cu[s + 1] - cu[s];
            for (int h = 0; h < Hq; ++h) {
                const int kh = h / g;
                if (ctx[s] == 0)                                   // the first token of a request returns its own V
                    for (int d = 0; d < D; ++d)
                        CHECK(out[((size_t)cu[s] * Hq + h) * D + d] == v[((size_t)cu[s] * Hkv + kh) * D + d]);
                // the softmax weights of the segment's last row are a distribution and reproduce its output
                const int r = cu[s + 1] - 1, p = ctx[s] + n - 1;
                Exact<double> probs((size_t)ctx[s] + n);
                CHECK(oracle_attn_row_probs(q.p, k.p, v.p, pool.p, bt.p, cu.p, ctx.p, S, Hq, Hkv, D, P, max_blocks, scale, r, h, probs.p) == p + 1);
                double sum = 0;
                for (int j = 0; j <= p; ++j) { CHECK(probs[j] >= 0); sum += probs[j]; }
                CHECK(std::fabs(sum - 1.0) < 1e-9);
                if (round % 4 == 1)                                // zero keys: uniform weights
                    for (int j = 0; j <= p; ++j) CHECK(std::fabs(probs[j] - 1.0 / (p + 1)) < 1e-12);
            }
        }
        for (size_t i = (size_t)cu[S] * Hq * D; i < out.n; ++i) CHECK(out[i] == 0.f);
        // sampled rows are the same rows
        const int ns = 5;
        Exact<int32_t> rows(ns), heads(ns);
        Exact<float> smp((size_t)ns * D);
        for (int i = 0; i < ns; ++i) { rows[i] = rng() % C; heads[i] = rng() % Hq; }
        CHECK(oracle_chunk_prefill_attn_samples(q.p, k.p, v.p, pool.p, bt.p, cu.p, ctx.p, S, Hq, Hkv, D, P, max_blocks, scale, rows.p, heads.p, ns, smp.p) == 0);
        for (int i = 0; i < ns; ++i)
            CHECK(std::memcmp(smp.p + (size_t)i * D, out.p + ((size_t)rows[i] * Hq + heads[i]) * D, sizeof(float) * D) == 0);
        // append: 16-bit elements into a sentinel-filled pool; every row found where the table says, the rest untouched
        Exact<uint16_t> k16(k.n), v16(v.n), pool16(pool_n);
        for (size_t i = 0; i < k.n; ++i) { k16[i] = (uint16_t)(rng() | 1); v16[i] = (uint16_t)(rng() | 1); }
        for (size_t i = 0; i < pool_n; ++i) pool16[i] = 0;
        CHECK(oracle_kv_append(k16.p, v16.p, pool16.p, bt.p, cu.p, ctx.p, S, Hkv, D, P, max_blocks, 2) == 0);
        size_t nonzero = 0;
        for (size_t i = 0; i < pool_n; ++i) nonzero += pool16[i] != 0;
        CHECK(nonzero == (size_t)cu[S] * 2 * Hkv * D);
        for (int s = 0; s < S; ++s)
            for (int t = 0; t < cu[s + 1] - cu[s]; ++t) {
                const int pos = ctx[s] + t, page = bt[(size_t)s * max_blocks + pos / P], slot = pos % P;
                for (int kh = 0; kh < Hkv; ++kh) {
                    const size_t src = ((size_t)(cu[s] + t) * Hkv + kh) * D;
                    const size_t dk = ((((size_t)page * 2 + 0) * Hkv + kh) * P + slot) * D, dv = ((((size_t)page * 2 + 1) * Hkv + kh) * P + slot) * D;
                    CHECK(std::memcmp(pool16.p + dk, k16.p + src, 2 * D) == 0 && std::memcmp(pool16.p + dv, v16.p + src, 2 * D) == 0);
                }
            }
    }
}

int main()
{
    std::mt19937 rng(20240111);
    packer_against_token_stream(rng);
    scheduler(rng);
    oracle_on_exact_buffers(rng);
    if (g_failed) {
        std::fprintf(stderr, "sanitize_host: %d check(s) failed\n", g_failed);
        return 1;
    }
    std::puts("sanitize_host: ok");
    return 0;
}
