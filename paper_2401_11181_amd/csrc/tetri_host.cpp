// Host layer of libtetri: handle, argument checks, launch shapes and the debug validator.
// (The chunk packer and the scheduler are in tetri_plan.cpp, which needs no HIP.)
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "tetri_internal.h"
#include "tetri_plan.h"

namespace {

tetri_status fail(tetri_ctx *h, tetri_status st, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (h) h->err = buf; else tetri_set_thread_error(buf);
    return st;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Query-head grouping of a workgroup: its 4 row/head slots are
// (hpw heads that share a kv head) x (rb blocks of 32 rows).
void wave_grouping(int g, int *hpw, int *rb)
{
    if (g % 4 == 0) *hpw = 4;
    else if (g % 2 == 0) *hpw = 2;
    else *hpw = 1;
    *rb = 4 / *hpw;
}

// Upper bound of the number of row tiles of a chunk: each of the S segments and the padding
// range may end in a partial tile.
int tile_bound(int C, int S, int BM) { return (C + (S + 1) * (BM - 1)) / BM; }

}  // namespace

extern "C" {

int32_t tetri_abi_version(void) { return 1; }

const char *tetri_last_error(const tetri_ctx *ctx)
{
    return ctx ? ctx->err.c_str() : tetri_thread_error();
}

tetri_status tetri_create(const tetri_config *c, tetri_ctx **out)
{
    if (!c || !out) return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_create: null argument");
    *out = nullptr;
    if (c->num_q_heads < 1 || c->num_kv_heads < 1 || c->num_q_heads % c->num_kv_heads != 0)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_create: num_q_heads=%d must be a positive multiple of num_kv_heads=%d",
                    c->num_q_heads, c->num_kv_heads);
    if (c->chunk_size < 1 || c->num_pages < 1 || c->max_blocks_per_seq < 1 || c->max_segs_per_chunk < 1)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_create: chunk_size, num_pages, max_blocks_per_seq and max_segs_per_chunk must be positive");
    if (c->max_segs_per_chunk > c->chunk_size)
        return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_create: max_segs_per_chunk=%d exceeds chunk_size=%d (segments are non-empty)",
                    c->max_segs_per_chunk, c->chunk_size);
    if (c->head_dim != 64 && c->head_dim != 128)
        return fail(nullptr, TETRI_ERR_UNSUPPORTED, "tetri_create: head_dim=%d (supported: 64, 128)", c->head_dim);
    if (c->page_size != 16)
        return fail(nullptr, TETRI_ERR_UNSUPPORTED, "tetri_create: page_size=%d (supported: 16)", c->page_size);
    if (c->dtype != TETRI_BF16)
        return fail(nullptr, TETRI_ERR_UNSUPPORTED, "tetri_create: dtype=%d (supported: TETRI_BF16)", c->dtype);
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev < 1)
        return fail(nullptr, TETRI_ERR_HIP, "tetri_create: no usable HIP device (%s)", e == hipSuccess ? "device count is 0" : hipGetErrorString(e));
    tetri_ctx *h = new (std::nothrow) tetri_ctx;
    if (!h) return fail(nullptr, TETRI_ERR_NOMEM, "tetri_create: out of host memory");
    h->cfg = *c;
    // Scratch memory for launches that divide the stages of a head group evenly over workgroups: such
    // a launch has at most one workgroup per CU, 4 (row block, head) slots each, and a workgroup leaves at
    // most two partial results per slot (its first and its last job); a partial result is O (32 x head_dim
    // floats), m and the row sum.  Arrival counters: one per (head group, row tile, slot), fewer than two
    // tiles per CU in such a launch; two sets, because every such launch uses one set and zeroes the other
    // for the launch after it.
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&h->device)) != hipSuccess || (e = hipGetDeviceProperties(&prop, h->device)) != hipSuccess) {
        delete h;
        return fail(nullptr, TETRI_ERR_HIP, "tetri_create: %s", hipGetErrorString(e));
    }
    h->num_cus = prop.multiProcessorCount;
    h->scratch_units = (size_t)h->num_cus * 4;
    h->unit_bytes = (size_t)32 * c->head_dim * 4 + 2 * 32 * 4;
    h->n_counters = (int32_t)(2 * h->scratch_units);
    if ((e = hipMalloc(reinterpret_cast<void **>(&h->scratch), 2 * h->scratch_units * h->unit_bytes)) != hipSuccess ||
        (e = hipMalloc(reinterpret_cast<void **>(&h->counters), 2 * (size_t)h->n_counters * sizeof(int32_t))) != hipSuccess ||
        (e = hipMemset(h->counters, 0, 2 * (size_t)h->n_counters * sizeof(int32_t))) != hipSuccess) {
        tetri_destroy(h);
        return fail(nullptr, TETRI_ERR_HIP, "tetri_create: scratch memory: %s", hipGetErrorString(e));
    }
    // the static scratch array of tetri_decode_attn_static: its address on this device, looked up here so that the
    // entry point itself makes no runtime call besides the launch
    if ((e = tetri_decode_static_scratch(&h->static_scratch, &h->static_scratch_bytes)) != hipSuccess) {
        tetri_destroy(h);
        return fail(nullptr, TETRI_ERR_HIP, "tetri_create: static scratch array: %s", hipGetErrorString(e));
    }
    *out = h;
    return TETRI_OK;
}

void tetri_destroy(tetri_ctx *ctx)
{
    if (!ctx) return;
    if (ctx->scratch) (void)hipFree(ctx->scratch);
    if (ctx->counters) (void)hipFree(ctx->counters);
    delete ctx;
}

tetri_status tetri_set_option(tetri_ctx *ctx, const char *key, int32_t value)
{
    if (!ctx || !key) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: null argument");
    if (std::strcmp(key, "split_keys") == 0) {
        if (value < 0 || value > 1) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: split_keys=%d (0 or 1)", value);
        ctx->split_keys = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "split_min_stages") == 0) {
        if (value < 2) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: split_min_stages=%d (at least 2)", value);
        ctx->split_min_stages = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "split_bias_stages") == 0) {
        if (value < 0) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: split_bias_stages=%d (not negative)", value);
        ctx->split_bias_stages = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "split_share_q8") == 0) {
        if (value < 1 || value > 128) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: split_share_q8=%d (1..128)", value);
        ctx->split_share_q8 = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "stream_wgs") == 0) {
        if (value < 0 || value > 255) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: stream_wgs=%d (0..255)", value);
        ctx->stream_wgs = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "decode_parts") == 0) {
        if (value < 0) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: decode_parts=%d (>= 0)", value);
        ctx->decode_parts = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "transfer_slabs") == 0) {
        if (value < 0) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: transfer_slabs=%d (>= 0)", value);
        ctx->transfer_slabs = value;
        return TETRI_OK;
    }
    if (std::strcmp(key, "attn_variant") == 0) {
        if (value < 0 || value > 2) return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: attn_variant=%d unknown", value);
        ctx->attn_variant = value;
        return TETRI_OK;
    }
    return fail(ctx, TETRI_ERR_INVALID_ARG, "tetri_set_option: unknown key '%s'", key);
}

static tetri_status check_common(tetri_ctx *h, const char *fn, const void *const *ptrs, const char *const *names, int n,
                                 int32_t num_segs)
{
    if (!h) return fail(nullptr, TETRI_ERR_INVALID_ARG, "%s: null handle", fn);
    for (int i = 0; i < n; ++i) {
        if (!ptrs[i]) return fail(h, TETRI_ERR_INVALID_ARG, "%s: %s is null", fn, names[i]);
        if (!aligned16(ptrs[i])) return fail(h, TETRI_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", fn, names[i]);
    }
    if (num_segs < 1 || num_segs > h->cfg.max_segs_per_chunk)
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: num_segs=%d outside 1..%d", fn, num_segs, h->cfg.max_segs_per_chunk);
    return TETRI_OK;
}

tetri_status tetri_kv_append(tetri_ctx *h, const void *k_new, const void *v_new, void *kv_pages,
                             const int32_t *block_table, const int32_t *cu, const int32_t *ctx_lens,
                             int32_t num_segs, void *stream)
{
    const void *ptrs[] = {k_new, v_new, kv_pages};
    const char *names[] = {"k_new", "v_new", "kv_pages"};
    tetri_status st = check_common(h, "tetri_kv_append", ptrs, names, 3, num_segs);
    if (st != TETRI_OK) return st;
    if (!block_table || !cu || !ctx_lens) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_kv_append: null metadata pointer");
    AppendParams p;
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.pages = static_cast<uint16_t *>(kv_pages);
    p.bt = block_table; p.cu = cu; p.ctx = ctx_lens;
    p.S = num_segs; p.Hkv = h->cfg.num_kv_heads; p.D = h->cfg.head_dim; p.max_blocks = h->cfg.max_blocks_per_seq;
    hipError_t e = tetri_launch_append(h, p, h->cfg.chunk_size, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(h, TETRI_ERR_HIP, "tetri_kv_append: launch failed: %s", hipGetErrorString(e));
    return TETRI_OK;
}

// mode 0: 16-bit pool <-> 16-bit buffer; 1: 16-bit pool -> buffer of FP8 codes (quantising);
// 2: FP8 pool <-> buffer of FP8 codes (bytes)
static tetri_status kv_transfer(const char *fn, tetri_ctx *h, void *kv_pages, void *buf, const int32_t *block_table,
                                const int32_t *cu_tokens, const int32_t *first_tokens, int32_t num_reqs,
                                int64_t total_tokens, bool to_pool, void *stream, int mode = 0, float k_scale = 1.f,
                                float v_scale = 1.f)
{
    if (!h) return fail(nullptr, TETRI_ERR_INVALID_ARG, "%s: null handle", fn);
    if (!kv_pages || !aligned16(kv_pages)) return fail(h, TETRI_ERR_INVALID_ARG, "%s: kv_pages is null or not 16-byte aligned", fn);
    if (!block_table || !cu_tokens) return fail(h, TETRI_ERR_INVALID_ARG, "%s: null metadata pointer", fn);
    if (num_reqs < 1 || num_reqs > (1 << 20)) return fail(h, TETRI_ERR_INVALID_ARG, "%s: num_reqs=%d outside 1..%d", fn, num_reqs, 1 << 20);
    const int64_t most = (int64_t)num_reqs * h->cfg.max_blocks_per_seq * h->cfg.page_size;
    if (total_tokens < 0 || total_tokens > most)
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: total_tokens=%lld outside 0..%lld (num_reqs block-table rows)", fn,
                    (long long)total_tokens, (long long)most);
    if (total_tokens == 0) return TETRI_OK;
    if (!buf || !aligned16(buf)) return fail(h, TETRI_ERR_INVALID_ARG, "%s: buf is null or not 16-byte aligned", fn);
    if (mode == 1 && !(std::isfinite(k_scale) && std::isfinite(v_scale) && k_scale > 0.f && v_scale > 0.f))
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: k_scale and v_scale must be positive and finite", fn);
    // 16-bit units of a row as the kernel moves it: an FP8 row of head_dim codes is head_dim / 2 units
    const int32_t row_units = mode == 2 ? h->cfg.head_dim / 2 : h->cfg.head_dim;
    const int64_t tile_tokens = 2048 / row_units;           // a workgroup's tile: 256 lanes of 16 bytes per slab
    const int64_t tiles = total_tokens / tile_tokens + num_reqs;     // >= sum of ceil(n_r / tile_tokens)
    if (tiles > 0x7fffffff) return fail(h, TETRI_ERR_INVALID_ARG, "%s: too many tokens for one launch", fn);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device)
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: the handle was created on device %d, the current device is %d", fn, h->device, dev);
    TransferParams p;
    p.pool = static_cast<uint16_t *>(kv_pages);
    p.buf = static_cast<uint16_t *>(buf);
    p.bt = block_table; p.cu = cu_tokens; p.first = first_tokens;
    p.R = num_reqs; p.Hkv = h->cfg.num_kv_heads; p.max_blocks = h->cfg.max_blocks_per_seq;
    // enough workgroups for eight per compute unit (a short transfer is bound by the latency of each
    // workgroup's look-ups, so it wants them all resident at once); beyond that a workgroup takes several slabs, amortises
    // its page lookups over them and keeps the next slab's loads in flight behind the current one's stores
    const int64_t slabs = 2 * (int64_t)p.Hkv;
    const int64_t want = 8 * (int64_t)std::max(h->num_cus, 1);
    p.slabs_per_wg = (int32_t)std::min<int64_t>(slabs, std::max<int64_t>(1, tiles * slabs / want));
    if (h->transfer_slabs > 0) p.slabs_per_wg = (int32_t)std::min<int64_t>(slabs, h->transfer_slabs);
    p.k_inv = 1.0f / k_scale; p.v_inv = 1.0f / v_scale;
    hipError_t e = mode == 1 ? tetri_launch_kv_export_fp8(h, p, (int32_t)tiles, static_cast<hipStream_t>(stream))
                             : tetri_launch_kv_transfer(h, p, row_units, (int32_t)tiles, to_pool, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(h, TETRI_ERR_HIP, "%s: launch failed: %s", fn, hipGetErrorString(e));
    return TETRI_OK;
}

tetri_status tetri_kv_export_fp8(tetri_ctx *h, const void *kv_pages, const int32_t *block_table, const int32_t *cu_tokens,
                                 const int32_t *first_tokens, int32_t num_reqs, int64_t total_tokens, float k_scale,
                                 float v_scale, void *buf, void *stream)
{
    return kv_transfer("tetri_kv_export_fp8", h, const_cast<void *>(kv_pages), buf, block_table, cu_tokens, first_tokens,
                       num_reqs, total_tokens, false, stream, 1, k_scale, v_scale);
}

tetri_status tetri_kv_import_fp8(tetri_ctx *h, const void *buf, const int32_t *block_table, const int32_t *cu_tokens,
                                 const int32_t *first_tokens, int32_t num_reqs, int64_t total_tokens, void *kv_pages_fp8,
                                 void *stream)
{
    return kv_transfer("tetri_kv_import_fp8", h, kv_pages_fp8, const_cast<void *>(buf), block_table, cu_tokens,
                       first_tokens, num_reqs, total_tokens, true, stream, 2);
}

tetri_status tetri_kv_export(tetri_ctx *h, const void *kv_pages, const int32_t *block_table, const int32_t *cu_tokens,
                             const int32_t *first_tokens, int32_t num_reqs, int64_t total_tokens, void *buf, void *stream)
{
    return kv_transfer("tetri_kv_export", h, const_cast<void *>(kv_pages), buf, block_table, cu_tokens, first_tokens,
                       num_reqs, total_tokens, false, stream);
}

tetri_status tetri_kv_import(tetri_ctx *h, const void *buf, const int32_t *block_table, const int32_t *cu_tokens,
                             const int32_t *first_tokens, int32_t num_reqs, int64_t total_tokens, void *kv_pages, void *stream)
{
    return kv_transfer("tetri_kv_import", h, kv_pages, const_cast<void *>(buf), block_table, cu_tokens, first_tokens,
                       num_reqs, total_tokens, true, stream);
}

static tetri_status decode_common(const char *fn, tetri_ctx *h, const void *q, const void *k_new, const void *v_new,
                                  const void *kv_pages, void *kv_pages_w, const int32_t *block_table,
                                  const int32_t *ctx_lens, int32_t num_reqs, int32_t max_ctx_len, float scale, void *out,
                                  void *stream, bool fp8 = false, float k_scale = 1.f, float v_scale = 1.f,
                                  bool static_scratch = false)
{
    if (!h) return fail(nullptr, TETRI_ERR_INVALID_ARG, "%s: null handle", fn);
    const void *ptrs[] = {q, k_new, v_new, kv_pages, out};
    const char *names[] = {"q", "k_new", "v_new", "kv_pages", "out"};
    for (int i = 0; i < 5; ++i) {
        if (!ptrs[i]) return fail(h, TETRI_ERR_INVALID_ARG, "%s: %s is null", fn, names[i]);
        if (!aligned16(ptrs[i])) return fail(h, TETRI_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", fn, names[i]);
    }
    if (!block_table || !ctx_lens) return fail(h, TETRI_ERR_INVALID_ARG, "%s: null metadata pointer", fn);
    if (!std::isfinite(scale)) return fail(h, TETRI_ERR_INVALID_ARG, "%s: scale is not finite", fn);
    const tetri_config &cfg = h->cfg;
    if (num_reqs < 1 || (int64_t)num_reqs * cfg.num_kv_heads > (1 << 24))
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: num_reqs=%d outside 1..%d", fn, num_reqs, (1 << 24) / cfg.num_kv_heads);
    // with the fused append the new token itself needs a slot
    const int64_t most = (int64_t)cfg.max_blocks_per_seq * cfg.page_size - (kv_pages_w ? 1 : 0);
    if (max_ctx_len < 0 || max_ctx_len > most)
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: max_ctx_len=%d outside 0..%lld", fn, max_ctx_len, (long long)most);
    if (cfg.num_q_heads / cfg.num_kv_heads > 32)
        return fail(h, TETRI_ERR_UNSUPPORTED, "%s: more than 32 query heads per kv head", fn);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device)
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: the handle was created on device %d, the current device is %d", fn, h->device, dev);
    DecodeParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.pages = static_cast<const uint16_t *>(kv_pages);
    p.bt = block_table; p.ctx = ctx_lens;
    p.out = static_cast<uint16_t *>(out);
    p.pages_w = static_cast<uint16_t *>(kv_pages_w);
    p.partial = static_scratch ? h->static_scratch : reinterpret_cast<float *>(h->scratch);
    p.B = num_reqs; p.Hq = cfg.num_q_heads; p.Hkv = cfg.num_kv_heads; p.g = p.Hq / p.Hkv;
    p.max_blocks = cfg.max_blocks_per_seq;
    p.c = std::fmax(std::fabs(scale) * 1.4426950408889634f, 1e-30f);
    p.neg = scale < 0.f;
    if (fp8 && !(std::isfinite(k_scale) && std::isfinite(v_scale) && k_scale > 0.f && v_scale > 0.f))
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: k_scale and v_scale must be positive and finite", fn);
    p.fp8 = fp8;
    p.k_scale = k_scale; p.v_scale = v_scale;
    p.k_inv = 1.0f / k_scale; p.v_inv = 1.0f / v_scale;
    p.out_scale = fp8 ? v_scale : 1.0f;
    // Few requests: split every request's keys over several workgroups until the device has four
    // workgroups per compute unit, each with at least eight 32-key steps, as far as the scratch
    // memory for the parts reaches.
    const int64_t pairs = (int64_t)num_reqs * p.Hkv;
    const int64_t steps = ((int64_t)max_ctx_len + 32) / 32;
    const int64_t per_part = (int64_t)num_reqs * p.Hq * (cfg.head_dim + 2) * 4;        // scratch bytes of one part
    const int64_t room = static_scratch ? (int64_t)h->static_scratch_bytes : (int64_t)(2 * h->scratch_units * h->unit_bytes);
    if (static_scratch && 2 * per_part > room)
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: num_reqs x num_q_heads = %lld exceeds what the static scratch array of %lld bytes "
                    "holds (two parts of head_dim + 2 floats per request and head: at most %lld)", fn,
                    (long long)num_reqs * cfg.num_q_heads, (long long)room, (long long)(room / (2 * (cfg.head_dim + 2) * 4)));
    const int64_t fit = room / per_part;
    int64_t parts = (4 * (int64_t)std::max(h->num_cus, 1) + pairs - 1) / pairs;
    parts = std::min(parts, std::max<int64_t>(1, steps / 8));
    if (h->decode_parts > 0) parts = h->decode_parts;
    parts = std::max<int64_t>(1, std::min(parts, std::min<int64_t>(fit, 1024)));
    p.parts = (int32_t)parts;
    if (pairs * parts > 0x7fffffff) return fail(h, TETRI_ERR_INVALID_ARG, "%s: too many workgroups", fn);
    hipError_t e = tetri_launch_decode(h, p, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(h, TETRI_ERR_HIP, "%s: launch failed: %s", fn, hipGetErrorString(e));
    return TETRI_OK;
}

tetri_status tetri_decode_attn(tetri_ctx *h, const void *q, const void *k_new, const void *v_new, const void *kv_pages,
                               const int32_t *block_table, const int32_t *ctx_lens, int32_t num_reqs, int32_t max_ctx_len,
                               float scale, void *out, void *stream)
{
    return decode_common("tetri_decode_attn", h, q, k_new, v_new, kv_pages, nullptr, block_table, ctx_lens, num_reqs,
                         max_ctx_len, scale, out, stream);
}

tetri_status tetri_decode_attn_static(tetri_ctx *h, const void *q, const void *k_new, const void *v_new, const void *kv_pages,
                                      const int32_t *block_table, const int32_t *ctx_lens, int32_t num_reqs, int32_t max_ctx_len,
                                      float scale, void *out, void *stream)
{
    return decode_common("tetri_decode_attn_static", h, q, k_new, v_new, kv_pages, nullptr, block_table, ctx_lens, num_reqs,
                         max_ctx_len, scale, out, stream, false, 1.f, 1.f, true);
}

tetri_status tetri_decode_attn_fp8(tetri_ctx *h, const void *q, const void *k_new, const void *v_new, void *kv_pages_fp8,
                                   const int32_t *block_table, const int32_t *ctx_lens, int32_t num_reqs,
                                   int32_t max_ctx_len, float scale, float k_scale, float v_scale, int32_t append,
                                   void *out, void *stream)
{
    if (append != 0 && append != 1) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_decode_attn_fp8: append must be 0 or 1");
    return decode_common("tetri_decode_attn_fp8", h, q, k_new, v_new, kv_pages_fp8, append ? kv_pages_fp8 : nullptr,
                         block_table, ctx_lens, num_reqs, max_ctx_len, scale, out, stream, true, k_scale, v_scale);
}

tetri_status tetri_decode_attn_append(tetri_ctx *h, const void *q, const void *k_new, const void *v_new, void *kv_pages,
                                      const int32_t *block_table, const int32_t *ctx_lens, int32_t num_reqs,
                                      int32_t max_ctx_len, float scale, void *out, void *stream)
{
    return decode_common("tetri_decode_attn_append", h, q, k_new, v_new, kv_pages, kv_pages, block_table, ctx_lens,
                         num_reqs, max_ctx_len, scale, out, stream);
}

static tetri_status attn_common(const char *fn, tetri_ctx *h, const void *q, const void *k_new, const void *v_new,
                                const void *kv_pages, void *kv_pages_w, const int32_t *block_table, const int32_t *cu,
                                const int32_t *ctx_lens, int32_t num_segs, float scale, void *out, void *stream,
                                bool fp8 = false, float k_scale = 1.f, float v_scale = 1.f)
{
    const void *ptrs[] = {q, k_new, v_new, kv_pages, out};
    const char *names[] = {"q", "k_new", "v_new", "kv_pages", "out"};
    tetri_status st = check_common(h, fn, ptrs, names, 5, num_segs);
    if (st != TETRI_OK) return st;
    if (!block_table || !cu || !ctx_lens) return fail(h, TETRI_ERR_INVALID_ARG, "%s: null metadata pointer", fn);
    if (!std::isfinite(scale)) return fail(h, TETRI_ERR_INVALID_ARG, "%s: scale is not finite", fn);
    if (fp8 && !(std::isfinite(k_scale) && std::isfinite(v_scale) && k_scale > 0.f && v_scale > 0.f))
        return fail(h, TETRI_ERR_INVALID_ARG, "%s: k_scale and v_scale must be positive and finite", fn);
    AttnParams p;
    p.k_scale = k_scale; p.v_scale = v_scale;
    p.k_inv = 1.0f / k_scale; p.v_inv = 1.0f / v_scale;
    p.q = static_cast<const uint16_t *>(q);
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.pages = static_cast<const uint16_t *>(kv_pages);
    p.pages_w = static_cast<uint16_t *>(kv_pages_w);
    p.bt = block_table; p.cu = cu; p.ctx = ctx_lens;
    p.out = static_cast<uint16_t *>(out);
    p.S = num_segs; p.C = h->cfg.chunk_size; p.Hq = h->cfg.num_q_heads; p.Hkv = h->cfg.num_kv_heads;
    p.g = p.Hq / p.Hkv;
    p.max_blocks = h->cfg.max_blocks_per_seq;
    // scale == 0 is run as a tiny positive scale: every finite score then maps to weight 1 exactly,
    // while masked scores (-inf) still map to weight 0
    p.c = std::fmax(std::fabs(scale) * 1.4426950408889634f, 1e-30f);
    p.neg = scale < 0.f;
    wave_grouping(p.g, &p.hpw, &p.rb);
    const int groups = p.Hq / p.hpw;
    const int cus = std::max(h->num_cus, 1);
    // Workgroup size of the shared-tile kernel.  A full chunk has at least C / (rows of a tile) tiles per head
    // group; when that alone gives five workgroups per four compute units or more, four-wavefront workgroups (two
    // to a CU, their barriers independent of each other), one per tile, do best: with two per CU everywhere they run
    // the block loop 4-15 % faster than eight-wavefront ones, and at 1.25 per CU (ChunkSize 1024 at 40 heads)
    // still 4 % faster than eight-wavefront workgroups that divide the stages of a head among them.  On smaller
    // launches the eight-wavefront workgroup, which puts twice the wavefronts on its tile's CU, is the better one.
    int key_parts = h->attn_variant == 1 ? 1 : 2;
    if (h->attn_variant == 0 && h->stream_wgs == 0 && (int64_t)(p.C / (32 * p.rb)) * groups * 4 >= 5 * (int64_t)cus) key_parts = 1;
    p.tiles = tile_bound(p.C, p.S, 32 * p.rb);
    p.gpx = (groups + 7) / 8;
    // How the work of a head group is handed out (see the kernel):
    //  - tail mode: a launch whose row tiles would occupy at most two thirds of the compute units gets one more
    //    workgroup per two tiles, which takes the tails of their key ranges; all tiles of a head start together and
    //    walk the keys side by side, so K and V come out of L2 for all but the first of them;
    //  - stream mode: a launch with more tiles than that but fewer than five per four compute units gives every head
    //    group G workgroups that share the stages of all its tiles evenly (measured: better than a second, mostly
    //    empty round of eight-wavefront workgroups, worse than tail mode where that applies: workgroups of a head
    //    then read different parts of K and V at any one time);
    //  - tile mode: one workgroup per row tile (launches with more tiles than that: four-wavefront workgroups).
    // The divisions are worked out on the device from the segment lengths; the host only has to know that
    // the numbers fit: scratch memory and arrival counters for every (tile, slot) resp. (workgroup, slot), and for
    // stream mode at most 64 segments (one lane each) and positions times G in 31 bits.
    int G = 0;
    p.helpers = 0;
    const bool counters_fit = (int64_t)groups * p.tiles * 4 <= h->n_counters;
    if (h->stream_wgs > 0) {
        G = h->stream_wgs;
    } else if (h->split_keys) {
        const int helpers = p.tiles / 2 + 1;
        // (the last tile of the bound and its helper exist only in chunks with ragged segments and are not counted)
        if (p.tiles >= 2 && (int64_t)(p.tiles - 1 + helpers - 1) * groups <= cus && (size_t)p.tiles * groups * 4 <= h->scratch_units)
            p.helpers = helpers;
        // (segments of under 256 rows on average are a batch of short prompts: a handful of stages per tile, which
        // the division would only cut into smaller pieces)
        else if ((key_parts == 2 || h->attn_variant == 1) && (int64_t)p.tiles * groups < 2 * (int64_t)cus && (int64_t)p.C >= 256 * (int64_t)p.S)
            G = std::min(255, (cus - (kv_pages_w ? 8 : 0)) / groups);
    }
    const int stage = 64 * key_parts;
    const int64_t stage_bound = (int64_t)p.tiles * (((int64_t)p.max_blocks * 16 + p.C) / stage + 2);
    if (G > 0 && (p.S > 64 || stage_bound * (G + 1) >= 0x7fffffffll || (size_t)groups * G * 4 > h->scratch_units || !counters_fit))
        G = 0;
    if (!counters_fit) p.helpers = 0;
    const bool shares = G > 0 || p.helpers > 0;         // the launch uses the handle's scratch memory and counters
    hipStream_t hs = static_cast<hipStream_t>(stream);
    // (a stream that is being captured into a graph takes no event queries or records: the graph orders its nodes)
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    const bool capturing = shares && (hipStreamIsCapturing(hs, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone);
    if (shares) {
        // the scratch memory lives on the device the handle was created on
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess || dev != h->device)
            return fail(h, TETRI_ERR_INVALID_ARG, "%s: the current device is %d, the handle was created on device %d", fn, dev, h->device);
        // such launches share the handle's scratch memory and counters: one on another stream must not start
        // before the previous one has ended.  (Asked of the stream, not of an event behind the launch: recording
        // an event per launch costs several microseconds of queue time between 20-us kernels.)
        if (!capturing && h->divide_launched && h->last_divide_stream != hs && hipStreamQuery(h->last_divide_stream) == hipErrorNotReady)
            return fail(h, TETRI_ERR_INVALID_ARG, "%s: the stream of this handle's previous launch that uses its scratch memory still has work "
                        "pending; launches on one handle must not overlap (use one handle per stream)", fn);
    }
    p.stream_wgs = G;
    // (in tail mode the bound's last tile and its helper are extra jobs of existing workgroups)
    p.attn_grid = 8 * p.gpx * (G > 0 ? G : (p.helpers > 0 ? p.tiles + p.helpers - 2 : p.tiles));
    p.attn_first = p.attn_grid;
    // fused append: a few dozen workgroups, each copying every 64th row of the chunk
    // (every eight-wavefront workgroup of this kernel occupies a whole CU: in stream mode only the CUs the
    // attention workgroups leave free take append workgroups right away)
    int append_wgs = 64;
    if (shares) {
        const int idle = cus - p.attn_first;
        append_wgs = idle >= 8 ? (idle < 64 ? idle / 8 * 8 : 64) : 8;
    }
    p.append_blocks = kv_pages_w ? (p.C < append_wgs ? p.C : append_wgs) : 0;
    // divisions the kernel does by launch constants, as multiplications
    auto magic = [](uint32_t d) -> uint32_t { return d <= 1 ? 0u : (uint32_t)((0x100000000ull + d - 1) / d); };
    auto log2i = [](int v) { int s = 0; while ((1 << s) < v) ++s; return s; };
    p.hpw_shift = log2i(p.hpw);
    p.rb_shift = log2i(p.rb);
    p.groups = groups;
    p.gpx_magic = magic((uint32_t)p.gpx);
    p.tail_q8 = h->split_share_q8;
    p.split_min = h->split_min_stages;
    p.split_bias = h->split_bias_stages;
    p.scratch = h->scratch;
    p.n_counters = h->n_counters;
    p.counters = h->counters + (size_t)h->counter_set * h->n_counters;
    p.counters_next = h->counters + (size_t)(1 - h->counter_set) * h->n_counters;
    p.kv_magic = magic((uint32_t)(p.g / p.hpw));
    if ((uint64_t)p.attn_grid * (uint64_t)(p.tiles + G + 1) >= 0x100000000ull)
        return fail(h, TETRI_ERR_UNSUPPORTED, "%s: chunk_size x heads too large for one launch", fn);
    hipError_t e = tetri_launch_attn(h, p, key_parts, fp8, hs);
    if (e != hipSuccess) return fail(h, TETRI_ERR_HIP, "%s: launch failed: %s", fn, hipGetErrorString(e));
    if (shares) {
        h->counter_set = 1 - h->counter_set;
        if (!capturing) {
            h->last_divide_stream = hs;
            h->divide_launched = true;
        }
    }
    return TETRI_OK;
}

tetri_status tetri_chunk_prefill_attn(tetri_ctx *h, const void *q, const void *k_new, const void *v_new,
                                      const void *kv_pages, const int32_t *block_table, const int32_t *cu,
                                      const int32_t *ctx_lens, int32_t num_segs, float scale, void *out, void *stream)
{
    return attn_common("tetri_chunk_prefill_attn", h, q, k_new, v_new, kv_pages, nullptr, block_table, cu, ctx_lens,
                       num_segs, scale, out, stream);
}

tetri_status tetri_chunk_prefill_attn_append(tetri_ctx *h, const void *q, const void *k_new, const void *v_new,
                                             void *kv_pages, const int32_t *block_table, const int32_t *cu,
                                             const int32_t *ctx_lens, int32_t num_segs, float scale, void *out,
                                             void *stream)
{
    return attn_common("tetri_chunk_prefill_attn_append", h, q, k_new, v_new, kv_pages, kv_pages, block_table, cu,
                       ctx_lens, num_segs, scale, out, stream);
}

tetri_status tetri_chunk_prefill_attn_fp8(tetri_ctx *h, const void *q, const void *k_new, const void *v_new,
                                          void *kv_pages_fp8, const int32_t *block_table, const int32_t *cu,
                                          const int32_t *ctx_lens, int32_t num_segs, float scale, float k_scale,
                                          float v_scale, int32_t append, void *out, void *stream)
{
    if (append != 0 && append != 1) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_chunk_prefill_attn_fp8: append must be 0 or 1");
    return attn_common("tetri_chunk_prefill_attn_fp8", h, q, k_new, v_new, kv_pages_fp8, append ? kv_pages_fp8 : nullptr,
                       block_table, cu, ctx_lens, num_segs, scale, out, stream, true, k_scale, v_scale);
}

tetri_status tetri_validate_chunk(tetri_ctx *h, const int32_t *block_table, const int32_t *cu, const int32_t *ctx_lens,
                                  int32_t num_segs, void *stream)
{
    if (!h) return fail(nullptr, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: null handle");
    if (!block_table || !cu || !ctx_lens) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: null metadata pointer");
    if (num_segs < 1 || num_segs > h->cfg.max_segs_per_chunk)
        return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: num_segs=%d outside 1..%d", num_segs, h->cfg.max_segs_per_chunk);
    const tetri_config &c = h->cfg;
    std::vector<int32_t> hcu((size_t)num_segs + 1), hctx((size_t)num_segs), hbt((size_t)num_segs * c.max_blocks_per_seq);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipStreamSynchronize(st);
    if (e == hipSuccess) e = hipMemcpy(hcu.data(), cu, hcu.size() * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(hctx.data(), ctx_lens, hctx.size() * 4, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(hbt.data(), block_table, hbt.size() * 4, hipMemcpyDeviceToHost);
    if (e != hipSuccess) return fail(h, TETRI_ERR_HIP, "tetri_validate_chunk: %s", hipGetErrorString(e));
    if (hcu[0] != 0) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: cu[0]=%d, expected 0", hcu[0]);
    std::vector<int32_t> writer((size_t)c.num_pages, -1);
    for (int32_t s = 0; s < num_segs; ++s) {
        const int32_t n = hcu[s + 1] - hcu[s];
        if (n <= 0) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: segment %d has length %d", s, n);
        if (hctx[s] < 0) return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: ctx_lens[%d]=%d", s, hctx[s]);
        const int64_t end = (int64_t)hctx[s] + n;
        const int64_t blocks = (end + c.page_size - 1) / c.page_size;
        if (blocks > c.max_blocks_per_seq)
            return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: segment %d needs %lld pages, block_table rows hold %d",
                        s, (long long)blocks, c.max_blocks_per_seq);
        for (int64_t b = 0; b < blocks; ++b) {
            const int32_t page = hbt[(size_t)s * c.max_blocks_per_seq + b];
            if (page < 0 || page >= c.num_pages)
                return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: block_table[%d][%lld]=%d outside the pool of %d pages",
                            s, (long long)b, page, c.num_pages);
            if (b >= hctx[s] / c.page_size) {      // a page this segment writes to
                if (writer[page] >= 0 && writer[page] != s)
                    return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: page %d is written by segments %d and %d", page, writer[page], s);
                writer[page] = s;
            }
        }
    }
    if (hcu[num_segs] > c.chunk_size)
        return fail(h, TETRI_ERR_INVALID_ARG, "tetri_validate_chunk: cu[num_segs]=%d exceeds chunk_size=%d", hcu[num_segs], c.chunk_size);
    return TETRI_OK;
}

}  // extern "C"
