// KV export / import for gfx950: the data plane of the dispatcher (TetriInfer Sec. 3.3.4).  Export
// gathers token ranges of requests out of the paged pool (Sec. 3.4) into a dense transfer buffer,
// request after request as [2 (K, V)][Hkv][n_r][D]; import scatters such a buffer into the pages of
// the receiving pool.  Pure 16-byte vector copies, HBM-bound, bit-exact by construction.
//
// Work split: a workgroup moves one tile of consecutive tokens of one request (4 KB per slab: 16 tokens
// for head dimension 128, 32 for 64) for a run of (K / V, head) slabs; each lane owns 16 bytes of one
// token and walks the slabs, four loads in flight.  On the pool side 16 consecutive tokens of a slab are
// one contiguous 16 * D * 2 bytes of a page, on the buffer side the tile is contiguous, so both sides
// are touched in whole cache lines.  The page of a token is looked up once and reused for all slabs.
// The data is used once: loads and stores are non-temporal.
#include "tetri_internal.h"

namespace {

constexpr int kPage = 16;
constexpr int kThreads = 256;
constexpr int kTileBytes = kThreads * 16;     // one slab of a tile

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The request that owns tile `tile` when the tiles (TILE tokens each) of all requests are numbered request
// after request (request r has ceil(n_r / TILE) of them), and the tile's first token inside the request.
// Wavefront-wide: 64 requests per step, prefix sum by shuffles.  Every wavefront computes the same
// result.  Returns -1 when the grid's upper bound overshoots the real number of tiles.
template <int TILE>
__device__ inline int find_request(const int32_t *cu, int R, int tile, int lane, int &j0)
{
    int base = 0;
    for (int r0 = 0; r0 < R; r0 += 64) {
        const int r = r0 + lane;
        int n = 0;
        if (r < R) n = cu[r + 1] - cu[r];
        const int t = (n + TILE - 1) / TILE;
        int incl = t;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int up = __shfl_up(incl, d);
            if (lane >= d) incl += up;
        }
        incl += base;
        const unsigned long long hit = __ballot(tile < incl && tile >= incl - t);
        if (hit) {
            const int src = __builtin_ctzll(hit);
            j0 = (tile - __shfl(incl - t, src)) * TILE;
            return r0 + src;
        }
        base = __shfl(incl, 63);
    }
    return -1;
}

// grid: (upper bound of the number of tiles, groups of slabs)
template <int D, bool TO_POOL>
__global__ __launch_bounds__(kThreads) void kv_transfer_kernel(TransferParams p)
{
    constexpr int LPR = D / 8;                 // lanes that move one token's D bf16 of one slab
    constexpr int TILE = kThreads / LPR;       // tokens per workgroup
    const int tid = threadIdx.x;
    int j0 = 0;
    const int r = __builtin_amdgcn_readfirstlane(find_request<TILE>(p.cu, p.R, blockIdx.x, tid & 63, j0));
    if (r < 0) return;
    j0 = __builtin_amdgcn_readfirstlane(j0);
    const int c0 = p.cu[r];
    const int n = p.cu[r + 1] - c0;
    const int first = p.first ? max(p.first[r], 0) : 0;
    const int j = j0 + tid / LPR;
    if (j >= n) return;                        // no barrier below: lanes past the request's end just leave
    const int col = (tid % LPR) * 8;
    const int slabs = 2 * p.Hkv;
    const int pos = first + j;
    // the block-table index is clamped: a range the table cannot describe never forms an address outside it
    const int page = p.bt[(size_t)r * p.max_blocks + min(pos / kPage, p.max_blocks - 1)];
    // slab = kv * Hkv + head in both layouts: from one slab to the next both sides advance by a fixed step
    const int slab0 = blockIdx.y * p.slabs_per_wg;
    int left = min(slabs, slab0 + p.slabs_per_wg) - slab0;
    const size_t pool_step = (size_t)kPage * D, buf_step = (size_t)n * D;
    uint16_t *in_pool = p.pool + ((size_t)page * slabs + slab0) * pool_step + (size_t)(pos % kPage) * D + col;
    uint16_t *in_buf = p.buf + (size_t)slabs * D * c0 + slab0 * buf_step + (size_t)j * D + col;
    const uint16_t *src = TO_POOL ? in_buf : in_pool;
    uint16_t *dst = TO_POOL ? in_pool : in_buf;
    const size_t src_step = TO_POOL ? buf_step : pool_step, dst_step = TO_POOL ? pool_step : buf_step;
    auto ld = [&]() {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
        src += src_step;
        return v;
    };
    auto st = [&](u32x4 v) {
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(dst));
        dst += dst_step;
    };
#pragma unroll 1
    for (; left >= 4; left -= 4) {
        const u32x4 v0 = ld(), v1 = ld(), v2 = ld(), v3 = ld();
        st(v0), st(v1), st(v2), st(v3);
    }
    if (left >= 2) {
        const u32x4 v0 = ld(), v1 = ld();
        st(v0), st(v1);
        left -= 2;
    }
    if (left) st(ld());
}

// Export with quantisation: the 16-bit pool is gathered into a dense buffer of FP8 E4M3 codes, the K
// half of every request's block under the K scale, the V half under the V scale (this build's extension:
// half the bytes on the link between the instances).  A code is fl32(x * inv_scale) clamped to +-448 and
// rounded to nearest even by v_cvt_pk_fp8_f32.  Same work split as the copy kernel: a lane reads 16 bytes
// (8 values) and writes 8 codes.
template <int D>
__global__ __launch_bounds__(kThreads) void kv_export_fp8_kernel(TransferParams p)
{
    constexpr int LPR = D / 8, TILE = kThreads / LPR;
    const int tid = threadIdx.x;
    int j0 = 0;
    const int r = __builtin_amdgcn_readfirstlane(find_request<TILE>(p.cu, p.R, blockIdx.x, tid & 63, j0));
    if (r < 0) return;
    j0 = __builtin_amdgcn_readfirstlane(j0);
    const int c0 = p.cu[r];
    const int n = p.cu[r + 1] - c0;
    const int first = p.first ? max(p.first[r], 0) : 0;
    const int j = j0 + tid / LPR;
    if (j >= n) return;
    const int col = (tid % LPR) * 8;
    const int slabs = 2 * p.Hkv;
    const int pos = first + j;
    const int page = p.bt[(size_t)r * p.max_blocks + min(pos / kPage, p.max_blocks - 1)];
    const int slab0 = blockIdx.y * p.slabs_per_wg;
    const int slab_end = min(slabs, slab0 + p.slabs_per_wg);
    const size_t pool_step = (size_t)kPage * D, buf_step = (size_t)n * D;
    const uint16_t *src = p.pool + ((size_t)page * slabs + slab0) * pool_step + (size_t)(pos % kPage) * D + col;
    uint8_t *dst = reinterpret_cast<uint8_t *>(p.buf) + (size_t)slabs * D * c0 + slab0 * buf_step + (size_t)j * D + col;
#pragma unroll 2
    for (int slab = slab0; slab < slab_end; ++slab) {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
        const float inv = slab < p.Hkv ? p.k_inv : p.v_inv;
        uint32_t codes[2];
#pragma unroll
        for (int w = 0; w < 2; ++w) {
            float y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t word = v[2 * w + e / 2];
                const float x = __builtin_bit_cast(float, (e & 1) ? (word & 0xffff0000u) : (word << 16));
                y[e] = __builtin_fminf(__builtin_fmaxf(x * inv, -448.0f), 448.0f);
            }
            int c = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
            c = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], c, true);
            codes[w] = (uint32_t)c;
        }
        __builtin_nontemporal_store(codes[0], reinterpret_cast<uint32_t *>(dst));
        __builtin_nontemporal_store(codes[1], reinterpret_cast<uint32_t *>(dst) + 1);
        src += pool_step;
        dst += buf_step;
    }
}

}  // namespace

hipError_t tetri_launch_kv_export_fp8(const tetri_ctx *h, const TransferParams &p, int32_t tiles, hipStream_t stream)
{
    dim3 grid(tiles, (2 * p.Hkv + p.slabs_per_wg - 1) / p.slabs_per_wg), block(kThreads);
    const int d = h->cfg.head_dim;
    if (d == 128) hipLaunchKernelGGL(kv_export_fp8_kernel<128>, grid, block, 0, stream, p);
    else if (d == 64) hipLaunchKernelGGL(kv_export_fp8_kernel<64>, grid, block, 0, stream, p);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// `row_units`: 16-bit units of one row of the pool (head_dim for a 16-bit pool, head_dim / 2 for FP8 codes,
// which the copy moves as opaque bytes)
hipError_t tetri_launch_kv_transfer(const tetri_ctx *, const TransferParams &p, int32_t row_units, int32_t tiles,
                                    bool to_pool, hipStream_t stream)
{
    dim3 grid(tiles, (2 * p.Hkv + p.slabs_per_wg - 1) / p.slabs_per_wg), block(kThreads);
    const int d = row_units;
    if (d == 32) {
        if (to_pool) hipLaunchKernelGGL((kv_transfer_kernel<32, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((kv_transfer_kernel<32, false>), grid, block, 0, stream, p);
    } else if (d == 128) {
        if (to_pool) hipLaunchKernelGGL((kv_transfer_kernel<128, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((kv_transfer_kernel<128, false>), grid, block, 0, stream, p);
    } else if (d == 64) {
        if (to_pool) hipLaunchKernelGGL((kv_transfer_kernel<64, true>), grid, block, 0, stream, p);
        else hipLaunchKernelGGL((kv_transfer_kernel<64, false>), grid, block, 0, stream, p);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
