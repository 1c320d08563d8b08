// KV export / import for gfx950: the data plane of the dispatcher (TetriInfer Sec. 3.3.4).  Export
// gathers token ranges of requests out of the paged pool (Sec. 3.4) into a dense transfer buffer,
// request after request as [2 (K, V)][Hkv][n_r][D]; import scatters such a buffer into the pages of
// the receiving pool.  Pure 16-byte vector copies, HBM-bound, bit-exact by construction.
//
// Work split: a workgroup moves 64 consecutive tokens of one request for a few (K / V, head) slabs.
// On the pool side 16 consecutive tokens of a slab are one contiguous 16 * D * 2 bytes of a page, on
// the buffer side the 64 tokens are contiguous, so both sides are touched in whole cache lines.
// The page of every row is looked up once and reused for all slabs of the workgroup.  The data is
// used once: loads and stores are non-temporal.
#include "tetri_internal.h"

namespace {

constexpr int kPage = 16;
constexpr int kTile = 64;      // tokens per workgroup
constexpr int kThreads = 256;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The request that owns 64-token tile `tile` when the tiles of all requests are numbered request after
// request (request r has ceil(n_r / 64) of them), and the tile's first token inside the request.
// Wavefront-wide: 64 requests per step, prefix sum by shuffles.  Every wavefront computes the same
// result.  Returns -1 when the grid's upper bound overshoots the real number of tiles.
__device__ inline int find_request(const int32_t *cu, int R, int tile, int lane, int &j0)
{
    int base = 0;
    for (int r0 = 0; r0 < R; r0 += 64) {
        const int r = r0 + lane;
        int n = 0;
        if (r < R) n = cu[r + 1] - cu[r];
        const int t = (n + kTile - 1) / kTile;
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
            j0 = (tile - __shfl(incl - t, src)) * kTile;
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
    constexpr int LPR = D / 8;                 // lanes that move one row of D bf16
    constexpr int RPP = kThreads / LPR;        // rows per pass of the workgroup
    constexpr int PASSES = kTile / RPP;
    const int tid = threadIdx.x;
    int j0 = 0;
    const int r = __builtin_amdgcn_readfirstlane(find_request(p.cu, p.R, blockIdx.x, tid & 63, j0));
    if (r < 0) return;
    j0 = __builtin_amdgcn_readfirstlane(j0);
    const int c0 = p.cu[r];
    const int n = p.cu[r + 1] - c0;
    const int first = p.first ? p.first[r] : 0;
    const int col = (tid % LPR) * 8;
    const int slabs = 2 * p.Hkv;
    const size_t page_elems = (size_t)slabs * kPage * D;

    size_t pool_at[PASSES], buf_at[PASSES];
    bool ok[PASSES];
#pragma unroll
    for (int i = 0; i < PASSES; ++i) {
        const int j = j0 + i * RPP + tid / LPR;
        ok[i] = j < n;
        const int pos = first + j;
        const int page = ok[i] ? p.bt[(size_t)r * p.max_blocks + pos / kPage] : 0;
        pool_at[i] = (size_t)page * page_elems + (size_t)(pos % kPage) * D + col;
        buf_at[i] = (size_t)slabs * D * c0 + (size_t)j * D + col;
    }
    const int slab_end = min(slabs, ((int)blockIdx.y + 1) * p.slabs_per_wg);
    for (int slab = blockIdx.y * p.slabs_per_wg; slab < slab_end; ++slab) {
        const size_t in_pool = (size_t)slab * kPage * D;      // slab = kv * Hkv + head in both layouts
        const size_t in_buf = (size_t)slab * n * D;
        u32x4 v[PASSES];
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            const uint16_t *src = TO_POOL ? p.buf + buf_at[i] + in_buf : p.pool + pool_at[i] + in_pool;
            if (ok[i]) v[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src));
        }
#pragma unroll
        for (int i = 0; i < PASSES; ++i) {
            uint16_t *dst = TO_POOL ? p.pool + pool_at[i] + in_pool : p.buf + buf_at[i] + in_buf;
            if (ok[i]) __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4 *>(dst));
        }
    }
}

}  // namespace

hipError_t tetri_launch_kv_transfer(const tetri_ctx *h, const TransferParams &p, int32_t tiles, bool to_pool,
                                    hipStream_t stream)
{
    dim3 grid(tiles, (2 * p.Hkv + p.slabs_per_wg - 1) / p.slabs_per_wg), block(kThreads);
    const int d = h->cfg.head_dim;
    if (d == 128) {
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
