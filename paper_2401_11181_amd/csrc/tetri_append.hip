// Paged KV append for gfx950: copies the chunk's new K/V rows into their page slots.
// TetriInfer Sec. 2.1 (prefill generates the KV cache) and Sec. 3.4 (the cache is paged).
// Pure 16-byte vector copy, HBM-bound: no arithmetic, bit-exact by construction.
#include "tetri_internal.h"

namespace {

constexpr int kPage = 16;

// grid: (chunk row, 0 = K / 1 = V).  One workgroup moves the Hkv*D elements of one token.
__global__ __launch_bounds__(256) void kv_append_kernel(AppendParams p)
{
    const int row = blockIdx.x;
    const int which = blockIdx.y;
    const int S = p.S;
    if (row >= p.cu[S]) return;                       // padding rows are never cached
    // segment of this row: largest s with cu[s] <= row (uniform across the workgroup)
    int lo = 0, hi = S - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (p.cu[mid] <= row) lo = mid; else hi = mid - 1;
    }
    const int s = lo;
    const int pos = p.ctx[s] + (row - p.cu[s]);
    const int page = p.bt[(size_t)s * p.max_blocks + pos / kPage];
    const int slot = pos % kPage;
    const int ch = p.D / 8;                           // 16-byte vectors per head row
    const int per_row = p.Hkv * ch;
    const uint4 *src = reinterpret_cast<const uint4 *>(which ? p.v_new : p.k_new) + (size_t)row * per_row;
    uint4 *dst = reinterpret_cast<uint4 *>(p.pages)
                 + ((size_t)page * 2 + which) * p.Hkv * kPage * ch + (size_t)slot * ch;
    for (int x = threadIdx.x; x < per_row; x += 256) {
        const int head = x / ch, c = x - head * ch;
        dst[(size_t)head * kPage * ch + c] = src[x];
    }
}

}  // namespace

hipError_t tetri_launch_append(const tetri_ctx *, const AppendParams &p, int32_t chunk_rows, hipStream_t stream)
{
    dim3 grid(chunk_rows, 2), block(256);
    hipLaunchKernelGGL(kv_append_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}
