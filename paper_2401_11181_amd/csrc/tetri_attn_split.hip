// Chunked-prefill attention, key-split variant for small grids (gfx950).
// Same function as the shared-tile kernel (TetriInfer Sec. 3.3.3 / 2.1 / 3.4: one chunk's causal
// attention over its requests' paged KV plus its own new K/V), different decomposition.
//
// At ChunkSize 512 with 40 heads there are only 640 blocks of 32 query rows, fewer than the 1024
// SIMDs of the chip, so rows alone cannot fill it.  Here a workgroup owns ONE block of 32 rows of
// one head and its 4 wavefronts split that block's key range into 4 contiguous parts.  Each
// wavefront runs the online-softmax loop over its part with wave-private LDS staging (32-key
// tiles, K and V in separate single buffers whose refills overlap the other phase: the next K
// tile streams in during softmax + PV, the next V tile during QK^T + softmax), so the main loop
// has no workgroup barrier at all.  The 4 partial results (row max, row sum, unnormalised O) are
// merged once through LDS, each wavefront finishing one quarter of the head dimension.
#include "attn_common.h"

namespace {

using namespace tetri_dev;

constexpr int kSplit = 4;     // wavefronts per workgroup = parts of the key range
constexpr int kBN = 32;       // keys per wave-private tile

// Loads of one 32-key tile of K or V (which = 0 / 1) into this wavefront's private buffer.
template <int D>
__device__ __forceinline__ void issue_split_loads(const KeySource &ks, const TilePages &tp, int it, int which, int lane,
                                                  uint32_t lds_buf)
{
    constexpr int CH = D / 8;
    constexpr int ROWS_PER_INST = 64 / CH;             // 4 for D=128, 8 for D=64
    constexpr int INSTS = kBN / ROWS_PER_INST;
    const bool is_ctx = it < ks.n_ctx_tiles;
    const int base = (is_ctx ? it : it - ks.n_ctx_tiles) * kBN;
    const int limit = is_ctx ? ks.L : ks.n_new;
    const size_t head_block = (size_t)kPage * D;
    const int lr = lane / CH, cpos = lane % CH;
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_zero_row);
#pragma unroll
    for (int q = 0; q < INSTS; ++q) {
        const int r = q * ROWS_PER_INST + lr;          // row inside the tile
        const int j = base + r;
        const int page = (q * ROWS_PER_INST) / kPage == 0 ? tp.p0 : tp.p1;
        const uint16_t *ctxp = ks.pages + (((size_t)page * 2 + which) * ks.Hkv + ks.kh) * head_block + (size_t)(j % kPage) * D;
        const uint16_t *newp = (which ? ks.v_new : ks.k_new) + ((size_t)(ks.row_base + j) * ks.Hkv + ks.kh) * D;
        const uint16_t *src = is_ctx ? ctxp : newp;
        const int swz = which ? v_swizzle<D>(r) : k_swizzle<D>(r);
        const uint16_t *ptr = (j < limit) ? src + ((cpos ^ swz) << 3) : zero;
        dma16(ptr, lds_buf + q * 1024);
    }
}

template <int D>
__global__ __launch_bounds__(kSplit * 64, 2) void attn_split_kernel(AttnParams p)
{
    constexpr int CH = D / 8;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;
    constexpr int TILE_U4 = kBN * CH;                  // uint4 per tile buffer
    constexpr int TILE_LOADS = TILE_U4 / 64;           // load instructions per tile (8 or 4)
    // wave-private staging; after the main loop the same memory carries the partial results
    __shared__ uint4 Kb[kSplit * TILE_U4];
    __shared__ uint4 Vb[kSplit * TILE_U4];
    __shared__ float Mstat[kSplit][2][32];             // per part: row max, row sum

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int S = p.S;

    // ---- workgroup id -> (head, 32-row block); all row blocks of a head share one XCD
    const int per_xcd = p.attn_grid / kXcd;
    const int logical = (blockIdx.x % kXcd) * per_xcd + blockIdx.x / kXcd;
    if (logical >= p.tiles * p.Hq) return;
    const int head = logical / p.tiles;
    int tile = p.tiles - 1 - logical % p.tiles;        // late (long) blocks first

    int s = 0, t0 = -1;
    for (; s < S; ++s) {
        const int n = p.cu[s + 1] - p.cu[s];
        const int nt = (n + 31) / 32;
        if (tile < nt) { t0 = tile * 32; break; }
        tile -= nt;
    }
    if (t0 < 0) {
        // padding rows [cu[S], C): written as +0 (wavefront 0 only)
        const int r = p.cu[S] + tile * 32 + l32;
        if (wave == 0 && r < p.C) {
            uint4 *o = reinterpret_cast<uint4 *>(p.out + ((size_t)r * p.Hq + head) * D);
            for (int c = half; c < CH; c += 2) o[c] = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    const int n_s = p.cu[s + 1] - p.cu[s], L = p.ctx[s];
    KeySource ks;
    ks.pages = p.pages; ks.k_new = p.k_new; ks.v_new = p.v_new;
    ks.bt_row = p.bt + (size_t)s * p.max_blocks;
    ks.Hkv = p.Hkv; ks.kh = head / p.g; ks.row_base = p.cu[s]; ks.L = L;
    ks.n_new = min(n_s, t0 + 32);
    ks.n_ctx_tiles = (L + kBN - 1) / kBN;
    ks.max_blocks = p.max_blocks;
    const int n_tiles = ks.n_ctx_tiles + (ks.n_new + kBN - 1) / kBN;
    // this wavefront's contiguous part of the key tiles
    const int it_begin = (int)((long long)n_tiles * wave / kSplit);
    const int it_end = (int)((long long)n_tiles * (wave + 1) / kSplit);

    const int t = t0 + l32;                // local row of this lane's query
    const bool row_ok = t < n_s;

    const uint4 *Kt = Kb + wave * TILE_U4;
    const uint4 *Vt = Vb + wave * TILE_U4;
    const uint32_t Kt_lds = __builtin_amdgcn_readfirstlane(lds_address(Kt));
    const uint32_t Vt_lds = __builtin_amdgcn_readfirstlane(lds_address(Vt));
    TilePages tp = load_tile_pages<kBN>(ks, it_begin);
    if (it_begin < it_end) {
        issue_split_loads<D>(ks, tp, it_begin, 0, lane, Kt_lds);
        issue_split_loads<D>(ks, tp, it_begin, 1, lane, Vt_lds);
    }
    tp = load_tile_pages<kBN>(ks, it_begin + 1);

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds q[t][16*st + 8*half .. +7]
    bf16x8 qf[KSTEPS];
    {
        const uint4 *qp = reinterpret_cast<const uint4 *>(p.q + ((size_t)(ks.row_base + (row_ok ? t : 0)) * p.Hq + head) * D);
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) {
            uint4 v = row_ok ? qp[2 * st + half] : make_uint4(0, 0, 0, 0);
            qf[st] = __builtin_bit_cast(bf16x8, v);
        }
    }

    f32x16 o[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m = -1e30f;        // running row max (in units of log2: score * c)
    float lsum = 0.f;        // this lane's share of the running row sum
    const float c = p.c;
    const int blk = lane >> 4, i16 = lane & 15;

    for (int it = it_begin; it < it_end; ++it) {
        const bool is_ctx = it < ks.n_ctx_tiles;
        const int base = (is_ctx ? it : it - ks.n_ctx_tiles) * kBN;
        const bool more = it + 1 < it_end;

        // ---- S^T = K Q^T for 32 keys x 32 queries (K tile `it` must have landed; the V tile
        // issued after it may still be in flight)
        wait_vm<TILE_LOADS>();
        f32x16 sacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) {
            const uint4 kq = Kt[l32 * CH + ((2 * st + half) ^ k_swizzle<D>(l32))];
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kq), qf[st], sacc, 0, 0, 0);
        }
        // the K buffer is free again: stream in the next K tile during softmax + PV
        if (more) issue_split_loads<D>(ks, tp, it + 1, 0, lane, Kt_lds);

        if (p.neg) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[v] = -sacc[v];
        }
        // ---- mask: accumulator element v is key base + (v/4)*8 + 4*half + v%4
        const bool need_mask = is_ctx ? (base + kBN > L) : (base + kBN - 1 > t0);
        if (need_mask) {
            const int bound = is_ctx ? L - 1 : t;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = base + (v / 4) * 8 + 4 * half + (v % 4);
                if (key > bound) sacc[v] = -INFINITY;
            }
        }
        // ---- online softmax
        float mx = sacc[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m, mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
        bf16x8 pf[2];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[v], c, -m_new));
            if (need_mask && sacc[v] == -INFINITY) pv = 0.f;
            lsum += pv;
            pf[v / 8][v % 8] = (__bf16)pv;
        }
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int i = 0; i < DBLK; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
        }
        // ---- O^T += V^T P^T (V tile `it` must have landed; the K tile just issued may be in flight)
        if (more) wait_vm<TILE_LOADS>();
        else wait_vm<0>();
        const char *vb = reinterpret_cast<const char *>(Vt);
#pragma unroll
        for (int kj = 0; kj < 2; ++kj) {
            const int ra = kj * 16 + 4 * half + (i16 >> 2), rb2 = ra + 8;
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                const int d0 = db * 32 + 16 * (blk & 1) + 4 * (i16 & 3);
                const int offa = ra * D * 2 + (((d0 >> 3) ^ v_swizzle<D>(ra)) << 4) + ((d0 & 7) << 1);
                const int offb = rb2 * D * 2 + (((d0 >> 3) ^ v_swizzle<D>(rb2)) << 4) + ((d0 & 7) << 1);
                const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vb + offa));
                const s16x4 vb4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vb + offb));
                const s16x8 v8 = __builtin_shufflevector(va, vb4, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v8), pf[kj], o[db], 0, 0, 0);
            }
        }
        // the V buffer is free again: stream in the next V tile during QK^T + softmax
        if (more) {
            issue_split_loads<D>(ks, tp, it + 1, 1, lane, Vt_lds);
            tp = load_tile_pages<kBN>(ks, it + 2);
        }
    }

    // ---- merge the 4 parts.  Every wavefront publishes (m, row sum, O); wavefront w then
    // finishes head-dim block w: out = sum_k O_k 2^(m_k - m*) / sum_k l_k 2^(m_k - m*).
    wait_vm<0>();
    __syncthreads();                       // all staging buffers are dead now
    float *part = reinterpret_cast<float *>(wave < 2 ? Kb + wave * 2 * TILE_U4 : Vb + (wave - 2) * 2 * TILE_U4);
    // partial O of wavefront w occupies 2 tile buffers = DBLK*16*64 floats, element (db, v, lane)
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) part[(db * 16 + v) * 64 + lane] = o[db][v];
    const float ltot = half_swap_sum(lsum);
    if (half == 0) { Mstat[wave][0][l32] = m; Mstat[wave][1][l32] = ltot; }
    __syncthreads();
    if (wave >= DBLK || !row_ok) return;
    float mstar = Mstat[0][0][l32];
#pragma unroll
    for (int k = 1; k < kSplit; ++k) mstar = fmaxf(mstar, Mstat[k][0][l32]);
    float wgt[kSplit], denom = 0.f;
#pragma unroll
    for (int k = 0; k < kSplit; ++k) {
        wgt[k] = __builtin_amdgcn_exp2f(Mstat[k][0][l32] - mstar);
        denom += wgt[k] * Mstat[k][1][l32];
    }
    const float inv = __builtin_amdgcn_rcpf(denom);
    const int db = wave;
    uint16_t *orow = p.out + ((size_t)(ks.row_base + t) * p.Hq + head) * D;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int v = q4 * 4 + e;
            float acc = 0.f;
#pragma unroll
            for (int k = 0; k < kSplit; ++k) {
                const float *pk = reinterpret_cast<const float *>(k < 2 ? Kb + k * 2 * TILE_U4 : Vb + (k - 2) * 2 * TILE_U4);
                acc += wgt[k] * pk[(db * 16 + v) * 64 + lane];
            }
            w[e] = (__bf16)(acc * inv);
        }
        *reinterpret_cast<uint2 *>(orow + db * 32 + q4 * 8 + 4 * half) = __builtin_bit_cast(uint2, w);
    }
}

template <int D>
hipError_t launch_split(const AttnParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL((attn_split_kernel<D>), dim3(p.attn_grid), dim3(kSplit * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t tetri_launch_attn_split(const tetri_ctx *h, const AttnParams &p, hipStream_t stream)
{
    return h->cfg.head_dim == 128 ? launch_split<128>(p, stream) : launch_split<64>(p, stream);
}
