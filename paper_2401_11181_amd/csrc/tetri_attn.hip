// Chunked-prefill causal attention over a paged KV cache for gfx950 (CDNA4).
// TetriInfer Sec. 3.3.3 (prefill one fixed-size chunk at a time; several requests may be merged
// into a chunk), Sec. 2.1 (causal prefill), Sec. 3.4 (paged KV).  The kernel is a flash-style
// single pass with online softmax; that structure is prior art (the paper names FlashAttention
// as orthogonal work), the paper itself gives no kernel.
//
// Mapping to the hardware
//   * One workgroup = 4 wavefronts of 64 lanes.  A wavefront owns 32 query rows of one query
//     head; the 4 wavefronts are (heads sharing one kv head) x (32-row blocks), so a K/V tile
//     staged in LDS is used by all of them.
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: K fragments
//     come from LDS (A operand), Q fragments stay in registers (B operand).  In the accumulator
//     layout every lane then holds 16 keys of ONE query, so row max / row sum are in-lane
//     reductions plus one exchange between the two half-waves, and the bf16-rounded weights are
//     already laid out as the B operand of the second product O^T += V^T P^T.
//   * V is staged row-major ([key][d]) and read with ds_read_b64_tr_b16, which hands each lane
//     four consecutive keys of one d: the A operand of the second product without a transpose
//     pass.
//   * LDS rows are XOR-swizzled in 16-byte units so that the 128-bit K reads and the transposing
//     V reads are bank-conflict free.
#include "tetri_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int kPage = 16;     // tokens per KV page
constexpr int kBN = 64;       // keys per LDS tile
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

template <int D> __device__ __forceinline__ int k_swizzle(int row)
{
    // 16 consecutive rows must land in 16 different 16-byte bank groups
    return (D == 128) ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int v_swizzle(int row)
{
    // 4 consecutive rows x 64 contiguous bytes must land in 4 different 64-byte bank groups
    return (D == 128) ? ((row & 3) << 2) : (((row ^ (row >> 1)) & 1) << 2);
}

// Exchange between the two half-waves (lanes l and l^32 hold the same query) with
// v_permlane32_swap: afterwards the first register holds, in every lane, the value of the lower
// half-wave and the second the value of the upper half-wave.  Written as inline assembly because
// the compiler builtin returned its first result for both elements when both were consumed by
// one arithmetic instruction; the s_nop cover the VALU-write -> permlane-swap wait states.
__device__ __forceinline__ void half_swap(float x, float &lo_half, float &hi_half)
{
    int a = __builtin_bit_cast(int, x), b = a;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    lo_half = __builtin_bit_cast(float, a);
    hi_half = __builtin_bit_cast(float, b);
}
__device__ __forceinline__ float half_swap_max(float x)
{
    float a, b;
    half_swap(x, a, b);
    return fmaxf(a, b);
}
__device__ __forceinline__ float half_swap_sum(float x)
{
    float a, b;
    half_swap(x, a, b);
    return a + b;
}

template <int D>
__global__ __launch_bounds__(kThreads) void attn_fwd_kernel(AttnParams p)
{
    constexpr int CH = D / 8;        // 16-byte chunks per K/V row
    constexpr int KSTEPS = D / 16;   // MFMA steps over d for S^T
    constexpr int DBLK = D / 32;     // 32-row blocks of O^T
    constexpr int LOADS = kBN * CH / kThreads;
    __shared__ uint4 Ks[kBN * CH];
    __shared__ uint4 Vs[kBN * CH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int BM = 32 * p.rb;
    const int S = p.S;

    // ---- which (segment, row tile) is this workgroup?  Tiles never span two segments.
    int tile = blockIdx.x;
    int s = 0, t0 = -1;
    for (; s < S; ++s) {
        const int n = p.cu[s + 1] - p.cu[s];
        const int nt = (n + BM - 1) / BM;
        if (tile < nt) { t0 = tile * BM; break; }
        tile -= nt;
    }
    const int hh = wave % p.hpw, rbk = wave / p.hpw;
    const int head = blockIdx.y * p.hpw + hh;
    if (t0 < 0) {
        // padding rows [cu[S], C): written as +0
        const int r0 = p.cu[S] + tile * BM + 32 * rbk;
        if (r0 >= p.C) return;
        const int r = r0 + l32;
        if (r < p.C) {
            uint4 *o = reinterpret_cast<uint4 *>(p.out + ((size_t)r * p.Hq + head) * D);
            for (int c = half; c < CH; c += 2) o[c] = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    const int n_s = p.cu[s + 1] - p.cu[s], row_base = p.cu[s], L = p.ctx[s];
    const int kh = (blockIdx.y * p.hpw) / p.g;
    const int tw0 = t0 + 32 * rbk;         // first local row of this wavefront
    const int t = tw0 + l32;               // local row of this lane's query
    const bool row_ok = t < n_s;
    const bool wave_has_rows = tw0 < n_s;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds q[t][16*st + 8*half .. +7]
    bf16x8 qf[KSTEPS];
    {
        const uint4 *qp = reinterpret_cast<const uint4 *>(p.q + ((size_t)(row_base + (row_ok ? t : 0)) * p.Hq + head) * D);
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

    const int32_t *bt_row = p.bt + (size_t)s * p.max_blocks;
    const size_t head_block = (size_t)kPage * D;                 // elements of one (page, K|V, head) block
    const int n_ctx_tiles = (L + kBN - 1) / kBN;
    const int n_new = min(n_s, t0 + BM);                         // new keys any row of this tile may see
    const int n_tiles = n_ctx_tiles + (n_new + kBN - 1) / kBN;
    const float c = p.c;

    for (int it = 0; it < n_tiles; ++it) {
        const bool is_ctx = it < n_ctx_tiles;
        const int base = (is_ctx ? it : it - n_ctx_tiles) * kBN;
        const int limit = is_ctx ? L : n_new;

        __syncthreads();     // everyone is done reading the previous tile
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            const int x = i * kThreads + tid;
            const int r = x / CH, ch = x % CH;
            const int j = base + r;
            uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
            if (j < limit) {
                if (is_ctx) {
                    const int page = bt_row[j / kPage];
                    const size_t off = ((size_t)page * 2 * p.Hkv + kh) * head_block + (size_t)(j % kPage) * D + ch * 8;
                    kv = *reinterpret_cast<const uint4 *>(p.pages + off);
                    vv = *reinterpret_cast<const uint4 *>(p.pages + off + (size_t)p.Hkv * head_block);
                } else {
                    const size_t off = ((size_t)(row_base + j) * p.Hkv + kh) * D + ch * 8;
                    kv = *reinterpret_cast<const uint4 *>(p.k_new + off);
                    vv = *reinterpret_cast<const uint4 *>(p.v_new + off);
                }
            }
            Ks[r * CH + (ch ^ k_swizzle<D>(r))] = kv;
            Vs[r * CH + (ch ^ v_swizzle<D>(r))] = vv;
        }
        __syncthreads();

        // a wavefront whose rows all precede this tile's keys has nothing to do here
        const bool active = wave_has_rows && (is_ctx || base <= tw0 + 31);
        if (!active) continue;

        // ---- S^T = K Q^T for 64 keys x 32 queries
        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[kb][v] = 0.f;
            const int r = kb * 32 + l32;
#pragma unroll
            for (int st = 0; st < KSTEPS; ++st) {
                const uint4 kq = Ks[r * CH + ((2 * st + half) ^ k_swizzle<D>(r))];
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kq), qf[st], sacc[kb], 0, 0, 0);
            }
        }
        if (p.neg) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[kb][v] = -sacc[kb][v];
        }
        // ---- mask: accumulator element v of block kb is key base + kb*32 + (v/4)*8 + 4*half + v%4
        const bool need_mask = is_ctx ? (base + kBN > L) : (base + kBN - 1 > tw0);
        if (need_mask) {
            const int bound = is_ctx ? L - 1 : t;      // last visible key index of this phase
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = base + kb * 32 + (v / 4) * 8 + 4 * half + (v % 4);
                    if (key > bound) sacc[kb][v] = -INFINITY;
                }
        }
        // ---- online softmax (per query = per lane pair)
        float mx = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[kb][v]);
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m, mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
        bf16x8 pf[4];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][v], c, -m_new));
                if (need_mask && sacc[kb][v] == -INFINITY) pv = 0.f;   // also right for scale == 0
                lsum += pv;
                pf[kb * 2 + v / 8][v % 8] = (__bf16)pv;
            }
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
            for (int i = 0; i < DBLK; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
        }
        // ---- O^T += V^T P^T.  Step (kb, j) contracts the 16 keys held in accumulator elements
        // 8j..8j+7 of block kb: rows kb*32 + 16j + 4*half + {0..3} and the same + 8.
        const int blk = lane >> 4, i16 = lane & 15;
#pragma unroll
        for (int kj = 0; kj < 4; ++kj) {
            const int r0 = kj * 16 + 4 * half + (i16 >> 2);
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                const int d0 = db * 32 + 16 * (blk & 1) + 4 * (i16 & 3);
                const char *vb = reinterpret_cast<const char *>(Vs);
                const int ra = r0, rb2 = r0 + 8;
                const int offa = ra * D * 2 + (((d0 >> 3) ^ v_swizzle<D>(ra)) << 4) + ((d0 & 7) << 1);
                const int offb = rb2 * D * 2 + (((d0 >> 3) ^ v_swizzle<D>(rb2)) << 4) + ((d0 & 7) << 1);
                const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vb + offa));
                const s16x4 vb4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vb + offb));
                const s16x8 v8 = __builtin_shufflevector(va, vb4, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, v8), pf[kj], o[db], 0, 0, 0);
            }
        }
    }

    // ---- normalise and store: lane holds out[t][head][db*32 + (v/4)*8 + 4*half + v%4]
    if (!row_ok) return;
    const float inv = __builtin_amdgcn_rcpf(half_swap_sum(lsum));
    uint16_t *orow = p.out + ((size_t)(row_base + t) * p.Hq + head) * D;
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][q4 * 4 + e] * inv);
            *reinterpret_cast<uint2 *>(orow + db * 32 + q4 * 8 + 4 * half) = __builtin_bit_cast(uint2, w);
        }
}

}  // namespace

hipError_t tetri_launch_attn(const tetri_ctx *h, const AttnParams &p, hipStream_t stream)
{
    const int BM = 32 * p.rb;
    // upper bound of the number of row tiles: every segment and the padding range may end in a
    // partial tile
    const int tiles = (p.C + (p.S + 1) * (BM - 1)) / BM;
    dim3 grid(tiles, p.Hq / p.hpw), block(kThreads);
    if (h->cfg.head_dim == 128)
        hipLaunchKernelGGL(attn_fwd_kernel<128>, grid, block, 0, stream, p);
    else
        hipLaunchKernelGGL(attn_fwd_kernel<64>, grid, block, 0, stream, p);
    return hipGetLastError();
}
