// Chunked-prefill causal attention over a paged KV cache for gfx950 (CDNA4).
// TetriInfer Sec. 3.3.3 (prefill one fixed-size chunk at a time; several requests may be merged
// into a chunk), Sec. 2.1 (causal prefill), Sec. 3.4 (paged KV).  The kernel is a flash-style
// single pass with online softmax; that structure is prior art (the paper names FlashAttention
// as orthogonal work), the paper itself gives no kernel.
//
// Mapping to the hardware
//   * A workgroup is NW wavefronts of 64 lanes.  A wavefront owns 32 query rows of one query
//     head; the wavefronts of a workgroup are (heads sharing one kv head) x (32-row blocks), so a
//     K/V tile staged in LDS is used by all of them.
//   * K/V tiles (64 or 32 keys) go from HBM/L2 straight into LDS with global_load_lds_dwordx4 (no
//     register staging), double buffered: the loads of tile i+1 are in flight while tile i is
//     consumed; one workgroup barrier per tile.
//   * Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: K fragments
//     come from LDS (A operand), Q fragments stay in registers (B operand).  In the accumulator
//     layout every lane then holds 16 keys of ONE query, so row max / row sum are in-lane
//     reductions plus one exchange between the two half-waves, and the bf16-rounded weights are
//     already laid out as the B operand of the second product O^T += V^T P^T.
//   * V is staged row-major ([key][d]) and read with ds_read_b64_tr_b16, which hands each lane
//     four consecutive keys of one d: the A operand of the second product without a transpose
//     pass.
//   * LDS rows are XOR-swizzled in 16-byte units (the permutation is applied to the per-lane
//     global address of the direct load) so that the 128-bit K reads and the transposing V reads
//     are bank-conflict free.
//   * Workgroup ids are remapped so that all row tiles of a kv head run on one XCD (one L2).
#include "tetri_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void gbl_cvoid;

constexpr int kPage = 16;     // tokens per KV page
constexpr int kXcd = 8;       // XCDs (L2 domains) workgroups are dealt to round-robin

// A row of zeros: out-of-range key rows of a partial tile are loaded from here.
__device__ __attribute__((aligned(256))) uint4 g_zero_row[16];

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

// Everything a wavefront needs to know about where its workgroup's keys come from.
struct KeySource {
    const uint16_t *pages, *k_new, *v_new;
    const int32_t *bt_row;
    int Hkv, kh, row_base, L, n_new, n_ctx_tiles, max_blocks;
};

// The block table is read-only for the whole launch, so its (wave-uniform) entries are read
// through the constant address space: the compiler then uses scalar loads and the page ids live
// in SGPRs, off the vector-memory queue that carries the K/V tiles.
typedef __attribute__((address_space(4))) const int32_t const_i32;

// Physical pages of the (up to 4) logical pages of context tile `it` (unused for new-token
// tiles).  Plain scalars, not an array, so that they stay in SGPRs.
struct TilePages { int p0, p1, p2, p3; };

template <int BN>
__device__ __forceinline__ TilePages load_tile_pages(const KeySource &ks, int it)
{
    const const_i32 *bt = (const const_i32 *)(uintptr_t)ks.bt_row;
    const int first = it * (BN / kPage), last = ks.max_blocks - 1;   // clamped entries are never used
    TilePages tp;
    tp.p0 = bt[min(first, last)];
    tp.p1 = bt[min(first + 1, last)];
    tp.p2 = BN > 32 ? bt[min(first + 2, last)] : 0;
    tp.p3 = BN > 32 ? bt[min(first + 3, last)] : 0;
    return tp;
}

// Issue the direct-to-LDS loads of this wavefront's share of tile `it` (K and V, BN keys).
// One instruction moves 1 KB = 4 key rows (8 for head_dim 64); lane l lands at byte 16*l of that
// KB, so it fetches row 4q + l/16, 16-byte chunk (l%16) ^ swizzle(row).
template <int D, int NW, int BN>
__device__ __forceinline__ void issue_tile_loads(const KeySource &ks, const TilePages &tp, int it, int wave, int lane,
                                                 uint4 *Kbuf, uint4 *Vbuf)
{
    constexpr int CH = D / 8;
    constexpr int ROWS_PER_INST = 64 / CH;             // 4 for D=128, 8 for D=64
    constexpr int INSTS = BN / ROWS_PER_INST;          // per matrix per tile
    constexpr int PER_WAVE = INSTS / NW;
    const bool is_ctx = it < ks.n_ctx_tiles;
    const int base = (is_ctx ? it : it - ks.n_ctx_tiles) * BN;
    const int limit = is_ctx ? ks.L : ks.n_new;
    const size_t head_block = (size_t)kPage * D;
    const int lr = lane / CH, cpos = lane % CH;
    const uint16_t *zero = reinterpret_cast<const uint16_t *>(g_zero_row);
#pragma unroll
    for (int i = 0; i < PER_WAVE; ++i) {
        const int q = wave * PER_WAVE + i;             // wave-uniform
        const int r = q * ROWS_PER_INST + lr;          // row inside the tile
        const int j = base + r;
        // the rows of one instruction lie inside one 16-token page
        const int pk = (q * ROWS_PER_INST) / kPage;    // wave-uniform
        const int page = pk == 0 ? tp.p0 : pk == 1 ? tp.p1 : pk == 2 ? tp.p2 : tp.p3;
        const uint16_t *kctx = ks.pages + ((size_t)page * 2 * ks.Hkv + ks.kh) * head_block + (size_t)(j % kPage) * D;
        const size_t noff = ((size_t)(ks.row_base + j) * ks.Hkv + ks.kh) * D;
        const uint16_t *ksrc = is_ctx ? kctx : ks.k_new + noff;
        const uint16_t *vsrc = is_ctx ? kctx + (size_t)ks.Hkv * head_block : ks.v_new + noff;
        const bool ok = j < limit;
        const uint16_t *kp = ok ? ksrc + ((cpos ^ k_swizzle<D>(r)) << 3) : zero;
        const uint16_t *vp = ok ? vsrc + ((cpos ^ v_swizzle<D>(r)) << 3) : zero;
        __builtin_amdgcn_global_load_lds((gbl_cvoid *)kp, (lds_void *)(Kbuf + q * 64), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((gbl_cvoid *)vp, (lds_void *)(Vbuf + q * 64), 16, 0, 0);
    }
}

template <int D, int NW, int BN>
__global__ __launch_bounds__(NW * 64, 2) void attn_fwd_kernel(AttnParams p)
{
    constexpr int CH = D / 8;        // 16-byte chunks per K/V row
    constexpr int KSTEPS = D / 16;   // MFMA steps over d for S^T
    constexpr int DBLK = D / 32;     // 32-row blocks of O^T
    constexpr int NKB = BN / 32;     // 32-key blocks of S^T per tile
    __shared__ uint4 Ks0[BN * CH], Ks1[BN * CH], Vs0[BN * CH], Vs1[BN * CH];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    const int BM = 32 * p.rb;
    const int S = p.S;

    // ---- workgroup id -> (head group, row tile); a head group's tiles share one XCD
    const int per_xcd = gridDim.x / kXcd;
    const int logical = (blockIdx.x % kXcd) * per_xcd + blockIdx.x / kXcd;
    const int groups = p.Hq / p.hpw;
    if (logical >= p.tiles * groups) return;
    const int grp = logical / p.tiles;
    int tile = p.tiles - 1 - logical % p.tiles;        // late (long) tiles first

    // ---- which (segment, row tile) is it?  Tiles never span two segments.
    int s = 0, t0 = -1;
    for (; s < S; ++s) {
        const int n = p.cu[s + 1] - p.cu[s];
        const int nt = (n + BM - 1) / BM;
        if (tile < nt) { t0 = tile * BM; break; }
        tile -= nt;
    }
    const int hh = wave % p.hpw, rbk = wave / p.hpw;
    const int head = grp * p.hpw + hh;
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
    const int n_s = p.cu[s + 1] - p.cu[s], L = p.ctx[s];
    KeySource ks;
    ks.pages = p.pages; ks.k_new = p.k_new; ks.v_new = p.v_new;
    ks.bt_row = p.bt + (size_t)s * p.max_blocks;
    ks.Hkv = p.Hkv; ks.kh = (grp * p.hpw) / p.g; ks.row_base = p.cu[s]; ks.L = L;
    ks.n_new = min(n_s, t0 + BM);                      // new keys any row of this tile may see
    ks.n_ctx_tiles = (L + BN - 1) / BN;
    ks.max_blocks = p.max_blocks;
    const int n_tiles = ks.n_ctx_tiles + (ks.n_new + BN - 1) / BN;

    const int tw0 = t0 + 32 * rbk;         // first local row of this wavefront
    const int t = tw0 + l32;               // local row of this lane's query
    const bool row_ok = t < n_s;
    const bool wave_has_rows = tw0 < n_s;

    TilePages tp = load_tile_pages<BN>(ks, 0);
    issue_tile_loads<D, NW, BN>(ks, tp, 0, wave, lane, Ks0, Vs0);
    tp = load_tile_pages<BN>(ks, 1);

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

    auto consume = [&](int it, const uint4 *Kt, const uint4 *Vt) {
        const bool is_ctx = it < ks.n_ctx_tiles;
        const int base = (is_ctx ? it : it - ks.n_ctx_tiles) * BN;
        // a wavefront whose rows all precede this tile's keys has nothing to do here
        if (!(wave_has_rows && (is_ctx || base <= tw0 + 31))) return;

        // ---- S^T = K Q^T for BN keys x 32 queries
        f32x16 sacc[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) sacc[kb][v] = 0.f;
            const int r = kb * 32 + l32;
#pragma unroll
            for (int st = 0; st < KSTEPS; ++st) {
                const uint4 kq = Kt[r * CH + ((2 * st + half) ^ k_swizzle<D>(r))];
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kq), qf[st], sacc[kb], 0, 0, 0);
            }
        }
        if (p.neg) {
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[kb][v] = -sacc[kb][v];
        }
        // ---- mask: accumulator element v of block kb is key base + kb*32 + (v/4)*8 + 4*half + v%4
        const bool need_mask = is_ctx ? (base + BN > L) : (base + BN - 1 > tw0);
        if (need_mask) {
            const int bound = is_ctx ? L - 1 : t;      // last visible key index of this phase
#pragma unroll
            for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = base + kb * 32 + (v / 4) * 8 + 4 * half + (v % 4);
                    if (key > bound) sacc[kb][v] = -INFINITY;
                }
        }
        // ---- online softmax (per query = per lane pair)
        float mx = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[kb][v]);
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m, mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        lsum *= alpha;
        bf16x8 pf[2 * NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
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
        // ---- O^T += V^T P^T.  Step kj contracts the 16 keys held in accumulator elements
        // 8j..8j+7 of block kb (kj = 2*kb + j): rows 16*kj + 4*half + {0..3} and the same + 8.
        const int blk = lane >> 4, i16 = lane & 15;
        const char *vb = reinterpret_cast<const char *>(Vt);
#pragma unroll
        for (int kj = 0; kj < 2 * NKB; ++kj) {
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
    };

    // ---- main loop, two tiles per trip so that each LDS buffer is named statically.  `tp` always
    // holds the page ids of the tile whose loads are issued next; they are fetched one tile ahead.
    for (int it = 0; it < n_tiles; it += 2) {
        __builtin_amdgcn_s_waitcnt(0);      // this wavefront's loads of tile `it` have landed
        __syncthreads();                    // ... and everyone's; the other buffer is free
        if (it + 1 < n_tiles) issue_tile_loads<D, NW, BN>(ks, tp, it + 1, wave, lane, Ks1, Vs1);
        tp = load_tile_pages<BN>(ks, it + 2);
        consume(it, Ks0, Vs0);
        if (it + 1 >= n_tiles) break;
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (it + 2 < n_tiles) issue_tile_loads<D, NW, BN>(ks, tp, it + 2, wave, lane, Ks0, Vs0);
        tp = load_tile_pages<BN>(ks, it + 3);
        consume(it + 1, Ks1, Vs1);
    }

    // ---- normalise and store: lane holds out[t][head][db*32 + (v/4)*8 + 4*half + v%4]
    if (!row_ok) return;
    const float inv = __builtin_amdgcn_rcpf(half_swap_sum(lsum));
    uint16_t *orow = p.out + ((size_t)(ks.row_base + t) * p.Hq + head) * D;
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][q4 * 4 + e] * inv);
            *reinterpret_cast<uint2 *>(orow + db * 32 + q4 * 8 + 4 * half) = __builtin_bit_cast(uint2, w);
        }
}

template <int D, int NW, int BN>
hipError_t launch(const AttnParams &p, hipStream_t stream)
{
    const int groups = p.Hq / p.hpw;
    const int nwg = p.tiles * groups;
    const int grid = (nwg + kXcd - 1) / kXcd * kXcd;
    hipLaunchKernelGGL((attn_fwd_kernel<D, NW, BN>), dim3(grid), dim3(NW * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t tetri_launch_attn(const tetri_ctx *h, const AttnParams &p, hipStream_t stream)
{
    const int nw = p.hpw * p.rb;
    if (h->cfg.head_dim == 128)
        return nw == 4 ? launch<128, 4, 64>(p, stream) : launch<128, 2, 32>(p, stream);
    return nw == 4 ? launch<64, 4, 64>(p, stream) : launch<64, 2, 32>(p, stream);
}
