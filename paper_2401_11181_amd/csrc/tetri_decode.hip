// One decode iteration over the paged KV cache for gfx950: the counterpart, on the decode instance, of
// the chunked-prefill kernel (TetriInfer Sec. 2.1: the decode phase produces one token per iteration
// and its query attends to the request's cached keys and values; Sec. 3.4: the decode instance batches
// the steps of many requests over a paged cache).
//
// The work is reading every cached K and V byte once: HBM-bound (per request and kv head 4 * D bytes
// per cached token against 4 * D * g flops).  Design:
//   * a workgroup of four wavefronts owns one (request, kv head, key part); the g query heads that
//     share the kv head are the columns of one matrix product, so K and V are read once for all of them;
//   * every wavefront walks its own 32-key steps (step s of the part goes to wavefront s % 4) with
//     no workgroup barrier in the loop: K and V of a step go straight from global memory into the
//     wavefront's own LDS tiles (16 bytes per lane per instruction, whole 256-byte rows, swizzled so
//     that the fragment reads are conflict-free), the next step's K is requested as soon as this
//     step's K fragments are in registers, the same for V: about 16 KB per wavefront are in flight
//     at any time, two workgroups per compute unit;
//   * scores and the PV product run on the matrix cores (S^T = K Q^T, O^T += V^T P^T with
//     32x32x16 bf16 MFMA; only g of the 32 columns are real, which costs nothing on a kernel that
//     waits for memory), V is transposed on the way out of LDS by ds_read_b64_tr_b16;
//   * the four wavefronts merge in LDS; when a request's keys are split over several workgroups
//     (few requests: the split fills the device) the parts go to scratch memory as unnormalised
//     (O, m, l) and a second small kernel merges them in a fixed order: results are deterministic.
// Keys past the end of a request's cache are loaded from a row of zeros and masked, so that stale
// page contents (which may be NaN bit patterns) never reach an MFMA.
//
// FP8 cache (template flag FP8; this build's extension, not the paper's): the pool holds E4M3 codes with
// one scale per tensor.  The codes of a step travel through registers (16 per lane and load, requested
// one step ahead), are converted to bf16 pairs by v_cvt_scalef32_pk_bf16_fp8 (exact: a code has four
// significant bits) and written into the same swizzled LDS tiles; everything after that is shared with
// the 16-bit path.  The scales are not applied per element: the K scale multiplies the scores of cached
// keys, the V scale the finished output; the new token, which is not quantised, gets the inverse factors
// on its score and on its weight in the last step.
#include <mutex>

#include "attn_common.h"

namespace {

using namespace tetri_dev;

constexpr int kWaves = 4;
constexpr int kMaxParts = 1024;   // most workgroups one (request, kv head)'s keys are split over

template <int D>
__device__ __forceinline__ void issue_tile(const char *page_lo, const char *page_hi, const char *new_row, int first_key, int L,
                                           bool is_v, int lane, uint32_t lds_base)
{
    constexpr int ROW = D * 2, NI = D / 16;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int at = i * 1024 + lane * 16;             // where this lane's 16 bytes land in the tile
        const int r = at / ROW, cpos = (at % ROW) / 16;
        const int chunk = cpos ^ (is_v ? v_swizzle<D>(r) : k_swizzle<D>(r));
        const int key = first_key + r;
        const char *src = (r < kPage ? page_lo : page_hi) + (r % kPage) * ROW;
        if (key == L) src = new_row;
        if (key > L) src = reinterpret_cast<const char *>(g_zero_row);
        dma16(src + chunk * 16, lds_base + i * 1024);
    }
}

// grid: num_reqs * Hkv * parts workgroups, part fastest
template <int D, bool FP8>
__global__ __launch_bounds__(kWaves * 64, 2) void decode_attn_kernel(DecodeParams p)
{
    constexpr int KSTEPS = D / 16, DBLK = D / 32, NI = D / 16;
    constexpr int ROW = D * 2, TILE_BYTES = 32 * ROW;      // rows and tiles in LDS are bf16 in both paths
    constexpr int ESZ = FP8 ? 1 : 2;                       // bytes of a cache element
    // FP8: a lane loads 16 codes; LPR lanes cover a row, a load instruction RPI rows, NL loads a tile
    constexpr int LPR = D / 16, RPI = 64 / LPR, NL = 32 / RPI;
    static_assert(NI == 4 || NI == 8, "wait counts below");
    __shared__ __attribute__((aligned(1024))) char smem[kWaves * 2 * TILE_BYTES];
    __shared__ float stat[kWaves][2][32];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int half = lane >> 5, l32 = lane & 31;
    int x = blockIdx.x;
    const int part = x % p.parts;
    x /= p.parts;
    const int kh = x % p.Hkv, b = x / p.Hkv;
    // a context length outside what the block table can describe is clamped: whatever the device
    // arrays hold, no address is formed from a block-table index out of range
    const int L = min(max(((const const_i32 *)(uintptr_t)p.ctx)[b], 0), p.max_blocks * kPage);
    const int steps = (L + 32) / 32;                     // 32-key steps over keys 0..L (key L is the new token)
    const int spp = (steps + p.parts - 1) / p.parts;     // steps per part
    const int s_begin = part * spp, s_end = min(steps, s_begin + spp);
    if (s_begin >= s_end) return;                        // fewer steps than parts: the merge kernel skips this part too

    const const_i32 *bt = (const const_i32 *)(uintptr_t)(p.bt + (size_t)b * p.max_blocks);
    const size_t head_bytes = (size_t)kPage * D * ESZ, page_bytes = 2 * (size_t)p.Hkv * head_bytes;
    const char *pool_k = reinterpret_cast<const char *>(p.pages) + (size_t)kh * head_bytes;
    const char *pool_v = pool_k + (size_t)p.Hkv * head_bytes;
    const char *new_k = reinterpret_cast<const char *>(p.k_new) + ((size_t)b * p.Hkv + kh) * ROW;
    const char *new_v = reinterpret_cast<const char *>(p.v_new) + ((size_t)b * p.Hkv + kh) * ROW;
    char *my = smem + wave * (2 * TILE_BYTES);
    const uint32_t k_lds = lds_address(my), v_lds = k_lds + TILE_BYTES;

    // pages of a step: clamped entries belong to keys past L and are never dereferenced
    auto page_of = [&](int step, int which) -> size_t {
        return (size_t)bt[min(2 * step + which, p.max_blocks - 1)] * page_bytes;
    };
    auto issue_k = [&](int step) {
        issue_tile<D>(pool_k + page_of(step, 0), pool_k + page_of(step, 1), new_k, step * 32, L, false, lane, k_lds);
    };
    auto issue_v = [&](int step) {
        issue_tile<D>(pool_v + page_of(step, 0), pool_v + page_of(step, 1), new_v, step * 32, L, true, lane, v_lds);
    };

    // FP8: the codes of one matrix of one step, 16 per lane and load; keys at and past L load nothing
    [[maybe_unused]] u32x4 rk[NL], rv[NL];
    auto load_codes = [&](const char *pool, int step, u32x4 (&raw)[NL]) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int r = i * RPI + lane / LPR;
            const char *src = pool + page_of(step, (i * RPI) / kPage) + (size_t)(r % kPage) * D + (lane % LPR) * 16;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (step * 32 + r < L) v = *reinterpret_cast<const u32x4 *>(src);
            raw[i] = v;
        }
    };
    // ... converted to bf16 and written to the wavefront's tile: codes c16*16 .. +15 of row r are two
    // 16-byte chunks of the bf16 row
    auto write_codes = [&](const u32x4 (&raw)[NL], bool is_v) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int r = i * RPI + lane / LPR, c16 = lane % LPR;
            u32x4 lo, hi;
            codes_to_bf16(raw[i], lo, hi);
            const int swz = is_v ? v_swizzle<D>(r) : k_swizzle<D>(r);
            char *row = my + (is_v ? TILE_BYTES : 0) + r * ROW;
            *reinterpret_cast<u32x4 *>(row + (((2 * c16) ^ swz) << 4)) = lo;
            *reinterpret_cast<u32x4 *>(row + (((2 * c16 + 1) ^ swz) << 4)) = hi;
        }
    };

    // the first step's K and V are requested before anything else is read
    int st = s_begin + wave;
    if (st < s_end) {
        if constexpr (FP8) {
            load_codes(pool_k, st, rk);
            load_codes(pool_v, st, rv);
        } else {
            issue_k(st);
            issue_v(st);
        }
    }
    // Fused append: the workgroup whose part ends with key L caches the new token's K and V row of
    // this kv head in slot L % 16 of page block_table[b][L / 16] (16 bytes per lane; nothing in this
    // launch reads that slot: every wavefront takes key L from k_new / v_new).
    // With an FP8 cache the row is quantised on the way: fl32(x * inv_scale) clamped to +-448, rounded to
    // nearest even by v_cvt_pk_fp8_f32, 8 codes per lane.
    if (p.pages_w != nullptr && s_end == steps && wave == kWaves - 1 && lane < 2 * (ROW / 16) && L < p.max_blocks * kPage) {
        const int which = lane / (ROW / 16), chunk = lane % (ROW / 16);
        const size_t at = (size_t)bt[L / kPage] * page_bytes + ((size_t)which * p.Hkv + kh) * head_bytes
                          + ((size_t)(L % kPage) * ROW + chunk * 16) / 2 * ESZ;
        const u32x4 v = *reinterpret_cast<const u32x4 *>((which ? new_v : new_k) + chunk * 16);
        if constexpr (FP8) {
            *reinterpret_cast<uint2 *>(reinterpret_cast<char *>(p.pages_w) + at) = bf16_to_codes(v, which ? p.v_inv : p.k_inv);
        } else {
            *reinterpret_cast<u32x4 *>(reinterpret_cast<char *>(p.pages_w) + at) = v;
        }
    }
    // Q fragments (B operand of S^T = K Q^T): column l32 is query head kh * g + l32, zero past g
    bf16x8 qf[KSTEPS];
    {
        const uint4 *qp = reinterpret_cast<const uint4 *>(p.q + ((size_t)b * p.Hq + (size_t)kh * p.g + min(l32, p.g - 1)) * D);
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) {
            uint4 v = qp[2 * st + half];
            if (l32 >= p.g) v = make_uint4(0, 0, 0, 0);
            qf[st] = __builtin_bit_cast(bf16x8, v);
        }
    }
    // fragment addresses inside the wavefront's tiles (the layouts of the chunked-prefill kernel)
    uint32_t kbase[KSTEPS], vbase[DBLK];
    {
        const int blk = lane >> 4, i16 = lane & 15;
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) kbase[st] = l32 * ROW + (((2 * st + half) ^ k_swizzle<D>(l32)) << 4);
        const int rv = 4 * half + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            const int d0 = db * 32 + 16 * (blk & 1) + 4 * (i16 & 3);
            vbase[db] = TILE_BYTES + rv * ROW + (((d0 >> 3) ^ v_swizzle<D>(rv)) << 4) + ((d0 & 7) << 1);
        }
    }

    f32x16 o[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m = -1e30f, lsum = 0.f;
    // FP8: the tiles hold code values; the K scale rides on the score factor (sign of c unchanged: scales
    // are positive)
    const float c = (p.neg ? -p.c : p.c) * (FP8 ? p.k_scale : 1.0f);
    const float masked = p.neg ? INFINITY : -INFINITY;
    bf16x2 ones;
    ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;

    for (; st < s_end; st += kWaves) {
        const bool more = st + kWaves < s_end;
        if constexpr (FP8) {
            // this step's codes (the compiler waits for the loads) become bf16 tiles; the row of the new
            // token, not quantised, is copied over its zeros; then the next step's codes are requested
            write_codes(rk, false);
            write_codes(rv, true);
            if (st == steps - 1 && lane < ROW / 16) {
                const int r = L - st * 32;
                *reinterpret_cast<u32x4 *>(my + r * ROW + ((lane ^ k_swizzle<D>(r)) << 4)) =
                    *reinterpret_cast<const u32x4 *>(new_k + lane * 16);
                *reinterpret_cast<u32x4 *>(my + TILE_BYTES + r * ROW + ((lane ^ v_swizzle<D>(r)) << 4)) =
                    *reinterpret_cast<const u32x4 *>(new_v + lane * 16);
            }
            if (more) {
                load_codes(pool_k, st + kWaves, rk);
                load_codes(pool_v, st + kWaves, rv);
            }
            asm volatile("" ::: "memory");               // the fragment reads below stay behind the tile writes
        } else {
            // K of this step has landed when only the V loads behind it are outstanding
            wait_vm<NI>();
        }
        bf16x8 kf[KSTEPS];
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) kf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(my + kbase[s]));
        if constexpr (!FP8) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // fragments are in registers: the tile may be overwritten
            if (more) issue_k(st + kWaves);
        }
        f32x16 sc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < KSTEPS; ++s) sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[s], sc, 0, 0, 0);
        // accumulator element v is key 32 * st + 8 * (v / 4) + 4 * half + v % 4; keys past L do not exist
        if (st * 32 + 31 > L) {
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (st * 32 + (v / 4) * 8 + 4 * half + (v % 4) > L) sc[v] = masked;
        }
        if constexpr (FP8) {
            if (st == steps - 1) {                       // the new token's key carries no K scale
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (st * 32 + (v / 4) * 8 + 4 * half + (v % 4) == L) sc[v] *= p.k_inv;
            }
        }
        float mx = sc[0] * c;
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sc[v] * c);
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m, mx);
        const float alpha = __builtin_amdgcn_exp2f(m - m_new);
        m = m_new;
        bf16x8 pf[2];
        float l_blk = 0.f;
#pragma unroll
        for (int v = 0; v < 16; v += 2) {
            bf16x2 pp;
            pp[0] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sc[v], c, -m));
            pp[1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sc[v + 1], c, -m));
            l_blk = __builtin_amdgcn_fdot2_f32_bf16(pp, ones, l_blk, false);
            pf[v / 8][v % 8] = pp[0];
            pf[v / 8][v % 8 + 1] = pp[1];
        }
        lsum = lsum * alpha + l_blk;
        if constexpr (FP8) {
            // ... and its value no V scale: the finished output is multiplied by the V scale, so the new
            // token's weight is divided by it
            if (st == steps - 1) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    if (st * 32 + (v / 4) * 8 + 4 * half + (v % 4) == L)
                        pf[v / 8][v % 8] = (__bf16)((float)pf[v / 8][v % 8] * p.v_inv);
            }
        }
#pragma unroll
        for (int i = 0; i < DBLK; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[i][v] *= alpha;
        if constexpr (!FP8) {
            // V of this step: behind it only the next step's K loads
            if (more) wait_vm<NI>();
            else wait_vm<0>();
        }
        s16x8 vf[2 * DBLK];
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                const char *a = my + vbase[db] + j * (16 * ROW);
                const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a);
                const s16x4 vb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + 8 * ROW));
                vf[j * DBLK + db] = __builtin_shufflevector(va, vb, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        if constexpr (!FP8) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (more) issue_v(st + kWaves);
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[j * DBLK + db]), pf[j], o[db], 0, 0, 0);
    }

    // ---- the four wavefronts meet in LDS: each writes its unnormalised O (real columns only) into
    // its own tiles (all its loads have landed, nobody else touches them), m and the row sum beside
    const float ltot = half_swap_sum(lsum);
    if (l32 < p.g) {
        float *mine = reinterpret_cast<float *>(my) + l32 * D;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f32x4 v4;
#pragma unroll
                for (int e = 0; e < 4; ++e) v4[e] = o[db][q4 * 4 + e];
                *reinterpret_cast<f32x4 *>(mine + 32 * db + 8 * q4 + 4 * half) = v4;
            }
        if (half == 0) { stat[wave][0][l32] = m; stat[wave][1][l32] = ltot; }
    }
    __syncthreads();
    for (int idx = tid; idx < p.g * D; idx += kWaves * 64) {
        const int col = idx / D, d = idx - col * D;
        float ms = stat[0][0][col];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, stat[w][0][col]);
        float acc = 0.f, l = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float wgt = __builtin_amdgcn_exp2f(stat[w][0][col] - ms);
            acc = __builtin_fmaf(reinterpret_cast<const float *>(smem + w * (2 * TILE_BYTES))[col * D + d], wgt, acc);
            l = __builtin_fmaf(stat[w][1][col], wgt, l);
        }
        const size_t head = (size_t)b * p.Hq + (size_t)kh * p.g + col;
        if (p.parts == 1) {
            p.out[head * D + d] = __builtin_bit_cast(uint16_t, (__bf16)(acc / l * p.out_scale));
        } else {
            float *dst = p.partial + (head * p.parts + part) * (D + 2);
            dst[d] = acc;
            if (d == 0) { dst[D] = ms; dst[D + 1] = l; }
        }
    }
}

// grid: num_reqs * Hq workgroups: merges the parts of one (request, head).  The parts' weights are
// computed once (one part per thread), then thread (group, d) sums every (256 / D)-th part of element
// d with several loads in flight and the groups are added in a fixed order: deterministic.
template <int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(DecodeParams p)
{
    constexpr int G = 256 / D;
    __shared__ float w[kMaxParts];
    __shared__ float red[2][4];
    __shared__ float sums[G][D];
    const int b = blockIdx.x / p.Hq, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int L = min(max(p.ctx[b], 0), p.max_blocks * kPage);     // clamped as in the main kernel
    const int steps = (L + 32) / 32;
    const int spp = (steps + p.parts - 1) / p.parts;
    const int used = (steps + spp - 1) / spp;            // parts that had keys (1 <= used <= parts)
    const float *src = p.partial + (size_t)blockIdx.x * p.parts * (D + 2);
    float ms = -INFINITY;
    for (int q = tid; q < used; q += 256) ms = fmaxf(ms, src[q * (D + 2) + D]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) ms = fmaxf(ms, __shfl_xor(ms, d));
    if (lane == 0) red[0][wave] = ms;
    __syncthreads();
    ms = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    float l = 0.f;
    for (int q = tid; q < used; q += 256) {
        const float wq = __builtin_amdgcn_exp2f(src[q * (D + 2) + D] - ms);
        w[q] = wq;
        l = __builtin_fmaf(src[q * (D + 2) + D + 1], wq, l);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) l += __shfl_xor(l, d);
    if (lane == 0) red[1][wave] = l;
    __syncthreads();
    l = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    const int grp = tid / D, d = tid - grp * D;
    float acc = 0.f;
#pragma unroll 4
    for (int q = grp; q < used; q += G) acc = __builtin_fmaf(src[q * (D + 2) + d], w[q], acc);
    sums[grp][d] = acc;
    __syncthreads();
    if (grp == 0) {
#pragma unroll
        for (int g = 1; g < G; ++g) acc += sums[g][d];
        p.out[(size_t)blockIdx.x * D + d] = __builtin_bit_cast(uint16_t, (__bf16)(acc / l * p.out_scale));
    }
}

}  // namespace

// Scratch memory of tetri_decode_attn_static: the parts of split requests, in an array that is part
// of the loaded code object instead of an allocation (8 MiB on every device the library runs on,
// held until the process ends).  On the host the array's name is only a stand-in for the symbol: the
// device address is looked up once per device, with that device current, and only that address
// is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[kDecodeStaticScratchBytes];

hipError_t tetri_decode_static_scratch(float **ptr, size_t *bytes)
{
    constexpr int kMaxDevices = 64;
    static std::mutex lock;
    static void *per_device[kMaxDevices];               // zero until the device's address is known
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(lock);
    if (!per_device[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        per_device[dev] = p;
    }
    *ptr = static_cast<float *>(per_device[dev]);
    *bytes = kDecodeStaticScratchBytes;
    return hipSuccess;
}

hipError_t tetri_launch_decode(const tetri_ctx *h, const DecodeParams &p, hipStream_t stream)
{
    const dim3 grid(p.B * p.Hkv * p.parts), block(kWaves * 64);
    const int d = h->cfg.head_dim;
    if (d == 128 && !p.fp8) hipLaunchKernelGGL((decode_attn_kernel<128, false>), grid, block, 0, stream, p);
    else if (d == 64 && !p.fp8) hipLaunchKernelGGL((decode_attn_kernel<64, false>), grid, block, 0, stream, p);
    else if (d == 128) hipLaunchKernelGGL((decode_attn_kernel<128, true>), grid, block, 0, stream, p);
    else if (d == 64) hipLaunchKernelGGL((decode_attn_kernel<64, true>), grid, block, 0, stream, p);
    else return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || p.parts == 1) return e;
    if (p.parts > kMaxParts) return hipErrorInvalidValue;
    if (d == 128) hipLaunchKernelGGL(decode_merge_kernel<128>, dim3(p.B * p.Hq), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(decode_merge_kernel<64>, dim3(p.B * p.Hq), dim3(256), 0, stream, p);
    return hipGetLastError();
}
