// Device helpers shared by the attention kernels of libtetri (gfx950 only).
#pragma once
#include "tetri_internal.h"

namespace tetri_dev {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
// Accesses through these go out as global-memory instructions whatever the compiler knows about the pointer.  (An
// access through a generic pointer is a FLAT instruction, which also counts as an LDS operation: every later wait
// for LDS reads then waits for it.)
typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
typedef __attribute__((address_space(1))) u32x4 global_u32x4_w;

constexpr int kPage = 16;     // tokens per KV page
constexpr int kXcd = 8;       // XCDs (L2 domains) workgroups are dealt to round-robin

// Numbered points of the kernels' timelines.  The library compiles them to nothing; a measurement
// build may define the macro before this header (e.g. to store a clock value per wavefront).
#ifndef TETRI_MARK
#define TETRI_MARK(i_) do { } while (0)
#endif

// A row of zeros: out-of-range key rows of a partial tile are loaded from here.
static __device__ __attribute__((aligned(256))) uint4 g_zero_row[16];

template <int D> __host__ __device__ __forceinline__ constexpr int k_swizzle(int row)
{
    // 16 consecutive rows must land in 16 different 16-byte bank groups
    return (D == 128) ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __host__ __device__ __forceinline__ constexpr int v_swizzle(int row)
{
    // 4 consecutive rows x 64 contiguous bytes must land in 4 different 64-byte bank groups
    return (D == 128) ? ((row & 3) << 2) : (((row ^ (row >> 1)) & 1) << 2);
}

// n / d for a divisor fixed at launch: magic = ceil(2^32 / d), or 0 for d = 1.  Exact while
// n * d < 2^32 (the host checks the launch's largest n).
__device__ __forceinline__ int magic_div(int n, uint32_t magic)
{
    return magic != 0 ? (int)__umulhi((uint32_t)n, magic) : n;
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


// Direct global -> LDS load of 16 bytes per lane, issued from inline assembly: lane l's 16 bytes
// land at LDS byte address lds_base + 16*l (lds_base is wave-uniform and goes to M0).  The
// compiler does not see this as a memory access, so it inserts no waits for it: the caller
// orders it with wait_vm<N>() below.  (The compiler's own tracking of such loads cannot tell
// apart two buffers that are slices of one array and falls back to waiting for everything.)
// Wave-uniform operands of the loads below, marked as such: they go into scalar registers whatever
// the compiler thinks of where they were computed.
__device__ __forceinline__ const void *uniform_ptr(const void *p)
{
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const void *)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_base)
{
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_base) : "memory", "m0");
}
// A group of such loads that share one scalar base and one LDS base: instruction i moves
// 16 bytes per lane from sbase + voff_i + 1024*i to LDS byte lds_base + 1024*i + 16*lane.  The
// instruction's immediate offset advances the global and the LDS address alike, so M0 is written
// once per group.
__device__ __forceinline__ void dma16_group4(const void *sbase, uint32_t v0, uint32_t v1, uint32_t v2, uint32_t v3, uint32_t lds_base)
{
    sbase = uniform_ptr(sbase);
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %5\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, %4\n\t"
                 "global_load_lds_dwordx4 %1, %4 offset:1024\n\t"
                 "global_load_lds_dwordx4 %2, %4 offset:2048\n\t"
                 "global_load_lds_dwordx4 %3, %4 offset:3072" ::"v"(v0), "v"(v1), "v"(v2), "v"(v3), "s"(sbase), "s"(lds_base) : "memory", "m0");
}
__device__ __forceinline__ void dma16_group2(const void *sbase, uint32_t v0, uint32_t v1, uint32_t lds_base)
{
    sbase = uniform_ptr(sbase);
    lds_base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\t"
                 "global_load_lds_dwordx4 %0, %2\n\t"
                 "global_load_lds_dwordx4 %1, %2 offset:1024" ::"v"(v0), "v"(v1), "s"(sbase), "s"(lds_base) : "memory", "m0");
}
// Accesses that are coherent across the whole device by themselves (cache policy sc1: they are
// served by the memory side, not by an XCD's L2), for data handed from one workgroup to another
// inside a launch.  No cache write-back or invalidation is needed around them, only order:
// coherent_stores_done() returns when this wavefront's stores have been performed.
__device__ __forceinline__ void store_coherent(f32x4 *p, f32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store_coherent(float *p, float v)
{
    asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void coherent_stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// A coherent read of one word that is not needed yet: every lane's copy of it goes to 256 bytes
// of LDS at lds_dst; it is there after wait_vm<0>().
__device__ __forceinline__ void peek_coherent(const void *p, uint32_t lds_dst)
{
    lds_dst = __builtin_amdgcn_readfirstlane(lds_dst);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off sc1" ::"v"(p), "s"(lds_dst) : "memory", "m0");
}
// A partial result read back in one go: n 16-byte vectors 1 KB apart from `po` on, two floats 128
// bytes apart at `ps`; one round trip to memory, all loads in flight together.  (One assembly
// statement including the wait: the registers are written long after the loads are issued, which
// the compiler must not get a chance to forget.)
__device__ __forceinline__ void load_partial(const f32x4 *po, const float *ps, f32x4 (&x)[16], float &a, float &b)
{
    const f32x4 *p1 = po + 4 * 64, *p2 = po + 8 * 64, *p3 = po + 12 * 64;
    asm volatile("global_load_dword %16, %22, off sc1\n\t"
                 "global_load_dword %17, %22, off offset:128 sc1\n\t"
                 "global_load_dwordx4 %0, %18, off sc1\n\t"
                 "global_load_dwordx4 %1, %18, off offset:1024 sc1\n\t"
                 "global_load_dwordx4 %2, %18, off offset:2048 sc1\n\t"
                 "global_load_dwordx4 %3, %18, off offset:3072 sc1\n\t"
                 "global_load_dwordx4 %4, %19, off sc1\n\t"
                 "global_load_dwordx4 %5, %19, off offset:1024 sc1\n\t"
                 "global_load_dwordx4 %6, %19, off offset:2048 sc1\n\t"
                 "global_load_dwordx4 %7, %19, off offset:3072 sc1\n\t"
                 "global_load_dwordx4 %8, %20, off sc1\n\t"
                 "global_load_dwordx4 %9, %20, off offset:1024 sc1\n\t"
                 "global_load_dwordx4 %10, %20, off offset:2048 sc1\n\t"
                 "global_load_dwordx4 %11, %20, off offset:3072 sc1\n\t"
                 "global_load_dwordx4 %12, %21, off sc1\n\t"
                 "global_load_dwordx4 %13, %21, off offset:1024 sc1\n\t"
                 "global_load_dwordx4 %14, %21, off offset:2048 sc1\n\t"
                 "global_load_dwordx4 %15, %21, off offset:3072 sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]), "=&v"(x[7]),
                   "=&v"(x[8]), "=&v"(x[9]), "=&v"(x[10]), "=&v"(x[11]), "=&v"(x[12]), "=&v"(x[13]), "=&v"(x[14]), "=&v"(x[15]),
                   "=&v"(a), "=&v"(b)
                 : "v"(po), "v"(p1), "v"(p2), "v"(p3), "v"(ps) : "memory");
}
__device__ __forceinline__ void load_partial(const f32x4 *po, const float *ps, f32x4 (&x)[8], float &a, float &b)
{
    const f32x4 *p1 = po + 4 * 64;
    asm volatile("global_load_dword %8, %12, off sc1\n\t"
                 "global_load_dword %9, %12, off offset:128 sc1\n\t"
                 "global_load_dwordx4 %0, %10, off sc1\n\t"
                 "global_load_dwordx4 %1, %10, off offset:1024 sc1\n\t"
                 "global_load_dwordx4 %2, %10, off offset:2048 sc1\n\t"
                 "global_load_dwordx4 %3, %10, off offset:3072 sc1\n\t"
                 "global_load_dwordx4 %4, %11, off sc1\n\t"
                 "global_load_dwordx4 %5, %11, off offset:1024 sc1\n\t"
                 "global_load_dwordx4 %6, %11, off offset:2048 sc1\n\t"
                 "global_load_dwordx4 %7, %11, off offset:3072 sc1\n\t"
                 "s_waitcnt vmcnt(0)"
                 : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]), "=&v"(x[7]),
                   "=&v"(a), "=&v"(b)
                 : "v"(po), "v"(p1), "v"(ps) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}
// Wait until at most N vector-memory operations of this wavefront are outstanding; also a
// compiler barrier for memory accesses, so LDS reads stay behind it.
template <int N> __device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N < 64, "the counter has six bits");
    // s_waitcnt operand of gfx9: vmcnt in bits 3:0 and 15:14, expcnt (6:4) and lgkmcnt (11:8) left at their maxima
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
    asm volatile("" ::: "memory");
}
// A workgroup barrier that orders LDS accesses only: vector-memory operations in flight (loads into
// other LDS buffers, stores of results) are not waited for.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// FP8 E4M3 cache: 16 codes (one 16-byte load) to 16 bf16 values, exactly (a code has four significant bits): lo
// gets the values of codes 0..7, hi those of codes 8..15.
__device__ __forceinline__ void codes_to_bf16(const u32x4 &raw, u32x4 &lo, u32x4 &hi)
{
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        lo[2 * w] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[w], 1.0f, false));
        lo[2 * w + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[w], 1.0f, true));
        hi[2 * w] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[2 + w], 1.0f, false));
        hi[2 * w + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(raw[2 + w], 1.0f, true));
    }
}
// ... and 8 bf16 values (16 bytes) to their 8 codes under fl32(1 / scale) = inv: fl32(x * inv) clamped to +-448,
// rounded to nearest even by v_cvt_pk_fp8_f32.
__device__ __forceinline__ uint2 bf16_to_codes(const u32x4 &v, float inv)
{
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
    return make_uint2(codes[0], codes[1]);
}

// Relaxed device-scope fetch-and-add on a word of global memory, as a global-memory instruction (see above).
__device__ __forceinline__ int atomic_add_global(int32_t *p, int v)
{
    return __hip_atomic_fetch_add(reinterpret_cast<__attribute__((address_space(1))) int32_t *>((uintptr_t)p), v, __ATOMIC_RELAXED,
                                  __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void store_global(int32_t *p, int32_t v)
{
    *reinterpret_cast<__attribute__((address_space(1))) int32_t *>((uintptr_t)p) = v;
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


}  // namespace tetri_dev
