// Chunked-prefill causal attention over a paged KV cache for gfx950 (CDNA4): shared-tile kernel.
// TetriInfer Sec. 3.3.3 (prefill one fixed-size chunk at a time; several requests may be merged
// into a chunk), Sec. 2.1 (causal prefill), Sec. 3.4 (paged KV).  The kernel is a flash-style
// single pass with online softmax; that structure is prior art (the paper names FlashAttention
// as orthogonal work), the paper itself gives no kernel.
//
// Mapping to the hardware
//   * A workgroup is 4*KS wavefronts.  A wavefront owns 32 query rows of one query head and one
//     of KS parts of every key stage; the 4 row/head slots are (heads sharing one kv head) x
//     (32-row blocks).  With KS = 2 a CU holds 8 wavefronts, two per SIMD, so one wavefront's
//     softmax (VALU) overlaps the other's MFMA, while every K/V byte brought into LDS still
//     serves 128 query rows.  The KS partial results are merged once through LDS at the end.
//     With KS = 1 a workgroup has 4 wavefronts and half the LDS, two workgroups share a CU and the
//     two wavefronts of a SIMD belong to different workgroups (no common barrier); the library
//     uses it for launches with at least two workgroups per CU (see softmax_pv for its schedule).
//   * A stage is 64*KS keys of K and V.  Stages go from HBM/L2 straight into LDS with
//     global_load_lds_dwordx4 (no register staging), double buffered: the loads of stage i+1 are
//     in flight while stage i is consumed; one workgroup barrier per stage.  The 16 key rows a
//     wavefront loads per stage are exactly one (page, kv head) block of the pool, 4 KB
//     contiguous: one scalar base address per block, per-lane offsets fixed for the whole kernel.
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
//   * Workgroup ids are remapped so that all workgroups of a kv head run on one XCD (one L2).
//   * Two ways of handing out the work of a head group (all row tiles of the heads of one
//     workgroup column):
//       - tile mode: one workgroup per row tile, long (late) tiles first; for launches with at
//         least two workgroups per compute unit;
//       - stream mode: the stages of all tiles of the head group, laid end to end in tile order,
//         are cut into G equal ranges, one per workgroup (G = compute units / head groups), so
//         every compute unit gets the same number of stages however the causal triangle and the
//         segment lengths fall.  A range may start and end inside a tile: the pieces of such a
//         tile meet in scratch memory of the library's handle, without anybody waiting: every
//         piece but the last to arrive leaves its unnormalised (O, m, row sum) there, the last
//         one merges all of them in piece order (see finish_tile).  A workgroup whose range
//         spans several tiles runs them as consecutive jobs; the first K/V stage and the Q rows of
//         the next job are requested before the current job's epilogue.
//   * The fused form of the launch has further workgroups that copy the chunk's new K/V rows
//     into the page pool (append_rows).
#include <type_traits>

#include "attn_common.h"

namespace {

using namespace tetri_dev;

constexpr int kSlots = 4;     // (head, 32-row block) slots of a workgroup
constexpr int kBNW = 64;      // keys per wavefront per stage

// Per-lane byte offsets of a wavefront's loads, fixed for the whole kernel.
// A wavefront loads 16 key rows per stage with NI = 4 (head_dim 128) or 2 (head_dim 64)
// instructions of 1 KB; lane l of instruction i lands at LDS byte 1024*i + 16*l, i.e. row
// r = RPI*i + l/CH of the wavefront's 16 rows, chunk position l%CH, and therefore fetches chunk
// (l%CH) ^ swizzle(r) of that row.  RPI*i only touches swizzle bits that l/CH leaves free, so
// instruction i's offset is instruction 0's offset with a constant XOR-ed in, plus i row groups.
template <int D>
struct LaneOffsets {
    uint32_t k_ctx, v_ctx;      // rows 512 (256) bytes apart inside a (page, head) block of the pool
};

// The lane index, read anew from the thread id.  Values derived from it where they are needed do not occupy
// registers across the main loop, which has none to spare.
__device__ __forceinline__ int fresh_lane()
{
    int x = threadIdx.x;
    asm volatile("" : "+v"(x));
    return x & 63;
}

template <int D>
__device__ __forceinline__ void init_lane_offsets(LaneOffsets<D> &lo, int lane)
{
    constexpr int CH = D / 8;
    const int r0 = lane / CH;                                    // row of instruction 0
    const int kc = (lane % CH) ^ k_swizzle<D>(r0);
    const int vc = (lane % CH) ^ v_swizzle<D>(r0);
    lo.k_ctx = r0 * D * 2 + kc * 16;
    lo.v_ctx = r0 * D * 2 + vc * 16;
}
// XOR that turns instruction 0's chunk into instruction i's (in bytes).
template <int D> __host__ __device__ __forceinline__ constexpr uint32_t k_inst_xor(int i)
{
    return (uint32_t)(k_swizzle<D>((64 / (D / 8)) * i) * 16);
}
template <int D> __host__ __device__ __forceinline__ constexpr uint32_t v_inst_xor(int i)
{
    return (uint32_t)(v_swizzle<D>((64 / (D / 8)) * i) * 16);
}

// Where the keys of one job (a stage range of one row tile) come from; wave-uniform.
struct JobSrc {
    int bt_off;                 // block-table row of the tile's segment: entries from the start of the table
    uint32_t new_off;           // first row of the segment, kv head of the workgroup: bytes from the start of k_new / v_new
    int L;                      // cached tokens of the segment's request
    int n_new;                  // new keys any row of the tile may see
    int n_ctx_tiles;            // stages of cached keys
};

// One job of a workgroup: stages [it_begin, it_end) of one row tile; wave-uniform.
struct Job {
    int seg_cu, n_s, t0;        // the tile's segment starts at chunk row seg_cu and has n_s rows; the tile starts at its row t0
    int tile_index;             // index of the tile in the chunk (names its arrival counters)
    int it_begin, it_end;
    int piece, npieces, wf;     // which of the tile's pieces this is, how many there are, the workgroup of piece 0
    JobSrc src;
};

// One of two jobs, chosen field by field (a choice between the addresses of two jobs would keep both in memory).
__device__ __forceinline__ Job pick(bool first, const Job &a, const Job &b)
{
    Job r;
    r.seg_cu = first ? a.seg_cu : b.seg_cu; r.n_s = first ? a.n_s : b.n_s; r.t0 = first ? a.t0 : b.t0;
    r.tile_index = first ? a.tile_index : b.tile_index;
    r.it_begin = first ? a.it_begin : b.it_begin; r.it_end = first ? a.it_end : b.it_end;
    r.piece = first ? a.piece : b.piece; r.npieces = first ? a.npieces : b.npieces; r.wf = first ? a.wf : b.wf;
    r.src.bt_off = first ? a.src.bt_off : b.src.bt_off; r.src.new_off = first ? a.src.new_off : b.src.new_off;
    r.src.L = first ? a.src.L : b.src.L; r.src.n_new = first ? a.src.n_new : b.src.n_new;
    r.src.n_ctx_tiles = first ? a.src.n_ctx_tiles : b.src.n_ctx_tiles;
    return r;
}

// Wave-uniform pieces of a wavefront's load addresses that no job changes.
struct WaveSrc {
    const int32_t *bt;          // the block table
    const char *new_k, *new_v;  // k_new and v_new
    const char *pool_k;         // K block of the workgroup's kv head in page 0 of the pool
    uint32_t page_bytes;        // one page: K and V blocks of every kv head
    uint32_t v_delta;           // from a page's K block to its V block of the same head
    uint32_t stage_new_bytes;   // a stage's worth of rows in k_new / v_new
    uint32_t wave_new_bytes;    // a wavefront's 16 rows
    int max_blocks;
};

template <int D, int KS, bool F8>
__device__ __forceinline__ WaveSrc make_wave_src(const AttnParams &p, int kh)
{
    constexpr int ESZ = F8 ? 1 : 2;                    // bytes of a pool element
    WaveSrc ws;
    ws.bt = p.bt;
    ws.new_k = reinterpret_cast<const char *>(p.k_new);
    ws.new_v = reinterpret_cast<const char *>(p.v_new);
    ws.pool_k = reinterpret_cast<const char *>(p.pages) + (size_t)kh * (kPage * D * ESZ);
    ws.page_bytes = 2 * p.Hkv * (kPage * D * ESZ);
    ws.v_delta = p.Hkv * (kPage * D * ESZ);
    ws.stage_new_bytes = (kBNW * KS) * (p.Hkv * D * 2);
    ws.wave_new_bytes = 16 * (p.Hkv * D * 2);
    ws.max_blocks = p.max_blocks;
    return ws;
}

// The direct-to-LDS loads of this wavefront's 16 rows of one stage (K and V): one scalar base per
// matrix; the NI instructions of a matrix differ only in their per-lane offsets.
struct StageLoads {
    const char *kb, *vb;        // row j0 of the stage part, K and V
    uint32_t step;              // bytes the rows of two instructions are further apart than 1 KB
    uint32_t kdst;              // LDS byte address of the K rows; the V rows are 2 * STAGE_BYTES further
    int j0, limit;              // first key row, and the end of the key range it belongs to
    uint32_t ko, vo;            // per-lane byte offsets of the first instruction's rows, K and V
    bool codes;                 // the rows are FP8 codes of a pool of codes: they travel through registers (fetch_stage_codes)
};

// Where stage `it` of a job comes from.  Returns whether all 16 rows exist.
template <int D, int KS, bool F8 = false>
__device__ __forceinline__ bool describe_stage_loads(const JobSrc &src, const WaveSrc &ws, const LaneOffsets<D> &lo, int page, int it,
                                                     int wave, int new_row_bytes, uint32_t k_lds, StageLoads &sl)
{
    constexpr int RPI = 64 / (D / 8);
    constexpr int STAGE = kBNW * KS;
    const bool ctx = it < src.n_ctx_tiles;
    const int jn = it - src.n_ctx_tiles;
    sl.j0 = (ctx ? it : jn) * STAGE + 16 * wave;
    sl.limit = ctx ? src.L : src.n_new;
    sl.kdst = k_lds + wave * (16 * D * 2);
    sl.codes = F8 && ctx;
    // (a lane's row is further away in k_new / v_new, whose rows are Hkv*D*2 bytes apart, than in a page)
    const uint32_t new_extra = ctx ? 0u : (uint32_t)(fresh_lane() / (D / 8)) * (uint32_t)(new_row_bytes - D * 2);
    sl.ko = lo.k_ctx + new_extra;
    sl.vo = lo.v_ctx + new_extra;
    // pool rows of an instruction follow the previous one's directly (the immediate offset covers
    // it); rows of k_new / v_new are `step` bytes further apart than that
    if (ctx) {
        sl.kb = ws.pool_k + (size_t)page * ws.page_bytes;
        sl.vb = sl.kb + ws.v_delta;
        sl.step = 0;
    } else {
        const size_t off = (size_t)src.new_off + (size_t)jn * ws.stage_new_bytes + (size_t)wave * ws.wave_new_bytes;
        sl.kb = ws.new_k + off;
        sl.vb = ws.new_v + off;
        sl.step = RPI * new_row_bytes - 1024;
    }
    return sl.j0 + 16 <= sl.limit;
}

// All loads of a stage at once.
template <int D, int KS>
__device__ __forceinline__ void issue_stage_loads(const StageLoads &sl, bool full)
{
    constexpr int CH = D / 8, RPI = 64 / CH, NI = 16 / RPI;
    constexpr uint32_t V_LDS = 2 * (kBNW * KS) * D * 2;
    static_assert(RPI * D * 2 == 1024 && (NI == 4 || NI == 2), "one instruction moves 1 KB");
    const uint32_t ko = sl.ko, vo = sl.vo, step = sl.step;
    const uint32_t kdst = sl.kdst, vdst = sl.kdst + V_LDS;
    if (full) {
        if constexpr (NI == 4) {
            dma16_group4(sl.kb, ko, (ko ^ k_inst_xor<D>(1)) + step, (ko ^ k_inst_xor<D>(2)) + 2 * step, (ko ^ k_inst_xor<D>(3)) + 3 * step, kdst);
            dma16_group4(sl.vb, vo, (vo ^ v_inst_xor<D>(1)) + step, (vo ^ v_inst_xor<D>(2)) + 2 * step, (vo ^ v_inst_xor<D>(3)) + 3 * step, vdst);
        } else {
            dma16_group2(sl.kb, ko, (ko ^ k_inst_xor<D>(1)) + step, kdst);
            dma16_group2(sl.vb, vo, (vo ^ v_inst_xor<D>(1)) + step, vdst);
        }
    } else {
        // ragged end of the key range: rows past the limit come from a row of zeros
        const char *zero = reinterpret_cast<const char *>(g_zero_row);
        const int lane = fresh_lane();
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bool ok = sl.j0 + RPI * i + lane / CH < sl.limit;
            const size_t inst = (size_t)i * (step + 1024);
            dma16(ok ? sl.kb + inst + (ko ^ k_inst_xor<D>(i)) : zero, kdst + 1024 * i);
            dma16(ok ? sl.vb + inst + (vo ^ v_inst_xor<D>(i)) : zero, vdst + 1024 * i);
        }
    }
}

// A pool of FP8 codes: the 16 cached key rows a wavefront loads per stage are 16 * D bytes of K and as many of V,
// each one contiguous (page, kv head) block.  They travel through registers: 16 codes per lane and load (D / 16
// lanes cover a row), requested where the 16-bit path issues its direct loads and, once arrived, converted to bf16
// (exactly) and written to the stage buffer in the layout the direct loads produce (write_stage_codes), before
// the barrier that opens the stage.  The scales are not applied per element (see tile_job).
template <int D>
struct StageCodes {
    u32x4 k[D / 64], v[D / 64];
};

template <int D>
__device__ __forceinline__ void fetch_stage_codes(const StageLoads &sl, bool full, StageCodes<D> &sc)
{
    constexpr int NL = D / 64, LPR = D / 16, RPL = 64 / LPR;     // loads per matrix, lanes per row, rows per load
    const int lane = fresh_lane();
    const char *kb = sl.kb + lane * 16, *vb = sl.vb + lane * 16;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        // rows past the end of the cached context hold whatever the pool holds: they read as zeros
        const bool ok = full || sl.j0 + RPL * i + lane / LPR < sl.limit;
        u32x4 a = {0u, 0u, 0u, 0u}, b = {0u, 0u, 0u, 0u};
        if (ok) {
            // (through the global address space: a load through a generic pointer also counts as an LDS operation,
            // and the next wait for LDS reads would wait for it)
            a = *reinterpret_cast<global_u32x4 *>((uintptr_t)(kb + 1024 * i));
            b = *reinterpret_cast<global_u32x4 *>((uintptr_t)(vb + 1024 * i));
        }
        sc.k[i] = a;
        sc.v[i] = b;
    }
}

// kdst: the wavefront's 16 K rows in the stage buffer; its V rows are v_lds bytes further.
template <int D>
__device__ __forceinline__ void write_stage_codes(const StageCodes<D> &sc, char *kdst, uint32_t v_lds)
{
    constexpr int NL = D / 64, LPR = D / 16, RPL = 64 / LPR;
    const int lane = fresh_lane();
    const int c16 = lane % LPR;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
        const int r = RPL * i + lane / LPR;              // row among the wavefront's 16
        u32x4 lo, hi;
        codes_to_bf16(sc.k[i], lo, hi);
        char *row = kdst + r * (D * 2);
        *reinterpret_cast<u32x4 *>(row + (((2 * c16) ^ k_swizzle<D>(r)) << 4)) = lo;
        *reinterpret_cast<u32x4 *>(row + (((2 * c16 + 1) ^ k_swizzle<D>(r)) << 4)) = hi;
        codes_to_bf16(sc.v[i], lo, hi);
        row += v_lds;
        *reinterpret_cast<u32x4 *>(row + (((2 * c16) ^ v_swizzle<D>(r)) << 4)) = lo;
        *reinterpret_cast<u32x4 *>(row + (((2 * c16 + 1) ^ v_swizzle<D>(r)) << 4)) = hi;
    }
}

// Physical page of the 16 cached rows wavefront `wave` loads in stage `it` (unused for stages of
// new keys).  Read through the constant address space: a scalar load, off the vector-memory queue.
template <int KS>
__device__ __forceinline__ int load_stage_page(const int32_t *bt_row, int max_blocks, int it, int wave)
{
    const const_i32 *bt = (const const_i32 *)(uintptr_t)bt_row;
    return bt[min(it * (kBNW * KS / kPage) + wave, max_blocks - 1)];   // clamped entries are never used
}

// Stages of new keys of the m row tiles before tile m of a segment: the sum over i = 1..m of
// ceil(i * BM / STAGE), BM = 1 << bm_shift rows per tile.
template <int STAGE>
__device__ __forceinline__ int new_stages_before(int m, int bm_shift)
{
    constexpr int SS = STAGE == 128 ? 7 : 6;
    static_assert(STAGE == 128 || STAGE == 64, "stage of 64 or 128 keys");
    if (bm_shift >= SS) return ((m * (m + 1)) >> 1) << (bm_shift - SS);
    const int rs = SS - bm_shift, q = m >> rs, rem = m & ((1 << rs) - 1);
    return (((q * (q + 1)) >> 1) << rs) + rem * (q + 1);
}

// Fused KV append: workgroup `blk` of `nblk` copies chunk rows blk, blk + nblk, ... (K and V of
// every kv head, 16 bytes per thread and pass) into slot (ctx + t) % 16 of page
// block_table[s][(ctx + t) / 16].  Same result as the stand-alone append kernel, bit for bit.
// First every thread looks up where one of the workgroup's rows goes (table in LDS); then rows
// are copied 8 at a time with all their loads issued before the first store, so that a
// workgroup has tens of KB in flight.
// F8: the pool holds FP8 codes; a row's 16-byte vectors (8 values) are quantised on the way (8 codes, 8 bytes) under
// the tensor's scale; the pool's layout is the same with half the element size.
template <int D, bool F8>
__device__ __forceinline__ void append_rows(const AttnParams &p, unsigned long long *row_dst, int blk, int nblk, int tid, int nthreads)
{
    constexpr int CH = D / 8, R = 8;
    const int n_real = p.cu[p.S];
    const int per_row = p.Hkv * CH;                    // 16-byte vectors per row and matrix
    for (int base = blk; base < n_real; base += nblk * nthreads) {     // one pass unless the chunk has more than nblk * nthreads rows
        const int mine = base + tid * nblk;
        if (mine < n_real) {
            int lo = 0, hi = p.S - 1;                  // largest s with cu[s] <= row
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (p.cu[mid] <= mine) lo = mid; else hi = mid - 1;
            }
            const int pos = p.ctx[lo] + (mine - p.cu[lo]);
            const int page = p.bt[(size_t)lo * p.max_blocks + pos / kPage];
            // of the row's K vector 0 of head 0, in units of a vector (16 bytes; 8 bytes of codes)
            row_dst[tid] = (unsigned long long)page * 2 * p.Hkv * (kPage * CH) + (unsigned long long)(pos % kPage) * CH;
        }
        __syncthreads();
        const int rows_here = min(nthreads, (n_real - base + nblk - 1) / nblk);
        for (int r0 = 0; r0 < rows_here; r0 += R) {
            for (int x = tid; x < 2 * per_row; x += nthreads) {
                const int which = x >= per_row, y = x - which * per_row;
                const int head = y / CH, c = y - head * CH;
                const size_t in_page = ((size_t)which * p.Hkv + head) * (kPage * CH) + c;
                const u32x4 *src = reinterpret_cast<const u32x4 *>(which ? p.v_new : p.k_new) + y;
                u32x4 v[R];                            // past the last row: that row once more
#pragma unroll
                for (int r = 0; r < R; ++r) v[r] = src[(size_t)(base + min(r0 + r, rows_here - 1) * nblk) * per_row];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const size_t at = row_dst[min(r0 + r, rows_here - 1)] + in_page;
                    if constexpr (F8) reinterpret_cast<uint2 *>(p.pages_w)[at] = bf16_to_codes(v[r], which ? p.v_inv : p.k_inv);
                    else reinterpret_cast<u32x4 *>(p.pages_w)[at] = v[r];
                }
            }
        }
        __syncthreads();
    }
}

// The launch parameters as the jobs of a workgroup read them: from a copy in LDS (the kernel
// argument segment is slow to re-read, one read of it per launch is enough), word by word into
// scalar registers, anew wherever they are needed, so that they do not occupy scalar registers
// across the main loop.
__device__ __forceinline__ AttnParams read_params(const AttnParams *lds_copy)
{
    static_assert(sizeof(AttnParams) % 4 == 0, "copied as 32-bit words");
    constexpr int N = sizeof(AttnParams) / 4;
    uint32_t w[N];
    const uint32_t *src = reinterpret_cast<const uint32_t *>(lds_copy);
#pragma unroll
    for (int i = 0; i < N; ++i) w[i] = __builtin_amdgcn_readfirstlane(src[i]);
    return __builtin_bit_cast(AttnParams, w);
}

// A piece of a tile whose result is in the scratch memory but whose arrival is not settled yet:
// what a wavefront remembers of it while it goes on with the workgroup's next job (see tile_job).
struct Handover {
    int unit = -1;          // arrival counter of the (head group, tile, slot); -1: nothing pending
    bool announced = false; // what the counter held then is kept in LDS (old_stash)
    bool fresh = false;     // the partial result's stores are the wavefront's most recent memory operations
    int seg_cu = 0, t0 = 0, n_s = 0;    // where the tile's rows are
    int npieces = 0, wf = 0, tile_index = 0;
};

// Byte size of one wavefront's partial result in the scratch memory: O (32 rows x D floats in the
// accumulator layout: 16-byte vector (db * 4 + q4) of lane l at index (db * 4 + q4) * 64 + l),
// then m and the row sum of the 32 rows.
// Store instructions a wavefront issues for one partial result (16-byte vectors of O, then m and the row sum).
template <int D> constexpr int kPartialStores = (D / 32) * 4 + 2;

template <int D> constexpr size_t unit_bytes() { return (size_t)(D / 32) * 4 * 64 * 16 + 2 * 32 * 4; }

// Where piece i of a tile keeps its partial result: a workgroup has two places, one for a piece
// that is not the first of its tile (only a workgroup's first job can be one) and one for a first
// piece (only its last job can be an unfinished one).
// In tail mode (two pieces per tile, found by the tile's index) piece i of every tile has a region of its own.
template <int D>
__device__ __forceinline__ char *piece_scratch(const AttnParams &p, int grp, int wf, int tile_index, int i, int slot)
{
    const size_t unit = p.stream_wgs != 0 ? (((size_t)grp * p.stream_wgs + wf + i) * 2 + (i == 0 ? 1 : 0)) * kSlots + slot
                                          : (((size_t)i * p.groups + grp) * p.tiles + tile_index) * kSlots + slot;
    return p.scratch + unit * unit_bytes<D>();
}

// The output rows of a wavefront.  Lane (l32, half) holds for its row and every (db, q4) the four values
// d = 32 db + 8 q4 + 4 half + 0..3 (8 bytes); chunk(db, q4) returns them rounded.  The two half-waves exchange what
// they hold of two neighbouring q4 (v_permlane32_swap: the upper half of the first register with the lower half of
// the second), after which the lower half-wave has the 8 values of the even q4 and the upper one those of the odd
// q4: 16 bytes per lane and store, half as many stores as without the exchange.
template <int D, typename F>
__device__ __forceinline__ void store_out_rows(uint16_t *orow, int half, F &&chunk)
{
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4 += 2) {
            uint2 a = chunk(db, q4), b = chunk(db, q4 + 1);
            asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %2\n\tv_permlane32_swap_b32 %1, %3\n\ts_nop 1" : "+v"(a.x), "+v"(a.y), "+v"(b.x), "+v"(b.y));
            // (a store through the global address space: where the pointer comes from the parameters' copy in LDS the
            // compiler knows no address space for it, and a generic access also counts as an LDS operation)
            *reinterpret_cast<global_u32x4_w *>((uintptr_t)(orow + db * 32 + (q4 + half) * 8)) = u32x4{a.x, a.y, b.x, b.y};
        }
}

// All pieces of a tile are there: merge them, normalise, write the rows.  `mine` is the piece this
// wavefront has not written to the scratch memory: its O is in LDS at `own` (parked there so that the
// merge holds two copies of O in registers, not three), its m and row sum in (m, l); -1 when all
// pieces are read from the scratch memory.  Whoever calls this, the value is the same: the pieces are combined one after the other
// in piece order, each step bringing the running result and the next piece to their common
// reference exponent: acc = acc * 2^(m_acc - m') + O_i * 2^(m_i - m'), m' = max(m_acc, m_i).
// One pass over the scratch memory: a piece's O, m and row sum arrive in one round trip.
template <int D>
__device__ __forceinline__ void finish_tile(const AttnParams &p, int grp, int wf, int tile_index, int npieces, int mine, int slot,
                                            const f32x4 *own, float m, float l, int lane, bool row_ok, int row, int head)
{
    constexpr int DBLK = D / 32;
    constexpr size_t STATS = (size_t)DBLK * 4 * 64 * 16;
    const int half = lane >> 5, l32 = lane & 31;
    float macc = 0.f, lacc = 0.f;
    f32x16 acc[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
    for (int i = 0; i < npieces; ++i) {
        float mi, li;
        f32x4 x[DBLK * 4];
        if (i == mine) {
            mi = m; li = l;
#pragma unroll
            for (int u = 0; u < DBLK * 4; ++u) x[u] = own[u * 64 + lane];
        } else {
            const char *src = piece_scratch<D>(p, grp, wf, tile_index, i, slot);
            load_partial(reinterpret_cast<const f32x4 *>(src) + lane, reinterpret_cast<const float *>(src + STATS) + l32, x, mi, li);
        }
        if (i == 0) {
            macc = mi; lacc = li;
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[db][v] = x[db * 4 + v / 4][v % 4];
        } else {
            const float mnew = fmaxf(macc, mi);
            const float wa = __builtin_amdgcn_exp2f(macc - mnew), wi = __builtin_amdgcn_exp2f(mi - mnew);
            macc = mnew;
            lacc = __builtin_fmaf(li, wi, lacc * wa);
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[db][v] = __builtin_fmaf(x[db * 4 + v / 4][v % 4], wi, acc[db][v] * wa);
        }
    }
    if (!row_ok) return;
    const float inv = __builtin_amdgcn_rcpf(lacc);
    uint16_t *orow = p.out + ((size_t)row * p.Hq + head) * D;     // (worked out here: a pointer kept across the loop above costs two registers)
    store_out_rows<D>(orow, half, [&](int db, int q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(acc[db][q4 * 4 + e] * inv);
        return __builtin_bit_cast(uint2, w);
    });
}

// The same for a tile of two pieces, of which this wavefront holds one (`piece`) in registers: one round trip for the
// other piece, no copy of O besides the two.  Bit for bit what finish_tile computes for two pieces.
template <int D>
__device__ __forceinline__ void finish_pair(const AttnParams &p, int grp, int wf, int tile_index, int piece, int slot, f32x16 (&o)[D / 32],
                                            float m, float l, int lane, bool row_ok, int row, int head)
{
    constexpr int DBLK = D / 32;
    constexpr size_t STATS = (size_t)DBLK * 4 * 64 * 16;
    const int half = lane >> 5, l32 = lane & 31;
    const char *other = piece_scratch<D>(p, grp, wf, tile_index, 1 - piece, slot);
    float m1, l1;
    f32x4 x[DBLK * 4];
    load_partial(reinterpret_cast<const f32x4 *>(other) + lane, reinterpret_cast<const float *>(other + STATS) + l32, x, m1, l1);
    const float mnew = fmaxf(m, m1);
    const float w_own = __builtin_amdgcn_exp2f(m - mnew), w_oth = __builtin_amdgcn_exp2f(m1 - mnew);
    // piece 1 joins piece 0: fma(piece 1, its weight, piece 0 * its weight)
    l = piece == 0 ? __builtin_fmaf(l1, w_oth, l * w_own) : __builtin_fmaf(l, w_own, l1 * w_oth);
    if (!row_ok) return;
    const float inv = __builtin_amdgcn_rcpf(l);
    uint16_t *orow = p.out + ((size_t)row * p.Hq + head) * D;
    store_out_rows<D>(orow, half, [&](int db, int q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float y = o[db][q4 * 4 + e], z = x[db * 4 + q4][e];
            const float r = piece == 0 ? __builtin_fmaf(z, w_oth, y * w_own) : __builtin_fmaf(y, w_own, z * w_oth);
            w[e] = (__bf16)(r * inv);
        }
        return __builtin_bit_cast(uint2, w);
    });
}

// What carries over from one job of a workgroup to the next.
template <int D>
struct Carry {
    bf16x8 qf[D / 16];      // Q fragments of the job about to run (requested before the previous job's epilogue)
    int par;                // stage `it` of the job about to run uses stage buffer (it & 1) ^ par
    int page;               // page of this wavefront's rows of the stage after the job's first one
    StageCodes<D> codes;    // pool of FP8 codes: this wavefront's rows of the job's first stage, if those are cached keys ...
    bool have_codes;        // ... and requested, not yet in the stage buffer
};

// Q fragments (B operand of S^T = K Q^T) of a job: lane holds q[t][16*st + 8*half .. +7].  Lanes
// past the segment's last row read its first row instead: their results are never stored.
template <int D>
__device__ __forceinline__ void request_q(const AttnParams &p, const Job &J, int head, int rbk, int lane, bf16x8 (&qf)[D / 16])
{
    const int t = J.t0 + 32 * rbk + (lane & 31);
    const global_u32x4 *qp = reinterpret_cast<const global_u32x4 *>((uintptr_t)(p.q + ((size_t)(J.seg_cu + (t < J.n_s ? t : 0)) * p.Hq + head) * D));
#pragma unroll
    for (int st = 0; st < D / 16; ++st) qf[st] = __builtin_bit_cast(bf16x8, u32x4(qp[2 * st + (lane >> 5)]));
}

// One job: stages [J.it_begin, J.it_end) of one row tile of one head group.  When the stage range is
// the whole key range of the tile (J.npieces == 1) the rows are finished here; otherwise the pieces
// of the tile meet through the launch's scratch memory: each wavefront stores its unnormalised
// (O, m, row sum) and announces it on the tile's arrival counter; the one whose announcement finds
// all other pieces there merges them and writes the output rows.  Nobody waits for anybody.
// `next`: the workgroup has a job after this one, N.  On entry the loads of the job's first
// stage are in flight and cy holds its Q fragments; on exit the same holds for `next`.
template <int D, int KS, bool F8>
__device__ __forceinline__ void tile_job(const AttnParams &kernarg, bool first_job, const AttnParams *params, uint4 *smem, float (*Mstat)[2][32],
                                         uint32_t (*peek)[64], int *old_stash, int grp, int kh, const Job &J, bool next, const Job &N, Carry<D> &cy,
                                         Handover &ho)
{
    constexpr int CH = D / 8;        // 16-byte chunks per K/V row
    constexpr int KSTEPS = D / 16;   // MFMA steps over d for S^T
    constexpr int DBLK = D / 32;     // 32-row blocks of O^T
    constexpr int NKB = kBNW / 32;   // 32-key blocks of S^T per wavefront per stage
    constexpr int STAGE = kBNW * KS; // keys per stage
    constexpr int STAGE_U4 = STAGE * CH;

    // a workgroup's first job starts from the kernel arguments themselves: the copy in LDS is only
    // known to be complete after the job's first barrier
    AttnParams p = kernarg;
    if (!first_job) {
        asm volatile("" ::: "memory");               // keeps this a branch: the reads are not done speculatively
        p = read_params(params);
    }
    const WaveSrc ws = make_wave_src<D, KS, F8>(p, kh);
    // The thread id is made opaque per job: values derived from it are then computed where a job
    // needs them instead of being kept in registers across the whole job loop.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = wave % kSlots, kq = wave / kSlots;    // row/head slot, key part
    const int half = lane >> 5, l32 = lane & 31;
    const int hh = slot & (p.hpw - 1), rbk = slot >> p.hpw_shift;
    const int head = grp * p.hpw + hh;
    const JobSrc src = J.src, nsrc = N.src;           // by value: selecting between fields of two referenced jobs would keep them in memory
    const int n_it_begin = N.it_begin;
    const int L = src.L, n_s = J.n_s;
    const int it_begin = J.it_begin, n_stages = J.it_end;      // end of this piece's stage range
    const int par = __builtin_amdgcn_readfirstlane(cy.par);

    const int tw0 = J.t0 + 32 * rbk;       // first local row of this wavefront; lane l's query is local row tw0 + l % 32
    const bool wave_has_rows = tw0 < n_s;

    const int new_row_bytes = p.Hkv * D * 2;
    LaneOffsets<D> lo;
    init_lane_offsets<D>(lo, lane);
    const uint32_t smem_lds = lds_address(smem);
    constexpr uint32_t STAGE_BYTES = STAGE_U4 * 16;   // bytes of one matrix of one stage

    // The loads of the next stage are not issued by all wavefronts at once right after the barrier:
    // the load unit takes a wavefront's 8 KB in about 128 cycles and a wavefront that finds it busy
    // stalls in front of its own matrix instructions.  Each wavefront has one of four points in
    // the instruction stream between two barriers at which it issues its loads (the two wavefronts
    // of a SIMD use different ones), so that at any time most wavefronts are computing.
    StageLoads sl;
    bool pend = false;                               // the next stage's loads are described in sl, not issued
    const int load_point = __builtin_amdgcn_readfirstlane((wave + (kq != 0 ? 2 : 0)) & 3);
    int page = __builtin_amdgcn_readfirstlane(cy.page);
    // the pages of this wavefront's rows of the next job's first two stages: asked for now, needed after the loop
    int page_n0 = 0, page_n1 = 0;
    if (next) {
        page_n0 = load_stage_page<KS>(ws.bt + nsrc.bt_off, ws.max_blocks, n_it_begin, wave);
        page_n1 = load_stage_page<KS>(ws.bt + nsrc.bt_off, ws.max_blocks, n_it_begin + 1, wave);
    }

    bf16x8 qf[KSTEPS];
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) qf[st] = cy.qf[st];

    f32x16 o[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m = -1e30f;        // running row max (in units of log2: score * c)
    float lsum = 0.f;        // this lane's share of the running row sum
    // scores are multiplied by c = scale * log2(e), of either sign; a masked score is the infinity
    // that c turns into -inf
    const float c_new = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.neg ? -p.c : p.c)));
    // A pool of FP8 codes: the stage buffers hold the code values of cached keys and values, the scales are applied
    // where one multiplication serves many elements.  K: the factor on the scores of cached keys is c * k_scale
    // (scales are positive: the sign of c is that of the scale).  V: O accumulates weight * code value over the
    // cached keys and is multiplied by v_scale once, before the first block of new keys adds to it (or when the job
    // ends, if its stage range has none).  The chunk's own rows are not quantised and take no scale.
    // (c: the factor of the block whose weights are being computed; what the change to new keys needs is read from the
    // launch parameters when it happens, once per job, not kept in registers across the stages of cached keys)
    float c = c_new;
    if constexpr (F8) {
        if (J.it_begin < src.n_ctx_tiles) c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, c_new * p.k_scale)));
    }
    [[maybe_unused]] bool o_scaled = src.n_ctx_tiles == 0;
    [[maybe_unused]] StageCodes<D> cr = cy.codes;
    [[maybe_unused]] bool have_codes = F8 && cy.have_codes;
    const int blk = lane >> 4, i16 = lane & 15;

    // Fragment loads from LDS.  K: lane holds key (row) l32 of a 32-key block, d = 16*st + 8*half .. +7
    // (A operand of S^T).  V: for step j (16 keys) and d block db the lane gets keys 16j + 4*half +
    // {0..3, 8..11} of d = 32*db + l32 through two transposing reads (A operand of O^T).
    // The per-lane parts of the addresses (row inside the wavefront's 64-key part, swizzled chunk)
    // never change: they are computed once; stage buffer and block are added as one byte offset,
    // which is an instruction immediate wherever it is known at compile time.
    constexpr int BLOCK_BYTES = 32 * D * 2;            // one 32-key block of K or of V
    uint32_t kbase[KSTEPS], vbase[DBLK];
    {
        const int r = kq * kBNW + l32;
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) kbase[st] = r * D * 2 + (((2 * st + half) ^ k_swizzle<D>(r)) << 4);
        const int rv = kq * kBNW + 4 * half + (i16 >> 2);
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            const int d0 = db * 32 + 16 * (blk & 1) + 4 * (i16 & 3);
            vbase[db] = 2 * STAGE_BYTES + rv * D * 2 + (((d0 >> 3) ^ v_swizzle<D>(rv)) << 4) + ((d0 & 7) << 1);
        }
    }
    const char *smem_b = reinterpret_cast<const char *>(smem);
    // byte offset of the stage buffer that holds stage `it` of this job
    auto buf_of = [&](int it) -> int { return ((it & 1) ^ par) * (int)STAGE_BYTES; };
    // off = buffer * STAGE_BYTES + block * BLOCK_BYTES
    auto load_k = [&](bf16x8 (&kf)[KSTEPS], int off) {
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st)
            kf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(smem_b + kbase[st] + off));
    };
    auto load_v_half = [&](s16x8 (&vf)[2 * DBLK], int off, int j) {        // the fragments of PV step j
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            const char *a = smem_b + vbase[db] + off + j * (16 * D * 2);
            const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a);
            const s16x4 vb4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + 8 * D * 2));
            vf[j * DBLK + db] = __builtin_shufflevector(va, vb4, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    auto load_v = [&](s16x8 (&vf)[2 * DBLK], int off) {
        load_v_half(vf, off, 0);
        load_v_half(vf, off, 1);
    };

    // Number of 32-key blocks of stage `it` this wavefront works on (a prefix of its 64-key part):
    // those inside the key range and not entirely past the wavefront's rows.
    auto stage_blocks = [&](int it) -> int {
        if (!wave_has_rows) return 0;
        const bool is_ctx = it < src.n_ctx_tiles;
        const int part0 = (is_ctx ? it : it - src.n_ctx_tiles) * STAGE + kq * kBNW;
        int nblk = 0;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const int key0 = part0 + kb * 32;
            if (is_ctx ? key0 < L : (key0 < src.n_new && key0 <= tw0 + 31)) nblk = kb + 1;
        }
        return nblk;
    };
    // Make stage `it` the current one: its loads have landed for every wavefront, nobody reads the
    // other buffer any more, so the loads of the stage after it can go there.  `page` always belongs
    // to the stage whose loads are issued next; it is fetched one stage ahead.
    // Entering a stage has two halves: the wait, after which the wavefront may read the stage (it
    // requests its first K fragments from LDS right away), and handing out the next stage's loads.
    // `pv_before`: a PV product is pending, i.e. deferred loads will meet their issue point before
    // the next stage is entered.
    // the loads a StageLoads describes: direct loads into the stage buffer, or codes into registers
    auto issue = [&](const StageLoads &x, bool full) {
        if (F8 && x.codes) {
            fetch_stage_codes<D>(x, full, cr);
            have_codes = true;
        } else {
            issue_stage_loads<D, KS>(x, full);
        }
    };
    // codes that have arrived go to this wavefront's rows of the buffer of stage `it`, which nobody reads before the
    // barrier that follows
    auto place_codes = [&](int it) {
        if constexpr (F8) {
            if (have_codes) {
                write_stage_codes<D>(cr, reinterpret_cast<char *>(smem) + buf_of(it) + wave * (16 * D * 2), 2 * STAGE_BYTES);
                have_codes = false;
            }
        }
    };
    auto issue_pending = [&](int point) {
        if (pend && load_point == point) {
            issue(sl, true);
            pend = false;
        }
    };
    auto sync_stage = [&](int it) -> int {
        if (pend) {                                    // rare: the stage had too few blocks to reach the point
            issue(sl, true);
            pend = false;
        }
        wait_vm<0>();
        place_codes(it);
        __syncthreads();
        return stage_blocks(it);
    };
    const int32_t *bt_row = ws.bt + src.bt_off;      // the job's block-table row
    auto next_stage_loads = [&](int it, int nb, bool pv_before) {
        if (it + 1 < n_stages) {
            const bool full = describe_stage_loads<D, KS, F8>(src, ws, lo, page, it + 1, wave, new_row_bytes, smem_lds + (buf_of(it) ^ STAGE_BYTES), sl);
            if (full && pv_before && nb != 0 && load_point != 0) pend = true;
            else issue(sl, full);
        }
        page = load_stage_page<KS>(bt_row, ws.max_blocks, it + 2, wave);
    };
    auto qk = [&](const bf16x8 (&kf)[KSTEPS]) -> f32x16 {
        f32x16 sacc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st)
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st], qf[st], sacc, 0, 0, 0);
        return sacc;
    };

    // ---- main loop over this wavefront's blocks, software pipelined: while the softmax of block b
    // runs on the VALU, the matrix cores compute the scores of block b+1; then O += V_b P_b.
    // Every wavefront enters every stage exactly once (one barrier each), whether or not it has
    // blocks there.
    int it = it_begin;
    TETRI_MARK((first_job ? 0 : 12) + 2);
    int nblk;
    // A partial result left by an earlier job is announced behind a wait for all of this wavefront's memory
    // operations, its stores included.  What the counter held is looked at when the workgroup's jobs are done.
    // (called behind a wait for all memory operations: the answer to an announcement made at the previous such
    // point has arrived and is put away)
    int old = 0;            // lane 0: what the counter held when the piece was announced, until it is put away in LDS
    bool stashed = true;    // (a register kept across all jobs would be spilled to memory)
    auto announce = [&]() {
        if (!stashed) {
            if (fresh_lane() == 0) old_stash[slot] = old;
            stashed = true;
        }
        if (ho.unit >= 0 && !ho.announced) {
            if (fresh_lane() == 0) old = atomic_add_global(p.counters + ho.unit, 1);
            ho.announced = true;
            stashed = false;
        }
    };
    if (ho.unit >= 0 && ho.fresh) {
        // The job before this one left a partial result: its stores were issued after this job's first stage and
        // Q rows were requested, they are this wavefront's most recent memory operations, and they go all the way
        // to memory.  Memory operations complete in the order they were issued: the first stage waits for all but
        // those stores; the announcement follows at the job's second stage (a job of one stage: when its loop is done).
        wait_vm<kPartialStores<D>>();
        place_codes(it);
        if constexpr (F8) lds_barrier();
        else __builtin_amdgcn_s_barrier();
        nblk = stage_blocks(it);
        ho.fresh = false;
    } else {
        nblk = sync_stage(it);
        announce();
    }
    TETRI_MARK((first_job ? 0 : 12) + 3);
    // (pool of FP8 codes) O leaves the units of code values; scores take the plain factor from here on.  Called behind
    // the job's first barrier: the copy of the launch parameters in LDS is complete.
    [[maybe_unused]] auto scale_o = [&]() {
        asm volatile("" ::: "memory");
        const AttnParams pq = read_params(params);
        const float v_scale = pq.v_scale;
#pragma unroll
        for (int i = 0; i < DBLK; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[i][v] *= v_scale;
        c = pq.neg ? -pq.c : pq.c;
        o_scaled = true;
    };
    // ... before the first block of new keys
    [[maybe_unused]] auto stage_kind = [&](bool is_ctx) {
        if constexpr (F8) {
            if (!is_ctx && !o_scaled) scale_o();
        }
    };
    while (nblk == 0 && it + 1 < n_stages) {
        next_stage_loads(it, 0, false);
        nblk = sync_stage(++it);
        announce();
    }
    if (nblk != 0) {
        int kb = 0;
        bf16x8 kf[KSTEPS];
        load_k(kf, buf_of(it));
        next_stage_loads(it, nblk, false);
        // weights of a block from its scores and the row's reference exponent m: bf16-rounded, laid out
        // as the B operand of the PV product
        auto weights = [&](const f32x16 &sc, bf16x8 (&pf)[2]) {
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                pf[v / 8][v % 8] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sc[v], c, -m));
                pf[v / 8][v % 8 + 1] = (__bf16)__builtin_amdgcn_exp2f(__builtin_fmaf(sc[v + 1], c, -m));
            }
        };
        // Is one of the lane's 16 weights 2 or more (or infinite, or not a number)?  Those are the bf16 patterns with
        // the top exponent bit set; weights are not negative.
        auto weights_out_of_range = [&](const bf16x8 (&pf)[2]) -> bool {
            const u32x4 a = __builtin_bit_cast(u32x4, pf[0]), b = __builtin_bit_cast(u32x4, pf[1]);
            const uint32_t any = (a[0] | a[1] | a[2]) | (a[3] | b[0] | b[1]) | (b[2] | b[3]);
            return (any & 0x40004000u) != 0;
        };
        // This lane's sum of the rounded weights (the row sum is taken over the weights the PV product uses):
        // plain VALU additions, which go out between the matrix instructions of the PV product.
        auto weight_sum = [&](const bf16x8 &pfj) -> float {       // of the 8 weights of one PV step
            const u32x4 a = __builtin_bit_cast(u32x4, pfj);
            float lo = 0.f, hi = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                lo += __builtin_bit_cast(float, a[i] << 16);
                hi += __builtin_bit_cast(float, a[i] & 0xffff0000u);
            }
            return lo + hi;
        };
        // The second half of a block: scores of the next block (its K fragments
        // are in kf; discarded after the last block) on the matrix cores, interleaved with
        // exponentiating and rounding this block's weights on the VALU against the reference exponent
        // m the row already has; then the PV product with the V fragments in vf.
        // v_off: where in LDS the block's V fragments are, if they are still to be read (spread between the score
        // products, behind the K fragments those wait for); a negative value: vf holds them already.
        // at_point(1), at_point(2): two of the places where a wavefront may issue the next stage's loads.
        // vn_off: where the V fragments of the block after this one are, if they are to be read into vn between the
        // matrix instructions of this block's PV product.
        auto softmax_pv = [&](f32x16 &s_cur, f32x16 &s_next, s16x8 (&vf)[2 * DBLK], auto v_off, auto &&at_point, s16x8 (&vn)[2 * DBLK],
                              auto vn_off) {
            constexpr int V_OFF = decltype(v_off)::value, VN_OFF = decltype(vn_off)::value;
            bf16x8 pf[2];
            constexpr bool PHASED = KS == 1;
            if constexpr (PHASED) {
                // Four-wavefront workgroups run two to a compute unit, so the two wavefronts of a SIMD belong
                // to different workgroups and are not held in step by a common barrier.  Here the block has a
                // VALU phase (the weights) and an MFMA phase at raised wavefront priority: one wavefront's
                // matrix instructions go out back to back while the other, in its VALU phase, takes the issue
                // slots in between (measured: +7 to +13 % on launches with two workgroups per compute unit; for
                // eight-wavefront workgroups, whose SIMD partners meet at every barrier, no gain).
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (V_OFF >= 0) load_v(vf, V_OFF);
                weights(s_cur, pf);
                __builtin_amdgcn_sched_barrier(0);
                at_point(1);
                __builtin_amdgcn_s_setprio(3);
                s_next = qk(kf);
                __builtin_amdgcn_sched_barrier(0);
            } else {
                __builtin_amdgcn_sched_barrier(0);
                s_next = qk(kf);
                if constexpr (V_OFF >= 0) load_v(vf, V_OFF);
                weights(s_cur, pf);
                // wanted order: one MFMA of the score chain, then its share of the LDS reads and of the VALU
                // operations (exponentials are a class of their own), 8 times
#pragma unroll
                for (int g = 0; g < KSTEPS; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if constexpr (V_OFF >= 0) __builtin_amdgcn_sched_group_barrier(0x100, 4 * DBLK / KSTEPS, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 16 / KSTEPS, 0);
                    __builtin_amdgcn_sched_group_barrier(0x400, 16 / KSTEPS, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 8 / KSTEPS, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                // (the weights are needed here: computed in front of the branch below, inside the region the
                // order above applies to, not moved behind it)
                asm volatile("" : "+v"(pf[0]), "+v"(pf[1]));
                at_point(1);
            }
            // m is only a reference point, not the exact row maximum: any value keeps the result exact
            // as long as the weights stay in range.  Only when one of a lane's weights of this block reaches 2
            // (or overflowed: first block, or scores far above anything seen before) is m raised to
            // the true maximum, O and the row sum rescaled in place, and the weights recomputed.  The
            // two half-waves of a row take the same decision.  (In the phased order the vote sits
            // behind the score MFMAs, where its operands are long there.)
            if (__builtin_amdgcn_ballot_w64(weights_out_of_range(pf)) != 0) {
                float mx = s_cur[0] * c;
#pragma unroll
                for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s_cur[v] * c);
                mx = half_swap_max(mx);
                const float m_new = fmaxf(m, mx);
                float alpha = __builtin_amdgcn_exp2f(m - m_new);
                // the wait state a transcendental result needs before a VALU use; the compiler does not
                // insert it in front of inline assembly
                asm volatile("s_nop 1" : "+v"(alpha));
                m = m_new;
                lsum *= alpha;
#pragma unroll
                for (int i = 0; i < DBLK; ++i)
#pragma unroll
                    for (int v = 0; v < 16; ++v) asm volatile("v_mul_f32 %0, %1, %0" : "+v"(o[i][v]) : "v"(alpha));
                weights(s_cur, pf);
            }
            // O^T += V^T P^T.  Step j contracts the 16 keys held in accumulator elements 8j..8j+7.  The row sum's
            // additions are spread between the matrix instructions.
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if constexpr (!PHASED) __builtin_amdgcn_sched_barrier(0);
                float wsum = weight_sum(pf[j]);
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[j * DBLK + db]), pf[j], o[db], 0, 0, 0);
                if constexpr (VN_OFF >= 0) load_v_half(vn, VN_OFF, j);
                if constexpr (!PHASED) {
#pragma unroll
                    for (int db = 0; db < DBLK; ++db) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if constexpr (VN_OFF >= 0) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                        __builtin_amdgcn_sched_group_barrier(0x002, 18 / DBLK + 1, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                asm volatile("" : "+v"(wsum));           // computed here, between the matrix instructions, not later
                lsum += wsum;
                if (!PHASED && j == 0) at_point(2);
            }
            if constexpr (PHASED) {
                __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);
                at_point(2);
            }
        };
        // One block: scores s_cur are ready; computes s_next for the block after it.  Returns false
        // after the last block.
        auto block = [&](f32x16 &s_cur, f32x16 &s_next) -> bool {
            const bool is_ctx = it < src.n_ctx_tiles;
            stage_kind(is_ctx);
            const int key0 = (is_ctx ? it : it - src.n_ctx_tiles) * STAGE + kq * kBNW + kb * 32;
            const bool need_mask = is_ctx ? (key0 + 32 > L) : (key0 + 31 > tw0);
            // V fragments of this block: in registers before the stage may be left
            s16x8 vf[2 * DBLK];
            load_v(vf, buf_of(it) + kb * BLOCK_BYTES);
            // ---- the block after this one
            bool have_next = true, entered = false;
            if (kb + 1 < nblk) {
                ++kb;
            } else {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // V fragments are out of LDS
                kb = 0;
                nblk = 0;
                while (nblk == 0 && it + 1 < n_stages) {
                    nblk = sync_stage(++it);
                    announce();
                    if (nblk == 0) next_stage_loads(it, 0, true);
                }
                have_next = entered = nblk != 0;
            }
            if (have_next) load_k(kf, buf_of(it) + kb * BLOCK_BYTES);
            if (entered) next_stage_loads(it, nblk, true);
            else issue_pending(3);
            // ---- mask: accumulator element v is key key0 + (v/4)*8 + 4*half + v%4; keys past `bound`
            // (the end of the cached context, or the query's own position) get weight exp2(-inf) = 0
            if (need_mask) {
                const int ln = fresh_lane();
                const int bound = is_ctx ? L - 1 : tw0 + (ln & 31);       // last visible key index of this phase
                const float masked = c < 0.f ? INFINITY : -INFINITY;     // the infinity that c turns into -inf
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = key0 + (v / 4) * 8 + 4 * (ln >> 5) + (v % 4);
                    if (key > bound) s_cur[v] = masked;
                }
            }
            softmax_pv(s_cur, s_next, vf, std::integral_constant<int, -1>(), issue_pending, vf, std::integral_constant<int, -1>());
            return have_next;
        };
        // ---- steady state.  Most of a key range is whole stages in which both of the wavefront's blocks exist and
        // nothing is masked: the whole stages of cached keys and, if the cached keys end on a stage boundary, the
        // stages of new keys that lie entirely in front of the wavefront's rows.  After the job's first stages no
        // announcement is pending either.  Two such stages are one trip of a loop in which all of that is
        // known: the stage buffers alternate at compile time (LDS offsets are instruction immediates) and no block
        // asks what kind of block it is; the loads of a whole stage of cached keys are its page base plus
        // constants (any other stage's loads are described the general way).  The general blocks below take
        // over with the same state wherever one of the conditions does not hold: the diagonal, a ragged end.
        // step<B>: on entry stage `it` is in buffer B, s_a holds the scores of its first block and the loads of stage
        // it + 1 are issued; on exit the same holds for stage it + 1 in buffer 1 - B.
        const int ctx_whole = L / STAGE;                       // stages before it are whole stages of cached keys
        // (new key j is visible to local row t >= j: stage x of new keys is unmasked for rows from tw0 on if (x + 1) * STAGE <= tw0 + 1)
        const int steady_whole = min(n_stages, L % STAGE == 0 ? ctx_whole + (tw0 + 1) / STAGE : ctx_whole);
        // A step finishes stage `it` and enters stage it + 1, of which it only computes the raw scores of the first
        // block: the stage behind the last whole one may be entered that way too if the wavefront has a block there (a
        // ragged or masked stage: its loads are described the general way, its blocks are the general ones).
        const int steady_end = steady_whole + (int)(steady_whole < n_stages && stage_blocks(steady_whole) != 0);
        f32x16 s_a = qk(kf), s_b;
        auto steady_step = [&](auto buffer) {
            constexpr int cur = decltype(buffer)::value * (int)STAGE_BYTES, nxt = (int)STAGE_BYTES - cur;
            s16x8 vf[2 * DBLK], vf2[2 * DBLK];
            stage_kind(it < src.n_ctx_tiles);                    // both blocks this step finishes are of stage `it`
            load_k(kf, cur + BLOCK_BYTES);
            softmax_pv(s_a, s_b, vf, std::integral_constant<int, cur>(), [](int) {}, vf2, std::integral_constant<int, cur + BLOCK_BYTES>());
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the second block's V fragments are out of LDS: the stage may be left
            ++it;
            wait_vm<0>();
            place_codes(it);
            __syncthreads();
            load_k(kf, nxt);
            const int pg = page;                                 // of stage it + 1, which goes where stage it - 1 was
            page = load_stage_page<KS>(bt_row, ws.max_blocks, it + 2, wave);
            auto loads_at = [&](int point) {
                if (load_point == point && it + 1 < n_stages) {
                    StageLoads st;
                    if (it + 1 < ctx_whole) {
                        st.kb = ws.pool_k + (size_t)pg * ws.page_bytes;
                        st.vb = st.kb + ws.v_delta;
                        st.step = 0;
                        st.kdst = smem_lds + cur + wave * (16 * D * 2);
                        st.ko = lo.k_ctx;
                        st.vo = lo.v_ctx;
                        st.codes = F8;
                        issue(st, true);
                    } else {
                        const bool full = describe_stage_loads<D, KS, F8>(src, ws, lo, pg, it + 1, wave, new_row_bytes, smem_lds + cur, st);
                        issue(st, full);
                    }
                }
            };
            loads_at(0);
            softmax_pv(s_b, s_a, vf2, std::integral_constant<int, -1>(), loads_at, vf2, std::integral_constant<int, -1>());
            loads_at(3);
        };
        for (;;) {
            // (a step enters stage it + 1: that one has to be a steady stage)
            if (kb == 0 && nblk == NKB && buf_of(it) == 0 && it + 1 < steady_end && stashed && (ho.unit < 0 || ho.announced)) {
                if (pend) {
                    issue(sl, true);
                    pend = false;
                }
                while (it + 2 < steady_end) {
                    steady_step(std::integral_constant<int, 0>());
                    steady_step(std::integral_constant<int, 1>());
                }
                if (it + 1 < steady_end) steady_step(std::integral_constant<int, 0>());
                nblk = stage_blocks(it);                 // (fewer than all only in the stage behind the last whole one)
            }
            if (!block(s_a, s_b)) break;
            if (!block(s_b, s_a)) break;
        }
    }
    if constexpr (F8) {
        if (!o_scaled) scale_o();                      // a stage range of cached keys only: the piece leaves in true units
    }
    // ---- the next job's first stage, into the buffer the job's last stage does not use: every wavefront has left it.
    // The loads travel during this job's epilogue.
    if (next) {
        const bool full = describe_stage_loads<D, KS, F8>(nsrc, ws, lo, page_n0, n_it_begin, wave, new_row_bytes,
                                                          smem_lds + (buf_of(n_stages - 1) ^ STAGE_BYTES), sl);
        cy.have_codes = F8 && sl.codes;
        if (F8 && sl.codes) fetch_stage_codes<D>(sl, full, cy.codes);     // placed by the next job, before its first barrier
        else issue_stage_loads<D, KS>(sl, full);
    }
    if (ho.unit >= 0 && (!ho.announced || !stashed)) {        // a partial result not announced, or announced at the job's last stage
        wait_vm<0>();
        announce();
        if (!stashed) {
            wait_vm<0>();
            announce();
        }
    }

    TETRI_MARK((first_job ? 0 : 12) + 4);
    // ---- the next job: its Q rows are requested now, so that they arrive during this job's epilogue
    asm volatile("" ::: "memory");                   // a fresh read, not the values from before the loop
    const AttnParams pe = read_params(params);
    const int lane_e = fresh_lane(), half_e = lane_e >> 5, l32_e = lane_e & 31;
    const int t_e = tw0 + l32_e;                     // local row of this lane's query
    const bool row_ok_e = t_e < n_s;
    if (next) {
        request_q<D>(pe, N, head, rbk, lane_e, cy.qf);
        cy.par = ((n_stages & 1) ^ par) ^ (n_it_begin & 1);      // its first stage goes where stage n_stages of this job would
        cy.page = page_n1;
    }
    // ---- merge the KS key parts through LDS: part 1 publishes (m, row sum, O), part 0 finishes.
    // The partial O goes into a stage buffer nobody reads any more.  After a workgroup's last job that
    // is the buffer of the stage before the last one (every wavefront has entered the last stage, so no
    // barrier is needed before writing).  With a next job that buffer is receiving the next job's first
    // stage: then the last stage's own buffer is used, after a barrier that says everybody has left it.
    // The buffer's K region takes slots 0 and 1, its V region slots 2 and 3; lane l's four consecutive
    // accumulator elements are one 16-byte unit.
    const size_t unit = ((size_t)grp * pe.tiles + J.tile_index) * kSlots + slot;
    const bool pieces = J.npieces > 1;
    // A tile of several pieces and no job after it: are the other pieces there already?  The answer
    // travels while the key parts merge.
    if (pieces && !next && kq == 0 && wave_has_rows) peek_coherent(pe.counters + unit, lds_address(peek[slot]));
    float ltot = half_swap_sum(lsum);
    // where this wavefront may keep one O (16-byte vector u of lane l at index u * 64 + l): the place of its key-part
    // partner's partial result, or, with one key part, a quarter of the stage buffers
    f32x4 *part = reinterpret_cast<f32x4 *>(smem) + slot * (DBLK * 4 * 64);
    if constexpr (KS == 2) {
        static_assert(2 * (DBLK * 16 * 64 * 4) == STAGE_BYTES, "two slots per matrix region");
        if (next) lds_barrier();
        TETRI_MARK((first_job ? 0 : 12) + 10);
        const int dead_off = next ? buf_of(n_stages - 1) : (buf_of(n_stages - 1) ^ (int)STAGE_BYTES);
        char *dead = reinterpret_cast<char *>(smem) + dead_off + (slot >> 1) * (2 * STAGE_BYTES);
        part = reinterpret_cast<f32x4 *>(dead + (slot & 1) * (DBLK * 16 * 64 * 4));
        if (kq == 1) {
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = o[db][q4 * 4 + e];
                    part[(db * 4 + q4) * 64 + lane_e] = x;
                }
            if (half_e == 0) { Mstat[slot][0][l32_e] = m; Mstat[slot][1][l32_e] = ltot; }
        }
        lds_barrier();
        TETRI_MARK((first_job ? 0 : 12) + 5);
        if (kq == 1) return;
        const float m1 = Mstat[slot][0][l32_e], l1 = Mstat[slot][1][l32_e];
        const float mstar = fmaxf(m, m1);
        const float w0 = __builtin_amdgcn_exp2f(m - mstar), w1 = __builtin_amdgcn_exp2f(m1 - mstar);
        ltot = ltot * w0 + l1 * w1;
        m = mstar;
        if (!wave_has_rows) return;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 x = part[(db * 4 + q4) * 64 + lane_e];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[db][q4 * 4 + e] = o[db][q4 * 4 + e] * w0 + x[e] * w1;
            }
    } else {
        static_assert(kSlots * (DBLK * 4 * 64 * 16) <= 4 * STAGE_BYTES, "an O per wavefront fits the stage buffers");
        // a tile finished here from several pieces parks O in the stage buffers: every wavefront has left them
        if (pieces && !next) lds_barrier();
        if (!wave_has_rows) return;
    }

    TETRI_MARK((first_job ? 0 : 12) + 11);
    // ---- a tile of several pieces.  unit = (head group, tile, slot); its counter starts at 0.
    if (pieces) {
        bool all_there = false;
        if (!next) {
            wait_vm<0>();
            all_there = __builtin_amdgcn_readfirstlane(peek[slot][lane_e]) == J.npieces - 1;
        }
        if (!all_there) {
            // leave (O, m, row sum) in the scratch memory ...
            char *mine = piece_scratch<D>(pe, grp, J.wf, J.tile_index, J.piece, slot);
            f32x4 *po = reinterpret_cast<f32x4 *>(mine);
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = o[db][q4 * 4 + e];
                    store_coherent(po + (db * 4 + q4) * 64 + lane_e, x);
                }
            float *ps = reinterpret_cast<float *>(mine + (size_t)DBLK * 4 * 64 * 16);
            if (half_e == 0) { store_coherent(ps + l32_e, m); store_coherent(ps + 32 + l32_e, ltot); }
            if (next) {
                // ... and go on with the next job: neither the end of the stores nor the answer of the
                // arrival counter is waited for here (about 4 us); the piece is announced after the next
                // job's first barrier and the answer looked at when the workgroup's jobs are done
                ho.unit = (int)unit;
                ho.announced = false;
                ho.fresh = true;
                ho.seg_cu = J.seg_cu; ho.t0 = J.t0; ho.n_s = n_s;
                ho.npieces = J.npieces; ho.wf = J.wf; ho.tile_index = J.tile_index;
                TETRI_MARK((first_job ? 0 : 12) + 6);
                return;
            }
            coherent_stores_done();                  // this wavefront's partial is in memory ...
            int arrived = 0;
            if (lane_e == 0) arrived = atomic_add_global(pe.counters + unit, 1);     // ... before it is announced
            arrived = __builtin_amdgcn_readfirstlane(arrived);
            if (arrived != J.npieces - 1) {          // not the last one: whoever is finishes the tile
                TETRI_MARK((first_job ? 0 : 12) + 6);
                return;
            }
        }
        // This wavefront is the last of the tile's pieces to arrive: nobody touches the unit's counter any more in this
        // launch.  It goes back to zero here, so that a launch leaves the counters it used clean whatever runs on
        // the handle next (the replay of a captured graph uses the counter set it was captured with).
        if (lane_e == 0) store_global(pe.counters + unit, 0);
        if (J.npieces == 2) {
            finish_pair<D>(pe, grp, J.wf, J.tile_index, J.piece, slot, o, m, ltot, lane_e, row_ok_e, J.seg_cu + t_e, head);
        } else {
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = o[db][q4 * 4 + e];
                    part[(db * 4 + q4) * 64 + lane_e] = x;
                }
            finish_tile<D>(pe, grp, J.wf, J.tile_index, J.npieces, J.piece, slot, part, m, ltot, lane_e, row_ok_e, J.seg_cu + t_e, head);
        }
        TETRI_MARK((first_job ? 0 : 12) + 6);
        return;
    }

    // ---- normalise and store: lane holds out[t][head][db*32 + (v/4)*8 + 4*half + v%4]
    if (!row_ok_e) return;
    const float inv = __builtin_amdgcn_rcpf(ltot);
    uint16_t *orow = pe.out + ((size_t)(J.seg_cu + t_e) * pe.Hq + head) * D;
    store_out_rows<D>(orow, half_e, [&](int db, int q4) {
        bf16x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][q4 * 4 + e] * inv);
        return __builtin_bit_cast(uint2, w);
    });
    TETRI_MARK((first_job ? 0 : 12) + 6);
}

// Everything about one segment a job needs, as wave-uniform values.
struct SegInfo {
    int s, seg_cu, n_s, L;
};

template <int D, int KS>
__device__ __forceinline__ JobSrc make_src(const AttnParams &p, int kh, const SegInfo &g, int t0)
{
    constexpr int STAGE = kBNW * KS;
    JobSrc src;
    src.bt_off = g.s * p.max_blocks;
    src.new_off = (uint32_t)((g.seg_cu * p.Hkv + kh) * (D * 2));
    src.L = g.L;
    src.n_new = min(g.n_s, t0 + (32 << p.rb_shift));
    src.n_ctx_tiles = (g.L + STAGE - 1) / STAGE;
    return src;
}

// Padding rows [cu[S], C) of this head group's heads, written as +0: row first, first + stride, ...
template <int D>
__device__ __forceinline__ void zero_padding_rows(const AttnParams &p, int grp, int first, int stride, int tid, int nthreads)
{
    constexpr int CH = D / 8;
    const int per_row = p.hpw * CH;                    // 16-byte vectors per row of this head group: a power of two <= 64
    const int rows_per_pass = nthreads / per_row;
    const int x = tid % per_row, rr = tid / per_row;
    for (int r = p.cu[p.S] + first + rr * stride; r < p.C; r += rows_per_pass * stride) {
        uint4 *o = reinterpret_cast<uint4 *>(p.out + ((size_t)r * p.Hq + (size_t)grp * p.hpw) * D);
        o[x] = make_uint4(0, 0, 0, 0);
    }
}

template <int D, int KS, bool F8>
__global__ __launch_bounds__(kSlots * KS * 64, 2) void attn_tile_kernel(AttnParams p)
{
    constexpr int STAGE = kBNW * KS;
    constexpr int STAGE_U4 = STAGE * (D / 8);
    constexpr int NT = kSlots * KS * 64;
    __shared__ uint4 smem[4 * STAGE_U4];             // K and V of two stage buffers: K0 | K1 | V0 | V1
    __shared__ float Mstat[kSlots][2][32];
    __shared__ uint32_t peek[kSlots][64];            // where a look at a tile's arrival counter lands
    __shared__ int old_stash[kSlots];                // what a wavefront's announcement of an earlier job's piece found
    __shared__ int4 seg_tab[64];                     // stream mode: (first row, rows, cached tokens) of every segment
    __shared__ AttnParams params;
    TETRI_MARK(0);

    // ---- fused KV append: append_blocks workgroups copy the chunk's new K/V rows into their page
    // slots.  They come after the attention workgroups, on the compute units those leave idle.
    int abid = blockIdx.x;                           // index in the attention grid
    if (abid >= p.attn_first) {
        if (abid < p.attn_first + p.append_blocks) {
            append_rows<D, F8>(p, reinterpret_cast<unsigned long long *>(smem), abid - p.attn_first, p.append_blocks, threadIdx.x, NT);
            return;
        }
        abid -= p.append_blocks;
    }
    // ---- workgroup id -> (head group, index inside the group).  The workgroups of a head group run
    // on one XCD (they read the same K and V through its L2); an XCD has gpx groups and starts their
    // workgroups index by index.
    const int xcd = abid % kXcd, local = abid / kXcd;
    const int widx = magic_div(local, p.gpx_magic);
    const int grp = xcd * p.gpx + (local - widx * p.gpx);
    const int G = p.stream_wgs;
    // the arrival counters of the next launch that divides tiles: all zero when this launch ends
    if (G != 0 || p.helpers != 0)
        for (int i = abid * NT + threadIdx.x; i < p.n_counters; i += p.attn_grid * NT) p.counters_next[i] = 0;
    if (grp >= p.groups || widx >= (G != 0 ? G : (p.helpers != 0 ? p.tiles + p.helpers - 2 : p.tiles))) return;
    if (threadIdx.x == 0) params = p;                // from scalar registers: no memory read to wait for

    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = wave % kSlots, kq = wave / kSlots;
    const int bm_shift = 5 + p.rb_shift, BM = 1 << bm_shift;
    const int S = p.S;
    const int kh = magic_div(grp, p.kv_magic);
    const int first_page = min(wave, p.max_blocks - 1), first_page_hi = min(wave + kSlots, p.max_blocks - 1);

    const WaveSrc ws = make_wave_src<D, KS, F8>(p, kh);    // for the first job's first loads; every job derives its own

    // ---- the workgroup's first job.  Lane l looks at segment s0 + l (64 at a time); it also fetches
    // what the owner of the job will need next (context length, the pages of the segment's first
    // stage), so that the kernel's first loads of K and V are one memory round trip away from its
    // start wherever possible.
    Job J;
    SegInfo seg = {-1, 0, 0, 0};
    int page = 0, page_hi = 0;
    // stream mode: the range of stages of this workgroup, [pos, b1) in the group's tile order, of W
    // stages shared by Gp workgroups; the tile the next job is in: tile j of nt in its segment,
    // starting at position tile_lin
    int pos = 0, b1 = 0, W = 1, Gp = 1, j = 0, nt = 1, tile_lin = 0, tile_index = 0;
    // stream mode, one segment whose block-table row fits two registers per lane: the whole row is fetched together
    // with the segment lengths, so that the pages of the workgroup's first stage, wherever its range starts, do not
    // cost a second round trip to memory
    const bool row_in_lanes = G != 0 && S == 1 && p.max_blocks <= 128;
    int bt_lo = 0, bt_hi = 0;
    // tile and tail modes: the workgroup's second tile (a helper's, or the bound's last tile), as found by the lookup;
    // its job is made when its turn comes
    SegInfo lg0 = {-1, 0, 0, 0};
    int lw0 = -1, lt0 = -1, n_later = 0, tail_piece = 0;
    bool later_whole = false;                        // the second tile is done whole, whatever its length
    int first_want = -1, first_t0 = -1;              // the first one (its segment is in `seg`)
    bool pages_fetched = true;                       // page / page_hi are those of the first job's stage 0
    if (G == 0) {
        // Tile mode: row tile T - 1 - widx, late (long) tiles first.  Tail mode (helpers != 0): first the owners
        // of the tiles but the last one of the host's bound (which is real only in chunks with ragged segments),
        // each doing its tile's key range but for the tail, then the helpers, each doing the tails of two of
        // those tiles.  The bound's last tile gets no workgroup of its own (it would start when the first compute
        // unit becomes free and, though empty, end after everybody else): it is one more job, done whole, of
        // the owner of tile 0, whose key range is the shortest.  Tiles never span two segments.
        const int T = p.tiles, H = p.helpers;
        int want0, want1 = -1;
        int &piece = tail_piece;
        if (H == 0) {
            want0 = T - 1 - widx;
        } else if (widx < T - 1) {
            want0 = T - 2 - widx;
            if (want0 == 0) { want1 = T - 1; later_whole = true; }
        } else {
            piece = 1;
            want0 = T - 2 - 2 * (widx - (T - 1));
            if (want0 >= 1) want1 = want0 - 1;
        }
        // one pass over the segments finds both
        SegInfo g0 = {-1, 0, 0, 0}, g1 = g0;
        int t00 = -1, t01 = -1, base = 0;
        for (int s0 = 0; s0 < S; s0 += 64) {
            const int idx = s0 + lane;
            const int a = idx < S ? p.cu[idx] : 0, b = idx < S ? p.cu[idx + 1] : 0;
            const int ctx_len = idx < S ? p.ctx[idx] : 0;
            const int pg = idx < S ? p.bt[(size_t)idx * p.max_blocks + first_page] : 0;
            const int pg_hi = idx < S ? p.bt[(size_t)idx * p.max_blocks + first_page_hi] : 0;
            const int ntl = (b - a + BM - 1) >> bm_shift;          // 0 for lanes past the last segment
            int incl = ntl;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int y = __shfl_up(incl, d, 64);
                if (lane >= d) incl += y;
            }
            auto find = [&](int want, SegInfo &g, int &t0, bool pages) __attribute__((always_inline)) {
                const int rel = want - base;
                const unsigned long long owner = __builtin_amdgcn_ballot_w64(t0 < 0 && want >= 0 && rel >= incl - ntl && rel < incl);
                if (owner != 0) {
                    const int o = __builtin_ctzll(owner);
                    g.s = s0 + o;
                    t0 = (rel - __builtin_amdgcn_readlane(incl - ntl, o)) * BM;
                    g.seg_cu = __builtin_amdgcn_readlane(a, o);
                    g.n_s = __builtin_amdgcn_readlane(b - a, o);
                    g.L = __builtin_amdgcn_readlane(ctx_len, o);
                    if (pages) {
                        page = __builtin_amdgcn_readlane(pg, o);
                        page_hi = __builtin_amdgcn_readlane(pg_hi, o);
                    }
                }
            };
            find(want0, g0, t00, true);
            if (want1 >= 0) find(want1, g1, t01, false);
            base += __builtin_amdgcn_readlane(incl, 63);
        }
        TETRI_MARK(8);
        // a wanted tile past the last segment's tiles: the padding rows [cu[S], C), one 32-row block per wavefront slot
        auto pad_tile = [&](int want, int t0) __attribute__((always_inline)) {
            if (want >= 0 && t0 < 0 && piece == 0 && kq == 0) {
                const int hh = slot & (p.hpw - 1), rbk = slot >> p.hpw_shift;
                const int r = p.cu[S] + (want - base) * BM + 32 * rbk + (lane & 31);
                if (r < p.C) {
                    uint4 *o = reinterpret_cast<uint4 *>(p.out + ((size_t)r * p.Hq + grp * p.hpw + hh) * D);
                    for (int c = lane >> 5; c < D / 8; c += 2) o[c] = make_uint4(0, 0, 0, 0);
                }
            }
        };
        pad_tile(want0, t00);
        if (want1 >= 0) pad_tile(want1, t01);
        auto tail_ok = [&](int want, const SegInfo &g, int t0) __attribute__((always_inline)) -> bool {
            // whether this workgroup has a job on that tile: it exists, and a helper's tile hands a tail over
            if (want < 0 || t0 < 0) return false;
            if (piece == 0) return true;
            const int n_new = min(g.n_s, t0 + BM);
            const int n_all = (g.L + STAGE - 1) / STAGE + (n_new + STAGE - 1) / STAGE;
            return n_all >= p.split_min && ((max(n_all - p.split_bias, 0) * p.tail_q8 + 128) >> 8) != 0;
        };
        const bool v0 = tail_ok(want0, g0, t00), v1 = want1 >= 0 && tail_ok(want1, g1, t01);
        if (!v0 && !v1) return;
        // the first valid one becomes J, a second one waits as (tile, segment, first row)
        pages_fetched = v0;
        seg.s = v0 ? g0.s : g1.s;
        seg.seg_cu = v0 ? g0.seg_cu : g1.seg_cu;
        seg.n_s = v0 ? g0.n_s : g1.n_s;
        seg.L = v0 ? g0.L : g1.L;
        first_want = v0 ? want0 : want1;
        first_t0 = v0 ? t00 : t01;
        n_later = (int)(v0 && v1);
        lg0 = g1; lw0 = want1; lt0 = t01;
    }
    // The piece of a tile this workgroup does in tile and tail mode: all of it, or with a tail handed over (key ranges
    // of at least split_min stages) everything but the tail / the tail.  A helper has about split_bias stages' worth of
    // extra work (a second tile's prologue, handing its first result over): owners and helpers finish together when
    // each tile hands over the share tail_q8 / 256 of what exceeds that.
    // (pp: the launch parameters, from the kernel arguments for a workgroup's first jobs, from their copy in LDS later:
    // kept in scalar registers across the jobs they would push other values out to memory)
    auto make_piece = [&](const AttnParams &pp, int want, const SegInfo &g, int t0, bool whole, Job &X) __attribute__((always_inline)) {
        const int H = whole ? 0 : pp.helpers, piece = tail_piece;
        {
            X.seg_cu = g.seg_cu; X.n_s = g.n_s; X.t0 = t0; X.tile_index = want;
            X.src = make_src<D, KS>(pp, kh, g, t0);
            const int n_all = X.src.n_ctx_tiles + (X.src.n_new + STAGE - 1) / STAGE;
            const int n_tail = (H != 0 && n_all >= pp.split_min) ? (max(n_all - pp.split_bias, 0) * pp.tail_q8 + 128) >> 8 : 0;
            X.it_begin = piece == 0 ? 0 : n_all - n_tail;
            X.it_end = piece == 0 ? n_all - n_tail : n_all;
            X.piece = piece; X.npieces = n_tail != 0 ? 2 : 1; X.wf = 0;
        }
    };
    if (G == 0) {
        make_piece(p, first_want, seg, first_t0, false, J);
    } else {
        // stream mode (S <= 64): every workgroup of the group works out the same division
        const int a = lane < S ? p.cu[lane] : 0, b = lane < S ? p.cu[lane + 1] : 0;
        const int ctx_len = lane < S ? p.ctx[lane] : 0;
        const int pg = lane < S ? p.bt[(size_t)lane * p.max_blocks + first_page] : 0;
        const int pg_hi = lane < S ? p.bt[(size_t)lane * p.max_blocks + first_page_hi] : 0;
        if (row_in_lanes) {
            bt_lo = p.bt[min(lane, p.max_blocks - 1)];
            bt_hi = p.bt[min(lane + 64, p.max_blocks - 1)];
        }
        const int n = b - a;
        const int ntl = (n + BM - 1) >> bm_shift;                  // 0 for lanes past the last segment
        const int csl = (ctx_len + STAGE - 1) / STAGE;
        const int wk = ntl > 0 ? ntl * csl + new_stages_before<STAGE>(ntl - 1, bm_shift) + (n + STAGE - 1) / STAGE : 0;
        if (lane < S) seg_tab[lane] = make_int4(a, n, ctx_len, 0);  // every wavefront writes the same values
        int t_incl = ntl, w_incl = wk;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(t_incl, d, 64), z = __shfl_up(w_incl, d, 64);
            if (lane >= d) { t_incl += y; w_incl += z; }
        }
        W = __builtin_amdgcn_readlane(w_incl, 63);
        TETRI_MARK(8);
        // the padding rows, shared by the G workgroups of the group
        zero_padding_rows<D>(p, grp, widx, G, tid, NT);
        Gp = min(G, W);
        if (widx >= Gp) return;
        // (the divisions run on the vector unit: their results are marked as the wave-uniform values they are)
        // and the host has checked that no product below reaches 2^31)
        pos = __builtin_amdgcn_readfirstlane((int)((uint32_t)(widx * W) / (uint32_t)Gp));
        b1 = __builtin_amdgcn_readfirstlane((int)((uint32_t)((widx + 1) * W) / (uint32_t)Gp));
        const unsigned long long owner = __builtin_amdgcn_ballot_w64(pos >= w_incl - wk && pos < w_incl);
        if (owner == 0) return;                      // cannot happen for well-formed metadata
        const int o = __builtin_ctzll(owner);
        seg.s = o;
        seg.seg_cu = __builtin_amdgcn_readlane(a, o);
        seg.n_s = __builtin_amdgcn_readlane(n, o);
        seg.L = __builtin_amdgcn_readlane(ctx_len, o);
        nt = __builtin_amdgcn_readlane(ntl, o);
        const int cs = __builtin_amdgcn_readlane(csl, o);
        page = __builtin_amdgcn_readlane(pg, o);
        page_hi = __builtin_amdgcn_readlane(pg_hi, o);
        const int seg_lin = __builtin_amdgcn_readlane(w_incl - wk, o);
        const int x = pos - seg_lin;
        // the tile of the segment position x falls into: the last one that starts at or before x
        j = 0;
        for (int j0 = 0; j0 < nt; j0 += 64) {
            const int cand = j0 + lane;
            const bool ok = cand < nt && cand * cs + new_stages_before<STAGE>(cand, bm_shift) <= x;
            const int cnt = __builtin_popcountll(__builtin_amdgcn_ballot_w64(ok));
            if (cnt == 0) break;
            j = j0 + cnt - 1;
            if (cnt < 64) break;
        }
        tile_lin = seg_lin + j * cs + new_stages_before<STAGE>(j, bm_shift);
        tile_index = __builtin_amdgcn_readlane(t_incl - ntl, o) + j;
    }

    // a job of stream mode from the cursor (seg, j, tile_lin, tile_index, pos); moves the cursor behind it
    auto stream_job = [&](const AttnParams &pp, Job &X) __attribute__((always_inline)) {
        X.seg_cu = seg.seg_cu; X.n_s = seg.n_s; X.t0 = j << bm_shift; X.tile_index = tile_index;
        X.src = make_src<D, KS>(pp, kh, seg, X.t0);
        const int n_all = X.src.n_ctx_tiles + (X.src.n_new + STAGE - 1) / STAGE;
        const int tile_end = tile_lin + n_all;
        X.it_begin = pos - tile_lin;
        X.it_end = min(b1, tile_end) - tile_lin;
        X.wf = __builtin_amdgcn_readfirstlane((int)((uint32_t)((tile_lin + 1) * Gp - 1) / (uint32_t)W));
        const int wl = __builtin_amdgcn_readfirstlane((int)((uint32_t)(tile_end * Gp - 1) / (uint32_t)W));
        X.npieces = wl - X.wf + 1;
        X.piece = widx - X.wf;
        pos = tile_lin + X.it_end;
        if (pos == tile_end) {
            tile_lin = tile_end;
            ++tile_index;
            if (++j >= nt) {
                j = 0;
                if (seg.s + 1 < S) {
                    const int4 e = seg_tab[seg.s + 1];
                    ++seg.s;
                    seg.seg_cu = __builtin_amdgcn_readfirstlane(e.x);
                    seg.n_s = __builtin_amdgcn_readfirstlane(e.y);
                    seg.L = __builtin_amdgcn_readfirstlane(e.z);
                    nt = (seg.n_s + BM - 1) >> bm_shift;
                }
            }
        }
    };
    if (G != 0) stream_job(p, J);
    TETRI_MARK(9);

    // ---- the first job's first stage and its Q rows.  The wavefronts of key part 0 reach this point
    // first (the older wavefront of a SIMD is served first), so they issue the loads of their partner
    // in part 1 as well.
    static_assert(kBNW * KS / kPage == kSlots * KS, "stage 0: wavefront w loads page w of the segment");
    Carry<D> cy;
    cy.par = J.it_begin & 1;                         // the first stage goes to buffer 0
    {
        const int new_row_bytes = p.Hkv * D * 2;
        LaneOffsets<D> lo;
        init_lane_offsets<D>(lo, lane);
        // entry e of the job's block-table row (clamped entries are never used)
        auto row_entry = [&](int e) -> int {
            e = min(e, p.max_blocks - 1);
            if (row_in_lanes) return e < 64 ? __builtin_amdgcn_readlane(bt_lo, e) : __builtin_amdgcn_readlane(bt_hi, e - 64);
            return ((const const_i32 *)(uintptr_t)(p.bt + J.src.bt_off))[e];
        };
        constexpr int PPS = kBNW * KS / kPage;           // pages per stage
        cy.have_codes = false;
        if (F8 && J.it_begin < J.src.n_ctx_tiles) {
            // a pool of FP8 codes and a first stage of cached keys: every wavefront requests the codes of its own rows
            if (J.it_begin != 0 || !pages_fetched) page = row_entry(J.it_begin * PPS + wave);
            StageLoads sl;
            const bool full = describe_stage_loads<D, KS, F8>(J.src, ws, lo, page, J.it_begin, wave, new_row_bytes, lds_address(smem), sl);
            fetch_stage_codes<D>(sl, full, cy.codes);
            cy.have_codes = true;
        } else if (kq == 0) {
            if (J.it_begin != 0 || !pages_fetched) {     // the lookup fetched the pages of stage 0 of its first tile
                page = row_entry(J.it_begin * PPS + wave);
                page_hi = row_entry(J.it_begin * PPS + wave + kSlots);
            }
            StageLoads sl;
#pragma unroll
            for (int part = 0; part < KS; ++part) {
                const bool full = describe_stage_loads<D, KS>(J.src, ws, lo, part == 0 ? page : page_hi, J.it_begin, wave + part * kSlots,
                                                              new_row_bytes, lds_address(smem), sl);
                issue_stage_loads<D, KS>(sl, full);
            }
        }
        cy.page = row_entry((J.it_begin + 1) * PPS + wave);
        const int hh = slot & (p.hpw - 1), rbk = slot >> p.hpw_shift;
        request_q<D>(p, J, grp * p.hpw + hh, rbk, lane, cy.qf);
    }
    TETRI_MARK(1);

    Handover ho;
    int guard = p.tiles + 2;                         // a workgroup never has more jobs than the chunk has tiles: malformed metadata cannot keep it here
    for (bool first = true;; first = false) {
        const bool more = G != 0 ? (pos < b1 && --guard > 0) : n_later > 0;
        Job N = J;
        if (more) {
            AttnParams pj = p;                       // before the first job's first barrier the copy in LDS may be incomplete
            if (!first) {
                asm volatile("" ::: "memory");
                pj = read_params(&params);
            }
            if (G != 0) {
                stream_job(pj, N);
            } else {
                make_piece(pj, lw0, lg0, lt0, later_whole, N);
                --n_later;
            }
        }
        tile_job<D, KS, F8>(p, first, &params, smem, Mstat, peek, old_stash, grp, kh, J, more, N, cy, ho);
        if (!more) break;
        J = N;
    }
    // ---- a piece whose hand-over was left open: if it was the last of its tile to arrive, this
    // wavefront finishes the tile from the partial results in the scratch memory (its own included).
    if (ho.unit >= 0) {
        constexpr int DBLK = D / 32;
        asm volatile("" ::: "memory");
        const AttnParams pd = read_params(&params);
        // (derived anew from the thread id: kept from the start of the kernel they would occupy registers across all jobs)
        int tid_end = threadIdx.x;
        asm volatile("" : "+v"(tid_end));
        const int lane = tid_end & 63, slot = __builtin_amdgcn_readfirstlane(tid_end >> 6) % kSlots;
        if (__builtin_amdgcn_readfirstlane(old_stash[slot]) == ho.npieces - 1) {
            const int head = grp * pd.hpw + (slot & (pd.hpw - 1));
            const int t = ho.t0 + 32 * (slot >> pd.hpw_shift) + (lane & 31);
            if (lane == 0) store_global(pd.counters + ho.unit, 0);      // (the last to arrive: see tile_job)
            finish_tile<D>(pd, grp, ho.wf, ho.tile_index, ho.npieces, -1, slot, nullptr, 0.f, 0.f, lane, t < ho.n_s, ho.seg_cu + t, head);
        }
    }
    TETRI_MARK(7);
}

template <int D, int KS, bool F8>
hipError_t launch(const AttnParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL((attn_tile_kernel<D, KS, F8>), dim3(p.attn_grid + p.append_blocks), dim3(kSlots * KS * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t tetri_launch_attn(const tetri_ctx *h, const AttnParams &p, int key_parts, bool fp8_pool, hipStream_t stream)
{
    if (fp8_pool) {
        if (h->cfg.head_dim == 128)
            return key_parts == 2 ? launch<128, 2, true>(p, stream) : launch<128, 1, true>(p, stream);
        return key_parts == 2 ? launch<64, 2, true>(p, stream) : launch<64, 1, true>(p, stream);
    }
    if (h->cfg.head_dim == 128)
        return key_parts == 2 ? launch<128, 2, false>(p, stream) : launch<128, 1, false>(p, stream);
    return key_parts == 2 ? launch<64, 2, false>(p, stream) : launch<64, 1, false>(p, stream);
}
