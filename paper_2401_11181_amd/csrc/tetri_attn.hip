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
//   * Workgroup ids are remapped so that all row tiles of a kv head run on one XCD (one L2).
//   * A launch with fewer row tiles than two thirds of the CUs adds helper workgroups: a tile
//     with a long key range hands its last stages to a helper (two tiles per helper) and the two
//     partial results meet in scratch memory of the library's handle, without anybody waiting
//     (tile_job, merge_pieces_and_store).
//   * The fused form of the launch has further workgroups that copy the chunk's new K/V rows
//     into the page pool (append_rows).
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
    uint32_t k_new, v_new;      // rows Hkv*D*2 bytes apart in k_new / v_new
};

template <int D>
__device__ __forceinline__ void init_lane_offsets(LaneOffsets<D> &lo, int lane, int new_row_bytes)
{
    constexpr int CH = D / 8;
    const int r0 = lane / CH;                                    // row of instruction 0
    const int kc = (lane % CH) ^ k_swizzle<D>(r0);
    const int vc = (lane % CH) ^ v_swizzle<D>(r0);
    lo.k_ctx = r0 * D * 2 + kc * 16;
    lo.v_ctx = r0 * D * 2 + vc * 16;
    lo.k_new = r0 * new_row_bytes + kc * 16;
    lo.v_new = r0 * new_row_bytes + vc * 16;
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

// Wave-uniform pieces of a wavefront's load addresses, fixed for the whole kernel.
struct WaveSrc {
    const char *pool_k;         // K block of kv head kh in page 0 of the pool
    uint32_t page_bytes;        // one page: K and V blocks of every kv head
    uint32_t v_delta;           // from a page's K block to its V block of the same head
    const char *new_k, *new_v;  // first row of the segment, kv head kh, in k_new / v_new
    uint32_t stage_new_bytes;   // a stage's worth of rows in k_new / v_new
    uint32_t wave_new_bytes;    // a wavefront's 16 rows
};

// The direct-to-LDS loads of this wavefront's 16 rows of one stage (K and V): one scalar base per
// matrix; the NI instructions of a matrix differ only in their per-lane offsets.
struct StageLoads {
    const char *kb, *vb;        // row j0 of the stage part, K and V
    uint32_t step;              // bytes the rows of two instructions are further apart than 1 KB
    uint32_t kdst;              // LDS byte address of the K rows; the V rows are 2 * STAGE_BYTES further
    int j0, limit;              // first key row, and the end of the key range it belongs to
    bool ctx;                   // pool rows (else rows of k_new / v_new)
    uint32_t ko, vo;            // per-lane byte offsets of the first instruction's rows, K and V
};

// Where stage `it` comes from.  Returns whether all 16 rows exist.
template <int D, int KS>
__device__ __forceinline__ bool describe_stage_loads(const KeySource &ks, const WaveSrc &ws, const LaneOffsets<D> &lo, int page, int it,
                                                     int wave, int new_row_bytes, uint32_t k_lds, StageLoads &sl)
{
    constexpr int RPI = 64 / (D / 8);
    constexpr int STAGE = kBNW * KS;
    sl.ctx = it < ks.n_ctx_tiles;
    const int jn = it - ks.n_ctx_tiles;
    sl.j0 = (sl.ctx ? it : jn) * STAGE + 16 * wave;
    sl.limit = sl.ctx ? ks.L : ks.n_new;
    sl.kdst = k_lds + wave * (16 * D * 2);
    sl.ko = sl.ctx ? lo.k_ctx : lo.k_new;
    sl.vo = sl.ctx ? lo.v_ctx : lo.v_new;
    // pool rows of an instruction follow the previous one's directly (the immediate offset covers
    // it); rows of k_new / v_new are `step` bytes further apart than that
    if (sl.ctx) {
        sl.kb = ws.pool_k + (size_t)page * ws.page_bytes;
        sl.vb = sl.kb + ws.v_delta;
        sl.step = 0;
    } else {
        const size_t off = (size_t)jn * ws.stage_new_bytes + (size_t)wave * ws.wave_new_bytes;
        sl.kb = ws.new_k + off;
        sl.vb = ws.new_v + off;
        sl.step = RPI * new_row_bytes - 1024;
    }
    return sl.j0 + 16 <= sl.limit;
}

// All loads of a stage at once.
template <int D, int KS>
__device__ __forceinline__ void issue_stage_loads(const StageLoads &sl, bool full, int lane)
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
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const bool ok = sl.j0 + RPI * i + lane / CH < sl.limit;
            const size_t inst = (size_t)i * (step + 1024);
            dma16(ok ? sl.kb + inst + (ko ^ k_inst_xor<D>(i)) : zero, kdst + 1024 * i);
            dma16(ok ? sl.vb + inst + (vo ^ v_inst_xor<D>(i)) : zero, vdst + 1024 * i);
        }
    }
}

template <int KS>
__device__ __forceinline__ int load_stage_page(const KeySource &ks, int it, int wave)
{
    const const_i32 *bt = (const const_i32 *)(uintptr_t)ks.bt_row;
    return bt[min(it * (kBNW * KS / kPage) + wave, ks.max_blocks - 1)];   // clamped entries are never used
}

// Fused KV append: workgroup `blk` of `nblk` copies chunk rows blk, blk + nblk, ... (K and V of
// every kv head, 16 bytes per thread and pass) into slot (ctx + t) % 16 of page
// block_table[s][(ctx + t) / 16].  Same result as the stand-alone append kernel, bit for bit.
// First every thread looks up where one of the workgroup's rows goes (table in LDS); then rows
// are copied 8 at a time with all their loads issued before the first store, so that a
// workgroup has tens of KB in flight.
template <int D>
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
            // of the row's K vector 0 of head 0, in 16-byte units
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
                for (int r = 0; r < R; ++r) reinterpret_cast<u32x4 *>(p.pages_w)[row_dst[min(r0 + r, rows_here - 1)] + in_page] = v[r];
            }
        }
        __syncthreads();
    }
}

// The launch parameters as the jobs of a workgroup read them: from a copy in LDS (the kernel
// argument segment is host memory, one read of it per launch is enough), word by word into
// scalar registers, anew by every job and once more after a job's main loop, so that they do not
// occupy scalar registers across the loop.
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

// What a helper workgroup's wavefront remembers of its first tile when it goes on to its second
// one before the hand-over of the first is settled (see tile_job).
struct Handover {
    int unit = -1;          // (head group, tile, slot) whose partial result is stored but not announced yet
    int old = 0;            // lane 0: what the arrival counter held when it was announced
    bool announced = false;
    int seg_cu = 0, t0 = 0, n_s = 0;    // where the tile's rows are
};

// The two pieces of a split tile, merged, normalised and written.  (o, m, l): this wavefront's
// piece; `other`: the other piece in the scratch memory.  Whichever piece calls this, the value is
// fma(piece 1, its weight, piece 0 * its weight).
template <int D>
__device__ __forceinline__ void merge_pieces_and_store(f32x16 (&o)[D / 32], float m, float l, const char *other, int piece, int lane,
                                                       bool row_ok, uint16_t *orow)
{
    constexpr int DBLK = D / 32;
    const int half = lane >> 5, l32 = lane & 31;
    const f32x4 *qo = reinterpret_cast<const f32x4 *>(other);
    const float *qs = reinterpret_cast<const float *>(other + (size_t)DBLK * 4 * 64 * 16);
    float m1, l1;
    f32x4 x[DBLK * 4];
    load_partial(qo + lane, qs + l32, x, m1, l1);
    const float mstar = fmaxf(m, m1);
    const float w_own = __builtin_amdgcn_exp2f(m - mstar), w_oth = __builtin_amdgcn_exp2f(m1 - mstar);
    l = piece == 0 ? __builtin_fmaf(l1, w_oth, l * w_own) : __builtin_fmaf(l, w_own, l1 * w_oth);
    if (!row_ok) return;
    const float inv = __builtin_amdgcn_rcpf(l);
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float y = o[db][q4 * 4 + e], z = x[db * 4 + q4][e];
                const float r = piece == 0 ? __builtin_fmaf(z, w_oth, y * w_own) : __builtin_fmaf(y, w_own, z * w_oth);
                w[e] = (__bf16)(r * inv);
            }
            *reinterpret_cast<uint2 *>(orow + db * 32 + q4 * 8 + 4 * half) = __builtin_bit_cast(uint2, w);
        }
}

// One piece of one row tile of one head group: `piece` 0 is the whole key range, or, when the
// launch splits key ranges (p.tail_q8 != 0), all but its last third; piece 1 is that last third.
// The two pieces of a split tile meet through the launch's scratch memory: each wavefront stores
// its unnormalised (O, m, row sum), and the one that finds the other's already there merges and
// writes the output rows.  Nobody waits for anybody.
template <int D, int KS>
__device__ __forceinline__ void tile_job(const AttnParams &kernarg, bool first_job, const AttnParams *params, uint4 *smem, float (*Mstat)[2][32],
                                         uint32_t (*peek)[64], int grp, int tile_index, int piece, Handover &ho, bool may_defer)
{
    // a workgroup's first job starts from the kernel arguments themselves: the copy in LDS is only
    // known to be complete after the job's first barrier
    AttnParams p = kernarg;
    if (!first_job) {
        asm volatile("" ::: "memory");               // keeps this a branch: the reads are not done speculatively
        p = read_params(params);
    }

    constexpr int CH = D / 8;        // 16-byte chunks per K/V row
    constexpr int KSTEPS = D / 16;   // MFMA steps over d for S^T
    constexpr int DBLK = D / 32;     // 32-row blocks of O^T
    constexpr int NKB = kBNW / 32;   // 32-key blocks of S^T per wavefront per stage
    constexpr int STAGE = kBNW * KS; // keys per stage
    constexpr int STAGE_U4 = STAGE * CH;

    // The thread id is made opaque per job: values derived from it are then computed where a job
    // needs them instead of being kept in registers across the whole job loop.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int slot = wave % kSlots, kq = wave / kSlots;    // row/head slot, key part
    const int half = lane >> 5, l32 = lane & 31;
    const int BM = 32 << p.rb_shift;
    const int S = p.S;
    int tile = tile_index;

    // ---- which (segment, row tile) is it?  Tiles never span two segments.  64 segments are
    // examined at a time: lane l takes segment s0 + l, a wave-wide prefix sum of the tile counts
    // finds the segment that owns `tile`.  The lane also fetches what the owner will need next
    // (context length, the page of this wavefront's first rows), so that the kernel's first loads
    // of K and V are one memory round trip away from its start, not three.
    int s = -1, t0 = -1, seg_cu = 0, n_s = 0, L = 0, page = 0, page_hi = 0;
    const int first_page = min(wave, p.max_blocks - 1), first_page_hi = min(wave + kSlots, p.max_blocks - 1);
    for (int s0 = 0; s0 < S; s0 += 64) {
        const int idx = s0 + lane;
        const int a = idx < S ? p.cu[idx] : 0, b = idx < S ? p.cu[idx + 1] : 0;
        const int ctx_len = idx < S ? p.ctx[idx] : 0;
        const int pg = idx < S ? p.bt[(size_t)idx * p.max_blocks + first_page] : 0;
        const int pg_hi = idx < S ? p.bt[(size_t)idx * p.max_blocks + first_page_hi] : 0;
        const int nt = (b - a + BM - 1) >> (5 + p.rb_shift);   // 0 for lanes past the last segment
        int incl = nt;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int y = __shfl_up(incl, d, 64);
            if (lane >= d) incl += y;
        }
        const unsigned long long owner = __builtin_amdgcn_ballot_w64(tile >= incl - nt && tile < incl);
        if (owner != 0) {
            const int src = __builtin_ctzll(owner);
            s = s0 + src;
            t0 = (tile - __builtin_amdgcn_readlane(incl - nt, src)) * BM;
            seg_cu = __builtin_amdgcn_readlane(a, src);
            n_s = __builtin_amdgcn_readlane(b - a, src);
            L = __builtin_amdgcn_readlane(ctx_len, src);
            page = __builtin_amdgcn_readlane(pg, src);
            page_hi = __builtin_amdgcn_readlane(pg_hi, src);
            break;
        }
        tile -= __builtin_amdgcn_readlane(incl, 63);
    }
    const int hh = slot & (p.hpw - 1), rbk = slot >> p.hpw_shift;
    const int head = grp * p.hpw + hh;
    if (t0 < 0) {
        // padding rows [cu[S], C): written as +0
        const int r0 = p.cu[S] + tile * BM + 32 * rbk;
        if (r0 >= p.C || kq != 0 || piece != 0) return;
        const int r = r0 + l32;
        if (r < p.C) {
            uint4 *o = reinterpret_cast<uint4 *>(p.out + ((size_t)r * p.Hq + head) * D);
            for (int c = half; c < CH; c += 2) o[c] = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    TETRI_MARK(1);
    KeySource ks;
    ks.pages = p.pages; ks.k_new = p.k_new; ks.v_new = p.v_new;
    ks.bt_row = p.bt + (size_t)s * p.max_blocks;
    ks.Hkv = p.Hkv; ks.kh = magic_div(grp, p.kv_magic); ks.row_base = seg_cu; ks.L = L;
    ks.n_new = min(n_s, t0 + BM);                      // new keys any row of this tile may see
    ks.n_ctx_tiles = (L + STAGE - 1) / STAGE;
    ks.max_blocks = p.max_blocks;
    const int n_all = ks.n_ctx_tiles + (ks.n_new + STAGE - 1) / STAGE;
    // 0 when the launch does not split, and for key ranges too short to be worth a hand-over.  A
    // helper has about split_bias stages' worth of extra work (a second tile's prologue, handing
    // its first result over): the three workgroups of two tiles finish together when each tile
    // hands over a third of what exceeds that.
    const int n_tail = n_all >= p.split_min ? (max(n_all - p.split_bias, 0) * p.tail_q8 + 128) >> 8 : 0;
    if (piece != 0 && n_tail == 0) return;
    const int it_begin = piece == 0 ? 0 : n_all - n_tail;
    const int n_stages = piece == 0 ? n_all - n_tail : n_all;          // end of this piece's stage range

    const int tw0 = t0 + 32 * rbk;         // first local row of this wavefront
    const int t = tw0 + l32;               // local row of this lane's query
    const bool row_ok = t < n_s;
    const bool wave_has_rows = tw0 < n_s;

    const int new_row_bytes = p.Hkv * D * 2;
    LaneOffsets<D> lo;
    init_lane_offsets<D>(lo, lane, new_row_bytes);
    const uint32_t smem_lds = lds_address(smem);
    constexpr uint32_t STAGE_BYTES = STAGE_U4 * 16;   // bytes of one matrix of one stage

    WaveSrc ws;
    ws.pool_k = reinterpret_cast<const char *>(p.pages) + (size_t)ks.kh * (kPage * D * 2);
    ws.page_bytes = 2 * p.Hkv * (kPage * D * 2);
    ws.v_delta = p.Hkv * (kPage * D * 2);
    {
        const size_t off = ((size_t)ks.row_base * p.Hkv + ks.kh) * (size_t)(D * 2);
        ws.new_k = reinterpret_cast<const char *>(p.k_new) + off;
        ws.new_v = reinterpret_cast<const char *>(p.v_new) + off;
    }
    ws.stage_new_bytes = STAGE * new_row_bytes;
    ws.wave_new_bytes = 16 * new_row_bytes;
    static_assert(kBNW * KS / kPage == kSlots * KS, "stage 0: wavefront w loads page w of the segment");
    // Stage 0: the wavefronts of key part 0 reach this point first (the older wavefront of a SIMD
    // is served first), so they issue the loads of their partner in part 1 as well.
    StageLoads sl;
    if (kq == 0) {
        if (it_begin != 0) {                         // the lookup fetched the pages of stage 0
            page = load_stage_page<KS>(ks, it_begin, wave);
            page_hi = load_stage_page<KS>(ks, it_begin, wave + kSlots);
        }
#pragma unroll
        for (int part = 0; part < KS; ++part) {
            const bool full = describe_stage_loads<D, KS>(ks, ws, lo, part == 0 ? page : page_hi, it_begin, wave + part * kSlots, new_row_bytes,
                                                          smem_lds + (it_begin & 1) * STAGE_BYTES, sl);
            issue_stage_loads<D, KS>(sl, full, lane);
        }
    }
    // The loads of the next stage are not issued by all wavefronts at once right after the barrier:
    // the load unit takes a wavefront's 8 KB in about 128 cycles and a wavefront that finds it busy
    // stalls in front of its own matrix instructions.  Each wavefront has one of four points in
    // the instruction stream between two barriers at which it issues its loads (the two wavefronts
    // of a SIMD use different ones), so that at any time most wavefronts are computing.
    bool pend = false;                               // the next stage's loads are described in sl, not issued
    const int load_point = (wave + (kq != 0 ? 2 : 0)) & 3;
    page = load_stage_page<KS>(ks, it_begin + 1, wave);

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds q[t][16*st + 8*half .. +7].  Lanes
    // past the segment's last row read its first row instead: their results are never stored.
    bf16x8 qf[KSTEPS];
    {
        const uint4 *qp = reinterpret_cast<const uint4 *>(p.q + ((size_t)(seg_cu + (row_ok ? t : 0)) * p.Hq + head) * D);
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st) qf[st] = __builtin_bit_cast(bf16x8, qp[2 * st + half]);
    }

    f32x16 o[DBLK];
#pragma unroll
    for (int i = 0; i < DBLK; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[i][v] = 0.f;
    float m = -1e30f;        // running row max (in units of log2: score * c)
    float lsum = 0.f;        // this lane's share of the running row sum
    // scores are multiplied by c = scale * log2(e), of either sign; a masked score is the infinity
    // that c turns into -inf
    const float c = p.neg ? -p.c : p.c;
    const float masked = p.neg ? INFINITY : -INFINITY;
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
    // off = buffer * STAGE_BYTES + block * BLOCK_BYTES
    auto load_k = [&](bf16x8 (&kf)[KSTEPS], int off) {
#pragma unroll
        for (int st = 0; st < KSTEPS; ++st)
            kf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(smem_b + kbase[st] + off));
    };
    auto load_v = [&](s16x8 (&vf)[2 * DBLK], int off) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                const char *a = smem_b + vbase[db] + off + j * (16 * D * 2);
                const s16x4 va = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)a);
                const s16x4 vb4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(a + 8 * D * 2));
                vf[j * DBLK + db] = __builtin_shufflevector(va, vb4, 0, 1, 2, 3, 4, 5, 6, 7);
            }
    };

    // Number of 32-key blocks of stage `it` this wavefront works on (a prefix of its 64-key part):
    // those inside the key range and not entirely past the wavefront's rows.
    auto stage_blocks = [&](int it) -> int {
        if (!wave_has_rows) return 0;
        const bool is_ctx = it < ks.n_ctx_tiles;
        const int part0 = (is_ctx ? it : it - ks.n_ctx_tiles) * STAGE + kq * kBNW;
        int nblk = 0;
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb) {
            const int key0 = part0 + kb * 32;
            if (is_ctx ? key0 < L : (key0 < ks.n_new && key0 <= tw0 + 31)) nblk = kb + 1;
        }
        return nblk;
    };
    // Make stage `it` the current one: its loads have landed for every wavefront, nobody reads the
    // other buffer any more, so the loads of stage it+1 can go there.  `page` always belongs to
    // the stage whose loads are issued next; it is fetched one stage ahead.
    // Entering a stage has two halves: the wait, after which the wavefront may read the stage (it
    // requests its first K fragments from LDS right away), and handing out the next stage's loads.
    // `pv_before`: a PV product is pending, i.e. deferred loads will meet their issue point before
    // the next stage is entered.
    auto issue_pending = [&](int point) {
        if (pend && load_point == point) {
            issue_stage_loads<D, KS>(sl, true, lane);
            pend = false;
        }
    };
    auto sync_stage = [&](int it) -> int {
        if (pend) {                                    // rare: the stage had too few blocks to reach the point
            issue_stage_loads<D, KS>(sl, true, lane);
            pend = false;
        }
        wait_vm<0>();
        __syncthreads();
        return stage_blocks(it);
    };
    auto next_stage_loads = [&](int it, int nb, bool pv_before) {
        if (it + 1 < n_stages) {
            const bool full = describe_stage_loads<D, KS>(ks, ws, lo, page, it + 1, wave, new_row_bytes, smem_lds + ((it + 1) & 1) * STAGE_BYTES, sl);
            if (full && pv_before && nb != 0 && load_point != 0) pend = true;
            else issue_stage_loads<D, KS>(sl, full, lane);
        }
        page = load_stage_page<KS>(ks, it + 2, wave);
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
    TETRI_MARK(2);
    int nblk = sync_stage(it);
    if (ho.unit >= 0 && !ho.announced) {
        // the previous tile's partial result was stored before this job began; the wait in front of
        // the barrier just passed covered those stores, so it can be announced now.  What the
        // counter held is looked at when this job is done.
        if (lane == 0) ho.old = atomicAdd(p.counters + ho.unit, 1);
        ho.announced = true;
    }
    TETRI_MARK(3);
    while (nblk == 0 && it + 1 < n_stages) {
        next_stage_loads(it, 0, false);
        nblk = sync_stage(++it);
    }
    if (nblk != 0) {
        int kb = 0;
        bf16x8 kf[KSTEPS];
        load_k(kf, (it & 1) * STAGE_BYTES);
        next_stage_loads(it, nblk, false);
        bf16x2 ones;
        ones[0] = (__bf16)1.0f; ones[1] = (__bf16)1.0f;
        // weights of a block from its scores and the row's reference exponent m: bf16-rounded, laid out
        // as the B operand of the PV product; returns this lane's sum of the rounded weights (the row
        // sum is taken over the weights the PV product uses)
        auto weights = [&](const f32x16 &sc, bf16x8 (&pf)[2]) -> float {
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
            return l_blk;
        };
        // The second half of a block: scores of the next block (its K fragments
        // are in kf; discarded after the last block) on the matrix cores, interleaved with
        // exponentiating and rounding this block's weights on the VALU against the reference exponent
        // m the row already has; then the PV product with the V fragments in vf.
        auto softmax_pv = [&](f32x16 &s_cur, f32x16 &s_next, const s16x8 (&vf)[2 * DBLK]) {
            bf16x8 pf[2];
            float l_blk;
            if constexpr (KS == 1) {
                // Four-wavefront workgroups run two to a compute unit, so the two wavefronts of a SIMD belong
                // to different workgroups and are not held in step by a common barrier.  Here the block has a
                // VALU phase (the weights) and an MFMA phase at raised wavefront priority: one wavefront's
                // matrix instructions go out back to back while the other, in its VALU phase, takes the issue
                // slots in between (measured: +7 to +13 % on launches with two workgroups per compute unit; for
                // eight-wavefront workgroups, whose SIMD partners meet at every barrier, no gain).
                __builtin_amdgcn_sched_barrier(0);
                l_blk = weights(s_cur, pf);
                __builtin_amdgcn_sched_barrier(0);
                issue_pending(1);
                __builtin_amdgcn_s_setprio(3);
                s_next = qk(kf);
                __builtin_amdgcn_sched_barrier(0);
            } else {
                __builtin_amdgcn_sched_barrier(0);
                s_next = qk(kf);
                l_blk = weights(s_cur, pf);
                // wanted order: one MFMA of the score chain, then its share of the VALU operations, 8 times
#pragma unroll
                for (int g = 0; g < KSTEPS; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 48 / KSTEPS, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                issue_pending(1);
            }
            // m is only a reference point, not the exact row maximum: any value keeps the result exact
            // as long as the weights stay in range.  Only when a lane's weights of this block sum to
            // more than 2^16 (or overflowed: first block, or scores far above anything seen before) is
            // m raised to the true maximum, O and the row sum rescaled in place, and the weights
            // recomputed.  The two half-waves of a row take the same decision.  (In the
            // phased order the vote sits behind the score MFMAs, where its operands are long there.)
            if (__builtin_amdgcn_ballot_w64(!(l_blk <= 65536.0f)) != 0) {
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
                l_blk = weights(s_cur, pf);
            }
            lsum += l_blk;
            // O^T += V^T P^T.  Step j contracts the 16 keys held in accumulator elements 8j..8j+7.
#pragma unroll
            for (int j = 0; j < 2; ++j) {
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
                    o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[j * DBLK + db]), pf[j], o[db], 0, 0, 0);
                if (KS != 1 && j == 0) issue_pending(2);
            }
            if constexpr (KS == 1) {
                __builtin_amdgcn_s_setprio(0);
                __builtin_amdgcn_sched_barrier(0);
                issue_pending(2);
            }
        };
        // One block: scores s_cur are ready; computes s_next for the block after it.  Returns false
        // after the last block.
        auto block = [&](f32x16 &s_cur, f32x16 &s_next) -> bool {
            const bool is_ctx = it < ks.n_ctx_tiles;
            const int key0 = (is_ctx ? it : it - ks.n_ctx_tiles) * STAGE + kq * kBNW + kb * 32;
            const bool need_mask = is_ctx ? (key0 + 32 > L) : (key0 + 31 > tw0);
            const int bound = is_ctx ? L - 1 : t;      // last visible key index of this phase
            // V fragments of this block: in registers before the stage may be left
            s16x8 vf[2 * DBLK];
            load_v(vf, (it & 1) * STAGE_BYTES + kb * BLOCK_BYTES);
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
                    if (nblk == 0) next_stage_loads(it, 0, true);
                }
                have_next = entered = nblk != 0;
            }
            if (have_next) load_k(kf, (it & 1) * STAGE_BYTES + kb * BLOCK_BYTES);
            if (entered) next_stage_loads(it, nblk, true);
            else issue_pending(3);
            // ---- mask: accumulator element v is key key0 + (v/4)*8 + 4*half + v%4; keys past `bound`
            // (the end of the cached context, or the query's own position) get weight exp2(-inf) = 0
            if (need_mask) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = key0 + (v / 4) * 8 + 4 * half + (v % 4);
                    if (key > bound) s_cur[v] = masked;
                }
            }
            softmax_pv(s_cur, s_next, vf);
            return have_next;
        };
        f32x16 s_a = qk(kf), s_b;
        for (;;) {
            if (!block(s_a, s_b)) break;
            if (!block(s_b, s_a)) break;
        }
    }

    TETRI_MARK(4);
    // ---- merge the KS key parts through LDS: part 1 publishes (m, row sum, O), part 0 finishes.
    // The partial O goes into the stage buffer that held the stage before the last one: nobody reads
    // it any more once every wavefront has entered the last stage, so no barrier is needed before
    // writing.  Its K region takes slots 0 and 1, its V region slots 2 and 3; lane l's four
    // consecutive accumulator elements are one 16-byte unit.
    // A split tile: is the other piece there already?  The answer travels while the key parts merge.
    asm volatile("" ::: "memory");                   // a fresh read, not the values from before the loop
    const AttnParams pe = read_params(params);
    const size_t unit = ((size_t)grp * pe.tiles + tile_index) * kSlots + slot;
    if (n_tail != 0 && kq == 0 && wave_has_rows) peek_coherent(pe.counters + unit, lds_address(peek[slot]));
    float ltot = half_swap_sum(lsum);
    if constexpr (KS == 2) {
        static_assert(2 * (DBLK * 16 * 64 * 4) == STAGE_BYTES, "two slots per matrix region");
        char *dead = reinterpret_cast<char *>(smem) + (n_stages & 1) * STAGE_BYTES + (slot >> 1) * (2 * STAGE_BYTES);
        f32x4 *part = reinterpret_cast<f32x4 *>(dead + (slot & 1) * (DBLK * 16 * 64 * 4));
        if (kq == 1) {
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = o[db][q4 * 4 + e];
                    part[(db * 4 + q4) * 64 + lane] = x;
                }
            if (half == 0) { Mstat[slot][0][l32] = m; Mstat[slot][1][l32] = ltot; }
        }
        __syncthreads();
        TETRI_MARK(5);
        if (kq == 1) return;
        const float m1 = Mstat[slot][0][l32], l1 = Mstat[slot][1][l32];
        const float mstar = fmaxf(m, m1);
        const float w0 = __builtin_amdgcn_exp2f(m - mstar), w1 = __builtin_amdgcn_exp2f(m1 - mstar);
        ltot = ltot * w0 + l1 * w1;
        m = mstar;
        if (!wave_has_rows) return;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 x = part[(db * 4 + q4) * 64 + lane];
#pragma unroll
                for (int e = 0; e < 4; ++e) o[db][q4 * 4 + e] = o[db][q4 * 4 + e] * w0 + x[e] * w1;
            }
    } else {
        if (!wave_has_rows) return;
    }

    // ---- a split tile: if the other piece is there, merge with it; else leave (O, m, row sum) in
    // the scratch memory and announce it, which tells whether the other piece has arrived in the
    // meantime.  unit = (head group, tile, slot); the counter of a unit goes 0 -> 1 -> 0.
    if (n_tail != 0) {
        constexpr size_t UNIT_BYTES = (size_t)DBLK * 4 * 64 * 16 + 2 * 32 * 4;
        const size_t units = (size_t)pe.groups * pe.tiles * kSlots;
        char *mine = pe.scratch + ((size_t)piece * units + unit) * UNIT_BYTES;
        const char *other = pe.scratch + ((size_t)(1 - piece) * units + unit) * UNIT_BYTES;
        wait_vm<0>();
        if (__builtin_amdgcn_readfirstlane(peek[slot][lane]) == 0) {
            f32x4 *po = reinterpret_cast<f32x4 *>(mine);
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    f32x4 x;
#pragma unroll
                    for (int e = 0; e < 4; ++e) x[e] = o[db][q4 * 4 + e];
                    store_coherent(po + (db * 4 + q4) * 64 + lane, x);
                }
            float *ps = reinterpret_cast<float *>(mine + (size_t)DBLK * 4 * 64 * 16);
            if (half == 0) { store_coherent(ps + l32, m); store_coherent(ps + 32 + l32, ltot); }
            if (may_defer) {
                // a helper with a second tile to do: neither the end of the stores nor the answer of
                // the arrival counter is waited for here (about 4 us)
                ho.unit = (int)unit;
                ho.announced = false;
                ho.seg_cu = seg_cu; ho.t0 = t0; ho.n_s = n_s;
                return;
            }
            coherent_stores_done();                  // this wavefront's partial is in memory ...
            int arrived = 0;
            if (lane == 0) arrived = atomicAdd(pe.counters + unit, 1);     // ... before it is announced
            arrived = __builtin_amdgcn_readfirstlane(arrived);
            if (arrived == 0) return;                // first of the two: the other piece finishes the tile
        }
        if (lane == 0) pe.counters[unit] = 0;        // ready for the next launch
        merge_pieces_and_store<D>(o, m, ltot, other, piece, lane, row_ok, pe.out + ((size_t)(ks.row_base + t) * pe.Hq + head) * D);
        return;
    }

    // ---- normalise and store: lane holds out[t][head][db*32 + (v/4)*8 + 4*half + v%4]
    if (!row_ok) return;
    const float inv = __builtin_amdgcn_rcpf(ltot);
    uint16_t *orow = pe.out + ((size_t)(ks.row_base + t) * pe.Hq + head) * D;
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o[db][q4 * 4 + e] * inv);
            *reinterpret_cast<uint2 *>(orow + db * 32 + q4 * 8 + 4 * half) = __builtin_bit_cast(uint2, w);
        }
    TETRI_MARK(6);
}

template <int D, int KS>
__global__ __launch_bounds__(kSlots * KS * 64, 2) void attn_tile_kernel(AttnParams p)
{
    constexpr int STAGE_U4 = kBNW * KS * (D / 8);
    __shared__ uint4 smem[4 * STAGE_U4];             // K and V of two stage buffers: K0 | K1 | V0 | V1
    __shared__ float Mstat[kSlots][2][32];
    __shared__ uint32_t peek[kSlots][64];            // where a look at a split tile's arrival counter lands
    __shared__ AttnParams params;
    TETRI_MARK(0);

    // ---- fused KV append: append_blocks workgroups copy the chunk's new K/V rows into their page
    // slots.  They come after the attention workgroups that certainly have work (attn_first of
    // them) and before those that probably have none, so that they start on the CUs the attention
    // grid leaves idle instead of waiting for one to finish.
    int abid = blockIdx.x;                           // index in the attention grid
    if (abid >= p.attn_first) {
        if (abid < p.attn_first + p.append_blocks) {
            append_rows<D>(p, reinterpret_cast<unsigned long long *>(smem), abid - p.attn_first, p.append_blocks, threadIdx.x, kSlots * KS * 64);
            return;
        }
        abid -= p.append_blocks;
    }
    // ---- workgroup id -> (head group, job).  The workgroups of a head group run on one XCD (they
    // read the same K and V through its L2); an XCD has gpx groups and starts their workgroups job
    // by job.  Without key-range splitting the jobs of a group are its row tiles, late (long) ones
    // first.  With it (helpers != 0): first the tiles but the last one of the host's bound (which
    // exists only if the chunk has ragged segments), then the helpers, each doing the last third
    // of the key ranges of two of those tiles.  The bound's last tile gets no workgroups of its own
    // (they would start when the first compute unit becomes free and, though empty, end after
    // everybody else: kernel start-up and the look-up take 2-3 us): its two pieces are one more job of
    // the workgroup of tile 0, whose key range is the shortest, and of the last helper.
    const int xcd = abid % kXcd, local = abid / kXcd;
    const int job = magic_div(local, p.gpx_magic);
    const int grp = xcd * p.gpx + (local - job * p.gpx);
    const int T = p.tiles, H = p.helpers;
    if (grp >= p.groups || job >= (H != 0 ? T + H - 2 : T)) return;
    if (threadIdx.x == 0) params = p;                // from scalar registers: no memory read to wait for
    int piece = 0, first = T - 1 - job, count = 1, extra = 0;
    if (H != 0) {
        if (job < T - 1) {
            first = T - 2 - job;
            extra = first == 0;
        } else {
            piece = 1;
            first = T - 2 - 2 * (job - (T - 1));
            count = min(2, first + 1);
            extra = job == T + H - 3;
        }
    }
    Handover ho;
    for (int i = 0; i < count + extra; ++i) {
        if (i != 0) __syncthreads();                 // the stage buffers change hands
        // only the hand-over of a helper's first tile is left open while it does its second one
        tile_job<D, KS>(p, i == 0, &params, smem, Mstat, peek, grp, i < count ? first - i : T - 1, piece, ho, i + 1 < count);
    }
    // ---- a helper's first tile whose hand-over was left open: if the other piece has arrived in the
    // meantime (it found the counter at 0 and went away), this wavefront finishes the tile from its
    // own stored partial result.
    if (ho.unit >= 0) {
        constexpr int DBLK = D / 32;
        constexpr size_t UNIT_BYTES = (size_t)DBLK * 4 * 64 * 16 + 2 * 32 * 4;
        asm volatile("" ::: "memory");
        const AttnParams pd = read_params(&params);
        const int lane = threadIdx.x & 63;
        if (!ho.announced) {                         // the second job ended before its first barrier
            wait_vm<0>();
            if (lane == 0) ho.old = atomicAdd(pd.counters + ho.unit, 1);
        }
        if (__builtin_amdgcn_readfirstlane(ho.old) != 0) {
            if (lane == 0) pd.counters[ho.unit] = 0;
            const size_t units = (size_t)pd.groups * pd.tiles * kSlots;
            const char *mine = pd.scratch + (units + ho.unit) * UNIT_BYTES;          // piece 1
            const char *other = pd.scratch + (size_t)ho.unit * UNIT_BYTES;           // piece 0
            f32x4 x[DBLK * 4];
            float m, l;
            load_partial(reinterpret_cast<const f32x4 *>(mine) + lane, reinterpret_cast<const float *>(mine + (size_t)DBLK * 4 * 64 * 16) + (lane & 31), x, m, l);
            f32x16 o[DBLK];
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] = x[db * 4 + v / 4][v % 4];
            const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), slot = wave % kSlots;
            const int head = grp * pd.hpw + (slot & (pd.hpw - 1));
            const int t = ho.t0 + 32 * (slot >> pd.hpw_shift) + (lane & 31);
            merge_pieces_and_store<D>(o, m, l, other, 1, lane, t < ho.n_s, pd.out + ((size_t)(ho.seg_cu + t) * pd.Hq + head) * D);
        }
    }
}

template <int D, int KS>
hipError_t launch(const AttnParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL((attn_tile_kernel<D, KS>), dim3(p.attn_grid + p.append_blocks), dim3(kSlots * KS * 64), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t tetri_launch_attn(const tetri_ctx *h, const AttnParams &p, int key_parts, hipStream_t stream)
{
    if (h->cfg.head_dim == 128)
        return key_parts == 2 ? launch<128, 2>(p, stream) : launch<128, 1>(p, stream);
    return key_parts == 2 ? launch<64, 2>(p, stream) : launch<64, 1>(p, stream);
}
