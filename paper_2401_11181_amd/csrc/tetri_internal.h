// Internal declarations shared by the host layer and the kernel launchers of libtetri.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>

#include "tetri.h"

struct tetri_ctx {
    tetri_config cfg;
    std::string err;
    int attn_variant = 0;   // 0 = library's choice, 1 / 2 = shared-tile kernel with 1 / 2 key parts
    int split_keys = 1;     // 1 = launches with fewer than two row tiles per CU divide the stages of every head group evenly over the CUs
    int stream_wgs = 0;     // workgroups per head group of such a launch (0: as many as the device has CUs for); > 0 forces the mode
    int split_min_stages = 8;   // tail mode: the shortest key range that hands its tail to a helper workgroup
    int split_bias_stages = 6;  // a helper's overhead, in stages (see the kernel)
    int split_share_q8 = 85;    // the share of the remaining stages a tile hands over, in 1/256 (a third)
    int decode_parts = 0;       // key parts per (request, kv head) of the decode kernel (0: the library chooses)
    int transfer_slabs = 0;     // (K / V, head) slabs per workgroup of the export / import kernels (0: the library chooses)
    int device = 0;         // the device the handle was created on; its scratch memory lives there
    int num_cus = 0;
    char *scratch = nullptr;        // partial results of tiles shared by workgroups: 2 x scratch_units units
    int32_t *counters = nullptr;    // two sets of n_counters arrival counters: a launch uses one and zeroes the other
    size_t scratch_units = 0, unit_bytes = 0;
    int32_t n_counters = 0;
    int counter_set = 0;            // the set the next dividing launch uses
    bool divide_launched = false;       // a launch has used scratch and counters ...
    hipStream_t last_divide_stream = nullptr;   // ... the last one on this stream
    float *static_scratch = nullptr;    // this device's address of the library's static scratch array (decode parts)
    size_t static_scratch_bytes = 0;
};

// Size of the static device array behind tetri_decode_attn_static.
constexpr size_t kDecodeStaticScratchBytes = (size_t)8 << 20;

// Launch parameters of the attention kernels (passed by value).
struct AttnParams {
    const uint16_t *q, *k_new, *v_new, *pages;   // bf16 bit patterns
    const int32_t *bt, *cu, *ctx;
    uint16_t *out;
    uint16_t *pages_w;    // pool for the fused append (null when append_blocks == 0)
    int32_t S, C, Hq, Hkv, g;
    int32_t hpw;          // query heads handled by one workgroup (they share one kv head)
    int32_t rb;           // 32-row blocks handled by one workgroup
    int32_t hpw_shift, rb_shift;   // log2 of the two
    int32_t groups;       // Hq / hpw: head groups, one workgroup column each
    int32_t stream_wgs;   // workgroups per head group that share its stages evenly (0: one workgroup per row tile ...)
    int32_t helpers;      // ... plus, per head group, this many that take the tails of two tiles' key ranges each (0: none)
    int32_t tail_q8;      // the share of a tile's stages that goes to its helper, in 1/256
    int32_t split_min;    // only key ranges of at least this many stages hand a tail over
    int32_t split_bias;   // stages not counted when a key range's tail is measured
    int32_t n_counters;   // size of a set of arrival counters
    int32_t gpx;          // head groups per XCD
    uint32_t gpx_magic;   // ceil(2^32 / gpx), 0 for 1
    char *scratch;        // partial results of tiles shared by several workgroups
    int32_t *counters;    // one per (group, tile, slot), all zero when the launch begins
    int32_t *counters_next;   // the set of the next such launch: zeroed by this one
    uint32_t kv_magic;    // the same for g / hpw: head group -> kv head
    int32_t max_blocks;
    int32_t tiles;        // upper bound of the number of row tiles of the chunk
    int32_t attn_grid;    // workgroups of the attention grid (a multiple of 8)
    int32_t append_blocks; // extra workgroups that do the fused KV append (0: none)
    int32_t attn_first;   // attention workgroups that precede them in the grid (a multiple of 8)
    float c;              // |scale| * log2(e)
    int32_t neg;          // 1 if scale < 0
    // FP8 cache (the kernel variant that reads a pool of E4M3 codes): cached K / V = value(code) * scale
    float k_scale, v_scale;
    float k_inv, v_inv;   // fl32(1 / scale): the fused append quantises with them
};

struct AppendParams {
    const uint16_t *k_new, *v_new;
    uint16_t *pages;
    const int32_t *bt, *cu, *ctx;
    int32_t S, Hkv, D, max_blocks;
};

// Launch parameters of the KV export / import kernels.
struct TransferParams {
    uint16_t *pool;       // the paged pool (read by export, written by import)
    uint16_t *buf;        // the dense transfer buffer (written by export, read by import)
    const int32_t *bt, *cu, *first;   // first may be null: every range starts at token 0
    int32_t R, Hkv, max_blocks;
    int32_t slabs_per_wg; // (K / V, head) slabs one workgroup moves
    float k_inv, v_inv;   // quantising export: fl32(1 / scale) of the K and of the V half
};

// Launch parameters of the decode-iteration kernels.
struct DecodeParams {
    const uint16_t *q, *k_new, *v_new, *pages;
    const int32_t *bt, *ctx;
    uint16_t *out;
    uint16_t *pages_w;    // pool for the fused append of the new token (null: no append)
    float *partial;       // scratch: [(request * Hq + head) * parts + part][D + 2] = unnormalised O, m, l
    int32_t B, Hq, Hkv, g, max_blocks;
    int32_t parts;        // workgroups that share one (request, kv head)'s keys
    float c;              // |scale| * log2(e)
    int32_t neg;          // 1 if scale < 0
    int32_t fp8;          // 1: the pool holds E4M3 codes (one byte per element) with per-tensor scales
    float k_scale, v_scale, k_inv, v_inv;   // the scales and fl32(1 / scale)
    float out_scale;      // factor on the finished output: v_scale for an FP8 pool, else 1
};

hipError_t tetri_launch_attn(const tetri_ctx *h, const AttnParams &p, int key_parts, bool fp8_pool, hipStream_t stream);
hipError_t tetri_launch_kv_transfer(const tetri_ctx *h, const TransferParams &p, int32_t row_units, int32_t tiles,
                                    bool to_pool, hipStream_t stream);
hipError_t tetri_launch_kv_export_fp8(const tetri_ctx *h, const TransferParams &p, int32_t tiles, hipStream_t stream);
hipError_t tetri_launch_decode(const tetri_ctx *h, const DecodeParams &p, hipStream_t stream);
// Device address (on the current device) and size of the static scratch array of the decode kernels.
hipError_t tetri_decode_static_scratch(float **ptr, size_t *bytes);
hipError_t tetri_launch_append(const tetri_ctx *h, const AppendParams &p, int32_t chunk_rows, hipStream_t stream);
