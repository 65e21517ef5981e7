// Internal declarations shared by the translation units of liblora (host side only;
// kernels live in the .hip files and are reached through the launch_* functions).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/lora.h"

namespace lora {

// One entry of the device pointer table: 32 bytes, ordered [layer][adapter][expert][proj].
struct Unit {
    const uint16_t *A;  // packed shrink operand of the unit
    const uint16_t *B;  // packed expand operand of the unit
    float scale;        // the adapter's scale
    int32_t rank;       // the adapter's own rank (<= pool rank; the rest is zero padding)
    int32_t pad[2];
};
static_assert(sizeof(Unit) == 32, "table entry is 32 bytes");

constexpr int kTileRows = 32;        // rows per tile of the long-segment kernels
constexpr int kDecodeTileRows = 16;  // rows per tile of the decode kernels
constexpr int kKBlock = 32;          // K elements per MFMA step (v_mfma_f32_16x16x32_bf16)
constexpr int kColChunk = 128;       // output columns one wave owns in expand
constexpr int kPartKBlocks = 32;     // K-blocks one shrink workgroup reduces (1024 inputs)
constexpr int kMaxParts = 64;
// Shrink and expand in one launch (fused_decode.hip): limits and work split, measured on MI355X
// with the Llama-3-8B query/key/value and output projections (rank 16, 4096 inputs): one launch
// takes 10.3-10.5 us against 13.2-14.1 us for two up to 27 tiles, 12.7 against 14.2 at 41 tiles,
// and the two are equal at 54 tiles; wide outputs (gate and up, 224 chunks) and long inputs
// (down, 14336) are slower in one launch at every size.
constexpr int kFusedMaxK = 4096;       // longest input
constexpr int kFusedMaxChunks = 64;    // widest group, in 128-column chunks per tile
constexpr int kFusedMaxTiles = 64;     // largest batch, as the host's upper bound of the tile count
constexpr int kFusedMinChunks = 16;    // 128-column chunks a workgroup expands at least
constexpr int kFusedWorkgroups = 1024; // workgroups aimed at
// Cache hints of the activation streams of the decode kernels, measured on MI355X with the Mixtral
// shapes (512 to 2900 tokens, top-2): input rows that are read once are streamed from 64 MiB on
// (a quarter of the 256 MiB memory-side cache), the output rows of one call from 256 MiB on.
constexpr int kLongMinRowsTimesRank = 1 << 17;   // long-segment kernels from this many rows x rank on
constexpr int kStreamXMiB = 64;
constexpr int kStreamYMiB = 256;
constexpr int kMaxFused = 3;         // projections that share an input in one launch (q/k/v, gate/up)

// ---- packed layout sizes ---------------------------------------------------------------
inline int kunit_of(int rank) { return rank == 8 ? 64 : kKBlock; }   // K values per packed A block
inline int kblocks_of(int h_in, int rank) { return (h_in + kunit_of(rank) - 1) / kunit_of(rank); }
inline int chunks_of(int h_out) { return (h_out + kColChunk - 1) / kColChunk; }
inline size_t packed_A_bytes(int h_in, int rank) { return (size_t)kblocks_of(h_in, rank) * kunit_of(rank) * rank * 2; }
inline size_t packed_B_bytes(int h_out, int rank) { return (size_t)chunks_of(h_out) * kColChunk * rank * 2; }
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- launch parameter blocks -----------------------------------------------------------
struct PackParams {
    const uint16_t *src;     // first unit's row-major matrix
    int64_t src_stride;      // elements between consecutive units' matrices
    uint16_t *dst;           // first unit's packed destination
    int64_t dst_stride;      // elements between consecutive units' packed matrices
    int n_units;
    int h;                   // h_in (A) or h_out (B)
    int rank;                // pool rank
    int src_rank;            // rank of the source matrices (<= rank)
};

// all A and B repacks of one (adapter, layer) in one launch: job 2j = A, 2j+1 = B of projection j
struct PackLayerParams {
    PackParams job[2 * LORA_MAX_PROJ];
    int n_jobs;
};

struct SegParams {
    const int32_t *adapter_id;
    const int32_t *expert_id;
    int P;
    int n_adapters;
    int n_experts;
    int tile_rows;
    int passes;              // radix passes of 8 bits over the key
    int key_bits;            // bits of the largest key
    int32_t *perm;
    int32_t *seg_start;
    int32_t *seg_key;
    lora_tile *tiles;
    int32_t *counts;
    uint32_t *status;
};

// the multi-workgroup segment builder (segments_large.hip)
struct LargeSegParams {
    SegParams p;
    unsigned *header;        // [0] = active rows, written by the first pass for the next
    unsigned *wg_hist;       // [chunks][256] digit counts per chunk
    unsigned *wg_info;       // [chunks][2] active rows and status bits per chunk
    unsigned *key_g;         // [P] key of every row (kept for later passes), may be null
    const unsigned *order_in;    // rows in the order the previous pass left them
    unsigned *order_out;
    unsigned *chunk_info;    // [chunks][4] segment heads of every chunk of the sorted order
    int G;                   // chunks = workgroups
    int pass;                // 8-bit digit this pass sorts by
};

struct ShrinkParams {
    const Unit *units;       // table rows of the layer
    int n_proj;              // projections per unit (table stride)
    int proj0;               // first projection handled
    int n_fused;             // 1 .. kMaxFused consecutive projections sharing x (same h_in)
    const uint16_t *x;
    int64_t ldx;
    const int32_t *src_row;  // may be null
    const int32_t *perm;
    const lora_tile *tiles;
    const int32_t *counts;
    float *v[kMaxFused];     // per fused projection: [n_parts][P][rank]
    int P;
    int h_in;
    int n_parts;
    int kb_per_part;
    int rank;
    int grid;
    int wave_per_tile;       // decode kernel: every wave takes a whole tile (no K split across waves)
    int build;               // decode kernel: the segments are built inside the launch, from `seg`
    int x_stream;            // decode kernel, K-split form: x rows loaded with the streaming hint (ranks 8, 16: as whole lines)
    SegParams seg;
};

struct ExpandParams {
    const Unit *units;
    int n_proj;
    int proj0;
    int n_fused;             // 1 .. kMaxFused consecutive projections; their widths may differ
    const float *v[kMaxFused];
    int n_parts;
    int P;
    const int32_t *perm;
    const lora_tile *tiles;
    const int32_t *counts;
    void *y[kMaxFused];
    int64_t ldy[kMaxFused];
    int h_out[kMaxFused];
    int n_chunks[kMaxFused]; // 128-column chunks
    int n_slices[kMaxFused]; // decode kernel: wave items per (tile, projection)
    int cps[kMaxFused];      // decode kernel: chunks per wave item (the last of a row may have fewer)
    int slice0[kMaxFused + 1];   // decode kernel: first wave item of a projection within a tile
    void *img[kMaxFused];    // long-segment kernel: operand images of the 16-row sub-tiles
    int image_grid;          // long-segment kernel: workgroups of the image launch
    int waves;               // waves per workgroup
    int tile_group;          // decode kernel: consecutive wave items walk over this many tiles
    int out_f32;
    int overwrite;           // decode kernel, bf16 output: write the update, do not read the rows
    int y_stream;            // decode kernel: output rows read and written with the streaming hint
    int rank;
    int grid;
};

// routing-weighted combine of per-pair update rows into token rows
struct CombineParams {
    const uint16_t *pair;    // bf16 [P][ld_pair] per-pair updates (rows of inactive pairs unspecified)
    int64_t ld_pair;
    const int32_t *adapter_id;
    const int32_t *expert_id;
    const float *route_w;    // [P]
    int T, top_k;
    int n_adapters, n_experts;
    int h_out;
    uint16_t *y;             // bf16 [T][ldy] token rows, updated in place
    int64_t ldy;
};

// shrink and expand of a decode batch in one launch
struct FusedParams {
    ShrinkParams s;          // n_parts = 1; v unused
    ExpandParams e;          // n_slices / cps / slice0: workgroup items of a tile; v unused
};

hipError_t launch_pack_A(const PackParams &p, hipStream_t s);
hipError_t launch_pack_B(const PackParams &p, hipStream_t s);
hipError_t launch_pack_layer(const PackLayerParams &p, hipStream_t s);
hipError_t launch_unpack_A(const PackParams &p, hipStream_t s);   // src = packed, dst = row-major
hipError_t launch_unpack_B(const PackParams &p, hipStream_t s);
hipError_t launch_set_adapter(Unit *table, int n_layers, int n_adapters, int per_adapter, int adapter,
                              int rank, float scale, hipStream_t s);
hipError_t launch_segments(const SegParams &p, void *ws, hipStream_t s);
hipError_t launch_segments_large(const SegParams &p, void *ws, hipStream_t s);
size_t segments_large_ws_bytes(int P);
int inline_build_max_rows();      // limits of the segment build inside the decode shrink
int inline_build_max_keys();
bool segments_large_handles(const SegParams &p);    // does the multi-workgroup builder take this batch?
int segments_large_launches(const SegParams &p);    // kernels it enqueues for it
hipError_t launch_shrink(const ShrinkParams &p, hipStream_t s);
int shrink_long_tiles();                                 // tiles per work item of launch_shrink
hipError_t launch_expand(const ExpandParams &p, hipStream_t s);
size_t expand_image_bytes(int rank, int64_t n_tiles);   // operand images of n_tiles 32-row tiles
int expand_long_group();                                 // tiles per wave item of launch_expand
hipError_t launch_shrink_decode(const ShrinkParams &p, hipStream_t s);   // tiles of <= 16 rows
hipError_t launch_expand_decode(const ExpandParams &p, hipStream_t s);
hipError_t launch_fused_decode(const FusedParams &p, hipStream_t s);
hipError_t launch_combine(const CombineParams &p, hipStream_t s);
int combine_max_top_k();
hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s);      // bytes a multiple of 16

}  // namespace lora
