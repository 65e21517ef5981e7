// Segment build inside the first kernel that consumes the segments (App. A.2.2: rows that share
// an adapter are aggregated before shrink and expand; Sec. 5.2: few launches per layer call).
//
// For small decode batches the stand-alone builder is one short kernel whose time is mostly the
// latency of a launch, and the shrink that follows cannot start before it ends.  Here every
// workgroup of the shrink sorts the whole batch for itself in LDS before its first work item:
// the same stable counting sort (key = adapter * E + expert ascending, original order inside a
// key, rows without adapter left out), the same segment records and tiles, bit for bit.  The
// sort is repeated by every workgroup, which costs each about as much as the dependent loads
// of tile records and row indices it replaces; nobody waits for anybody.  Workgroup 0 also
// writes the result to the caller's lora_segments for the launches that follow.
//
// Limits: kInlineMaxRows rows, kInlineMaxKeys keys, tiles of kDecodeTileRows rows, workgroups
// of kInlineThreads threads.
//
// Stability without order-defining atomics: the batch is cut into groups of 64 consecutive
// rows, one wave handles a group at a time and ranks equal keys inside it by lane order (ballot
// match); counts[group][key] is written by the group's first lane of that key.  Thread k then
// turns its key's counts into exclusive sums over the groups in order, a workgroup scan over
// the keys gives every key its start, and a row's position is
//   start of its key + rows of the key in earlier groups + lanes below it in its group.
#pragma once
#include "lora_device.h"
#include "segments_common.h"

namespace lora {

constexpr int kInlineMaxRows = 2048;
constexpr int kInlineMaxKeys = 256;
constexpr int kInlineThreads = 256;
constexpr int kInlineWaves = kInlineThreads / 64;
constexpr int kInlineGroups = kInlineMaxRows / 64;
constexpr int kInlineGroupsPerWave = kInlineGroups / kInlineWaves;
constexpr int kInlineMaxTiles = kInlineMaxRows / kDecodeTileRows + kInlineMaxKeys;
static_assert(kInlineMaxKeys == kInlineThreads, "one key per thread");

typedef uint16_t InlineCounts[kInlineGroups][kInlineMaxKeys];     // 16 KiB, free again after the build

struct InlineSegments {                 // lives in LDS for the whole kernel
    uint16_t perm[kInlineMaxRows];
    lora_tile tiles[kInlineMaxTiles];
    unsigned key_start[kInlineMaxKeys];
    unsigned wave_sums[kInlineWaves][3];
    unsigned status;
    int n_tiles;
};

// GPW: groups of 64 rows per wave that the code is unrolled for (batches of up to 256 * GPW rows)
template <int GPW>
__device__ inline void build_segments_inline_n(const SegParams &sp, InlineCounts &counts, InlineSegments &L,
                                               bool write_global)
{
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int P = sp.P;
    constexpr int G = GPW * kInlineWaves;               // groups looked at; those beyond the batch are empty

    // ids of this wave's groups (wave w takes groups w, w + 4, ...): all loads first
    int a[GPW], e[GPW];
#pragma unroll
    for (int u = 0; u < GPW; ++u) {
        const int row = (w + kInlineWaves * u) * 64 + lane;
        const int r = min(row, P - 1);                      // unconditional loads (P >= 1), then selects
        a[u] = sp.adapter_id[r];
        e[u] = sp.expert_id ? sp.expert_id[r] : 0;
        if (row >= P) a[u] = -1;
    }
    {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        u32x4 *c4 = reinterpret_cast<u32x4 *>(&counts[0][0]);
        for (int i = tid; i < G * (kInlineMaxKeys * 2 / 16); i += kInlineThreads) c4[i] = zero;
        if (tid == 0) L.status = 0;
    }
    __syncthreads();

    // equal keys inside each group, all of the wave's groups bit by bit together (the groups'
    // chains of ballots are independent, so they overlap)
    unsigned key[GPW], below[GPW];
    unsigned bad = 0;
    Match m[GPW];
#pragma unroll
    for (int u = 0; u < GPW; ++u) {
        key[u] = row_key(sp, a[u], e[u], bad);
        const unsigned long long v = __ballot(key[u] != kNoKey);
        m[u].lo = (unsigned)v;
        m[u].hi = (unsigned)(v >> 32);
    }
#pragma unroll 1
    for (int b = 0; b < sp.key_bits; ++b) {
#pragma unroll
        for (int u = 0; u < GPW; ++u) {
            const unsigned bit = (key[u] >> b) & 1u;         // kNoKey lanes are in no mask anyway
            const unsigned long long bal = __ballot(key[u] != kNoKey && bit);
            const unsigned same = 0u - bit;
            m[u].lo &= ~((unsigned)bal ^ same);
            m[u].hi &= ~((unsigned)(bal >> 32) ^ same);
        }
    }
#pragma unroll
    for (int u = 0; u < GPW; ++u) {
        const int g = w + kInlineWaves * u;                 // wave-uniform
        below[u] = lanes_below(m[u]);
        if (key[u] != kNoKey && below[u] == 0) counts[g][key[u]] = (uint16_t)(__popc(m[u].lo) + __popc(m[u].hi));
    }
    if (bad) atomicOr(&L.status, bad);                      // OR is order-independent
    __syncthreads();

    // thread k: counts of key k per group -> rows of the key in earlier groups; its total
    unsigned total = 0;
    {
        unsigned c[G];
#pragma unroll
        for (int g = 0; g < G; ++g) c[g] = counts[g][tid];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            counts[g][tid] = (uint16_t)total;
            total += c[g];
        }
    }
    const unsigned my_tiles = (total + kDecodeTileRows - 1) / kDecodeTileRows;
    const unsigned occ = total ? 1u : 0u;
    const unsigned ir = wave_incl_sum(total), is = wave_incl_sum(occ), it = wave_incl_sum(my_tiles);
    if (lane == 63) {
        L.wave_sums[w][0] = ir;
        L.wave_sums[w][1] = is;
        L.wave_sums[w][2] = it;
    }
    __syncthreads();
    unsigned row0 = ir - total, seg = is - occ, tile0 = it - my_tiles, P_act = 0, S = 0, n_tiles = 0;
#pragma unroll
    for (int k = 0; k < kInlineWaves; ++k) {
        const unsigned r = L.wave_sums[k][0], s = L.wave_sums[k][1], t = L.wave_sums[k][2];
        P_act += r;
        S += s;
        n_tiles += t;
        row0 += k < w ? r : 0u;
        seg += k < w ? s : 0u;
        tile0 += k < w ? t : 0u;
    }
    L.key_start[tid] = row0;
    if (tid == 0) L.n_tiles = (int)n_tiles;
    // tiles and segment record of my key
    for (unsigned j = 0; j < my_tiles; ++j) {
        lora_tile t;
        t.key = tid;
        t.row0 = (int32_t)(row0 + j * kDecodeTileRows);
        t.n_rows = (int32_t)min((unsigned)kDecodeTileRows, total - j * kDecodeTileRows);
        t.seg = (int32_t)seg;
        L.tiles[tile0 + j] = t;
    }
    if (write_global && total) {
        sp.seg_start[seg] = (int32_t)row0;
        sp.seg_key[seg] = tid;
    }
    __syncthreads();

    // rows to their positions
#pragma unroll
    for (int u = 0; u < GPW; ++u) {
        const int g = w + kInlineWaves * u;
        if (key[u] != kNoKey)
            L.perm[L.key_start[key[u]] + counts[g][key[u]] + below[u]] = (uint16_t)(g * 64 + lane);
    }
    __syncthreads();

    if (write_global) {
        for (unsigned i = tid; i < P_act; i += kInlineThreads) sp.perm[i] = (int32_t)L.perm[i];
        for (unsigned i = tid; i < n_tiles; i += kInlineThreads) sp.tiles[i] = L.tiles[i];
        if (tid == 0) {
            sp.seg_start[S] = (int32_t)P_act;
            sp.counts[0] = (int32_t)S;
            sp.counts[1] = (int32_t)P_act;
            sp.counts[2] = (int32_t)n_tiles;
            sp.counts[3] = 0;
            sp.status[0] = L.status;
        }
    }
}

__device__ inline void build_segments_inline(const SegParams &sp, InlineCounts &counts, InlineSegments &L,
                                             bool write_global)
{
    if (sp.P <= 256) build_segments_inline_n<1>(sp, counts, L, write_global);
    else if (sp.P <= 512) build_segments_inline_n<2>(sp, counts, L, write_global);
    else if (sp.P <= 1024) build_segments_inline_n<4>(sp, counts, L, write_global);
    else build_segments_inline_n<kInlineGroupsPerWave>(sp, counts, L, write_global);
}

}  // namespace lora
