// Shrink and expand of a small decode batch in one launch (Sec. 5.2 discusses scheduling the
// LoRA computation with few, persistent launches; a decode layer call is short enough for
// every dependent launch to show).  For tiles of at most 16 rows, short inputs and few tiles.
//
// Work item (per workgroup of four waves) = (row tile, projection, slice of 128-column chunks).
// The workgroup first computes the tile's whole v = gather(x) * A for its projection, the four
// waves splitting the K range and adding their sums through LDS in a fixed order; v stays in
// LDS.  Then every wave takes a run of the slice's chunks and does what a wave of the expand
// kernel does (scale, hi/lo split, multiply with B, add into the tile's output rows).
//
// The workgroups of one (tile, projection) all repeat the same shrink: A is fetched from HBM
// once and then served by the L2 to the other slices.  That trade is what makes one launch
// possible without any hand-off between workgroups: nobody waits for anybody, there is no
// intermediate in global memory, no counter, no fence, and the kernel cannot deadlock.  A
// workgroup walks through shrink and expand one after the other, so the launch is bound by the
// latency of that chain, not by bandwidth: it beats two launches (each with a latency floor of
// its own) only for batches of a few dozen tiles; the host decides (see fused_plan in api.hip).
//
// Sums are formed in a fixed order, so results are bit-identical run to run.  The K range is
// split over the waves differently from the two-launch path (which also splits it over
// workgroups), so the two paths agree to fp32 rounding, not bit for bit.
#include <type_traits>

#include "expand_item.h"
#include "segments_inline.h"
#include "shrink_wave.h"

namespace lora {

namespace {

constexpr int kFusedWaves = 4;      // waves of a workgroup (eight or sixteen measured no faster)

// BUILD: the segments are not there yet either; every workgroup sorts the batch for itself in LDS
// first (segments_inline.h), workgroup 0 writes the segments out, and the whole layer call of a
// small batch is this one launch.
template <int R, bool BUILD>
__global__ __launch_bounds__(64 * kFusedWaves) void fused16_kernel(FusedParams p,
                                                         const lora_tile *__restrict__ tiles,
                                                         const Unit *__restrict__ units,
                                                         const int32_t *__restrict__ counts)
{
    using Wave = ShrinkWave<R, 1, false>;
    constexpr int NACC = Wave::NACC, KU = Wave::KU;
    static_assert(64 * kFusedWaves == kInlineThreads, "the build is written for this workgroup size");
    union Scratch {                   // the build's counts are dead before the first sums are added
        f32x4 red[kFusedWaves][NACC][64];
        std::conditional_t<BUILD, InlineCounts, char> counts;
    };
    __shared__ Scratch scratch;
    __shared__ std::conditional_t<BUILD, InlineSegments, char> built;
    __shared__ __attribute__((aligned(16))) float vsh[kDecodeTileRows * R];
    auto &red = scratch.red;

    const ShrinkParams &sp = p.s;
    const ExpandParams &ep = p.e;
    const int tid = threadIdx.x, wave = tid >> 6;
    Wave w;
    w.lane = tid & 63;
    w.g = w.lane >> 4;
    w.i16 = w.lane & 15;
    w.h_in = sp.h_in;
    int n_tiles;
    const uint16_t *perm_lds = nullptr;
    if constexpr (BUILD) {
        build_segments_inline(sp.seg, scratch.counts, built, blockIdx.x == 0);   // `built` is complete behind its last barrier
        n_tiles = built.n_tiles;
        perm_lds = built.perm;
    } else {
        n_tiles = counts[2];
    }
    const int per_tile = ep.slice0[ep.n_fused];                  // workgroup items of one tile
    const int n_items = n_tiles * per_tile;
    const int kblocks = (sp.h_in + KU - 1) / KU;
    const int kb_per_wave = (((kblocks + kFusedWaves - 1) / kFusedWaves) + 3) & ~3;   // whole steps of the wave's loop

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile_ix = item / per_tile;
        const int rem = item - tile_ix * per_tile;
        const int pj = (rem >= ep.slice0[1] ? 1 : 0) + (ep.n_fused > 2 && rem >= ep.slice0[2] ? 1 : 0);
        const int slice = rem - ep.slice0[pj];
        lora_tile t;
        if constexpr (BUILD) t = built.tiles[tile_ix];
        else t = tiles[tile_ix];
        const Unit unit = units[(int64_t)t.key * sp.n_proj + sp.proj0 + pj];

        // ---- shrink: this tile, this projection, the whole K range over the four waves ----------
        w.Ap[0] = unit.A;
        w.row_ok = w.i16 < t.n_rows;
        {
            int s;
            if constexpr (BUILD) s = built.perm[t.row0 + min(w.i16, t.n_rows - 1)];
            else s = sp.perm[t.row0 + min(w.i16, t.n_rows - 1)];
            if (sp.src_row) s = sp.src_row[s];
            w.xp = sp.x + (int64_t)s * sp.ldx;
        }
        const int kb_begin = wave * kb_per_wave;
        w.run(kb_begin, min(kb_begin + kb_per_wave, kblocks));
#pragma unroll
        for (int a = 0; a < NACC; ++a) red[wave][a][w.lane] = w.acc[0][a];
        __syncthreads();
        // the four waves' sums in a fixed order -> v[row][j] in LDS
        constexpr int NOUT = (R == 8 ? 1 : NACC) * 64;
        for (int o = tid; o < NOUT; o += 64 * kFusedWaves) {
            const int l = o & 63;
            const int a = R == 8 ? 0 : o >> 6;
            const int row = l & 15;
            const int j = a * 16 + (l >> 4) * 4;
            if (j < R) {
                f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int k = 0; k < kFusedWaves; ++k) {
                    if (R == 8) s += red[k][0][l] + red[k][1][l + 32];
                    else s += red[k][a][l];
                }
                *reinterpret_cast<f32x4 *>(&vsh[row * R + j]) = s;
            }
        }
        __syncthreads();

        // ---- expand: the slice's chunks in four runs of even length, one per wave ----------------
        {
            const int cps = ep.cps[pj];
            const int s0 = slice * cps, s1 = min(s0 + cps, ep.n_chunks[pj]);
            const int per = ((((s1 - s0) + kFusedWaves - 1) / kFusedWaves) + 1) & ~1;
            const int c0 = s0 + wave * per, c1 = min(c0 + per, s1);
            if (c0 < c1) expand_tile_chunks<R, false, false>(ep, t, unit, pj, c0, c1, w.lane, vsh, perm_lds);
        }
        __syncthreads();              // vsh and red are reused by the next item
    }
}

template <int R>
hipError_t launch_r(const FusedParams &p, hipStream_t s)
{
    if (p.s.build) {
        if (p.s.seg.P > kInlineMaxRows || p.s.seg.n_adapters * (int64_t)p.s.seg.n_experts > kInlineMaxKeys)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL((fused16_kernel<R, true>), dim3(p.s.grid), dim3(64 * kFusedWaves), 0, s, p, p.s.tiles,
                           p.s.units, p.s.counts);
    } else {
        hipLaunchKernelGGL((fused16_kernel<R, false>), dim3(p.s.grid), dim3(64 * kFusedWaves), 0, s, p, p.s.tiles,
                           p.s.units, p.s.counts);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_fused_decode(const FusedParams &p, hipStream_t s)
{
    if (p.s.grid <= 0) return hipSuccess;
    switch (p.s.rank) {
    case 8: return launch_r<8>(p, s);
    case 16: return launch_r<16>(p, s);
    case 32: return launch_r<32>(p, s);
    case 64: return launch_r<64>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lora
