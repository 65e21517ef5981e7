// Expand for decode batches (tiles of at most 16 rows): y[row] += scale * v[row] * B, with
// every wave working on its own, no LDS and no barriers.
//
// Work item (per wave) = (row tile, projection, slice of 128-column chunks); what a wave does
// with an item is in expand_item.h.
#include "expand_item.h"

namespace lora {

namespace {

// tiles, units and counts are passed again as restrict-qualified kernel arguments: with a
// wave-uniform index the compiler then reads them through the scalar cache, which shortens
// the dependent chain tile -> unit -> first data load.
template <int R, bool F32, bool OVW, bool YNT>
__global__ __launch_bounds__(256, 2) void expand16_kernel(ExpandParams p,
                                                          const lora_tile *__restrict__ tiles,
                                                          const Unit *__restrict__ units,
                                                          const int32_t *__restrict__ counts)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wpb = blockDim.x >> 6;
    const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * wpb + wave), nw = gridDim.x * wpb;
    const int n_tiles = counts[2];
    const int per_tile = p.slice0[p.n_fused];                     // wave items of one tile
    // Item order: tile_group consecutive items take the same (projection, slice) of
    // tile_group consecutive tiles, so the waves of a workgroup that work on tiles of one
    // segment ask for the same B chunk at about the same time and all but one are served by
    // the L2.  tile_group 1: consecutive items are the slices of one tile.
    const int G = p.tile_group;
    const int n_items = (n_tiles + G - 1) / G * G * per_tile;

    for (int item = gw; item < n_items; item += nw) {
        const int grp = item / (per_tile * G);
        const int in_grp = item - grp * (per_tile * G);
        const int rem = in_grp / G;
        const int tile_ix = grp * G + (in_grp - rem * G);
        if (tile_ix >= n_tiles) continue;
        const int pj = (rem >= p.slice0[1] ? 1 : 0) + (p.n_fused > 2 && rem >= p.slice0[2] ? 1 : 0);
        const int slice = rem - p.slice0[pj];
        const int cps = p.cps[pj];                                // chunks per slice
        const int c0 = slice * cps, c1 = min(c0 + cps, p.n_chunks[pj]);
        if (c0 >= c1) continue;
        const lora_tile t = tiles[tile_ix];
        const Unit unit = units[(int64_t)t.key * p.n_proj + p.proj0 + pj];
        expand_tile_chunks<R, F32, OVW, YNT>(p, t, unit, pj, c0, c1, lane);
    }
}

template <int R, bool YNT>
hipError_t launch_ry(const ExpandParams &p, hipStream_t s)
{
    const dim3 block(p.waves * 64);
    if (p.out_f32)
        hipLaunchKernelGGL((expand16_kernel<R, true, false, YNT>), dim3(p.grid), block, 0, s, p, p.tiles, p.units, p.counts);
    else if (p.overwrite)
        hipLaunchKernelGGL((expand16_kernel<R, false, true, YNT>), dim3(p.grid), block, 0, s, p, p.tiles, p.units, p.counts);
    else
        hipLaunchKernelGGL((expand16_kernel<R, false, false, YNT>), dim3(p.grid), block, 0, s, p, p.tiles, p.units, p.counts);
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const ExpandParams &p, hipStream_t s)
{
    return p.y_stream ? launch_ry<R, true>(p, s) : launch_ry<R, false>(p, s);
}

}  // namespace

hipError_t launch_expand_decode(const ExpandParams &p, hipStream_t s)
{
    if (p.grid <= 0) return hipSuccess;
    switch (p.rank) {
    case 8: return launch_r<8>(p, s);
    case 16: return launch_r<16>(p, s);
    case 32: return launch_r<32>(p, s);
    case 64: return launch_r<64>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lora
