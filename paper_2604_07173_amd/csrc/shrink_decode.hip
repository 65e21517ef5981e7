// Shrink for decode batches (tiles of at most 16 rows): v = gather(x) * A.
//
// Two ways of dealing out the work, chosen on the host:
//  * K split: work item = (row tile, K part); a workgroup of four waves takes one item, each
//    wave owns a quarter of the part's K range, and the four waves' sums are added through
//    LDS in a fixed order.  For batches with few tiles and long inputs.
//  * wave per tile: every wave takes a whole tile over the whole K range, no LDS, no barrier.
//    For batches with thousands of small tiles and short inputs (fine-grained MoE).
// In both a wave streams its slice of the packed A (and of the second fused projection's A)
// with 16-byte loads that are contiguous per wave, two steps in flight (the loads of step
// s+1 are issued before the MFMAs of step s; all loads are unconditional so the loop is
// branch-free and the hardware counters keep them outstanding), and multiplies it with the
// tile's gathered x rows.  The rank index sits on the M side of v_mfma_f32_16x16x32_bf16 and
// the rows on the N side, so a lane ends up with four consecutive rank entries of one row.
//
// Rank 8: a packed block holds 64 K values (two 32-deep halves side by side in the 16 M
// rows), is multiplied once with each half's x values, and rows 0..7 of the first product
// plus rows 8..15 of the second give the eight rank entries.
#include <type_traits>

#include "segments_inline.h"
#include "shrink_wave.h"

namespace lora {

namespace {

// tiles, units and counts are passed again as restrict-qualified kernel arguments: with a
// uniform index the compiler then reads them through the scalar cache, which shortens the
// dependent chain tile -> unit -> first data load.
//
// BUILD: the segments are not there yet; every workgroup sorts the batch for itself in LDS
// first (segments_inline.h) and takes tile records and row indices from there, and workgroup 0
// writes them out for the launches that follow.
//
// XNT: the x rows are loaded with the streaming hint (K-split form only).
// LINES: the x rows are fetched as whole cache lines and transposed through LDS (shrink_wave.h;
// K-split form, ranks 8 and 16).  Used together with XNT: a streamed line that is fetched in two
// halves by two instructions is fetched twice.  Measured on MI355X (rank 16, 14336 inputs): 4096
// rows of the Mixtral down projection 48.5 -> 41.7 us, of the Llama one 60.9 -> 51.0 us for the
// whole application; with inputs that stay cached (4096 wide, or few rows) it costs 5-10 %.
template <int R, int NPROJ, bool NT, bool WPT, bool BUILD = false, bool XNT = false, bool LINES = false>
__global__ __launch_bounds__(256, 2) void shrink16_kernel(ShrinkParams p,
                                                          const lora_tile *__restrict__ tiles,
                                                          const Unit *__restrict__ units,
                                                          const int32_t *__restrict__ counts)
{
    using Wave = ShrinkWave<R, NPROJ, NT, XNT, LINES>;
    constexpr int NACC = Wave::NACC, KU = Wave::KU;
    static_assert(!(BUILD && WPT), "the build needs the whole workgroup");
    static_assert(!(XNT && (BUILD || WPT)), "streamed x rows: K-split form without the build only");
    static_assert(!(LINES && WPT), "whole-line rows: K-split form only");
    union Scratch {                   // the build's counts are dead before the first sums are added
        f32x4 red[WPT ? 1 : 4][NPROJ][NACC][WPT ? 1 : 64];
        std::conditional_t<BUILD, InlineCounts, char> counts;
    };
    __shared__ Scratch scratch;
    __shared__ std::conditional_t<BUILD, InlineSegments, char> built;
    __shared__ u32x4 xt_all[LINES ? 4 * 256 : 1];      // LINES: 4 KiB per wave
    auto &red = scratch.red;

    const int tid = threadIdx.x, wave = tid >> 6;
    Wave w;
    w.lane = tid & 63;
    w.g = w.lane >> 4;
    w.i16 = w.lane & 15;
    w.h_in = p.h_in;
    w.xt = xt_all + (LINES ? wave * 256 : 0);
    int n_tiles;
    if constexpr (BUILD) {
        build_segments_inline(p.seg, scratch.counts, built, blockIdx.x == 0);   // `built` is complete behind its last barrier
        n_tiles = built.n_tiles;
    } else {
        n_tiles = counts[2];
    }
    const int n_items = n_tiles * p.n_parts;
    const int kblocks = (p.h_in + KU - 1) / KU;

    // item loop: a workgroup's item in the K-split form, a wave's item otherwise
    const int first = WPT ? __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wave) : blockIdx.x;
    const int stride = WPT ? gridDim.x * 4 : gridDim.x;
    for (int item = first; item < n_items; item += stride) {
        const int tile_ix = item / p.n_parts;
        const int part = item - tile_ix * p.n_parts;
        lora_tile t;
        if constexpr (BUILD) t = built.tiles[tile_ix];
        else t = tiles[tile_ix];
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
            w.Ap[pj] = units[(int64_t)t.key * p.n_proj + p.proj0 + pj].A;
        w.row_ok = w.i16 < t.n_rows;
        if constexpr (LINES) {
            int s[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int at = t.row0 + min(4 * q + w.g, t.n_rows - 1);
                if constexpr (BUILD) s[q] = built.perm[at];
                else s[q] = p.perm[at];
            }
            if (p.src_row) {
#pragma unroll
                for (int q = 0; q < 4; ++q) s[q] = p.src_row[s[q]];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) w.xq[q] = p.x + (int64_t)s[q] * p.ldx;
            w.xp = w.xq[0];
        } else {
            int s;
            if constexpr (BUILD) s = built.perm[t.row0 + min(w.i16, t.n_rows - 1)];
            else s = p.perm[t.row0 + min(w.i16, t.n_rows - 1)];
            if (p.src_row) s = p.src_row[s];
            w.xp = p.x + (int64_t)s * p.ldx;
        }
        const int part_begin = part * p.kb_per_part;
        const int part_end = min(part_begin + p.kb_per_part, kblocks);

        if constexpr (WPT) {
            w.run(part_begin, part_end);
            // lane (row i16, group g) holds rank entries 4g..4g+3 of its row; for rank 8 the
            // entries of groups 2,3 belong to the second half product and are added to the
            // first half's entries held 32 lanes below
#pragma unroll
            for (int pj = 0; pj < NPROJ; ++pj) {
                if (R == 8) {
                    f32x4 s = w.acc[pj][0];
#pragma unroll
                    for (int q = 0; q < 4; ++q) s[q] += __shfl_down(w.acc[pj][1][q], 32, 64);
                    if (w.row_ok && w.g < 2)
                        st16f(p.v[pj] + ((int64_t)part * p.P + t.row0 + w.i16) * R + w.g * 4, s);
                } else {
#pragma unroll
                    for (int nb = 0; nb < Wave::NB; ++nb)
                        if (w.row_ok)
                            st16f(p.v[pj] + ((int64_t)part * p.P + t.row0 + w.i16) * R + nb * 16 + w.g * 4,
                                  w.acc[pj][nb]);
                }
            }
        } else {
            // the four waves take the part's steps in turn, so that together they read a
            // contiguous kilobyte or more of every x row (and of A) at about the same time
            w.run(part_begin + wave * Wave::KB, part_end, 4 * Wave::KB);

            // add the four waves' sums in a fixed order and store this part of v
#pragma unroll
            for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                for (int a = 0; a < NACC; ++a) red[wave][pj][a][w.lane] = w.acc[pj][a];
            __syncthreads();
            constexpr int NOUT = NPROJ * (R == 8 ? 1 : NACC) * 64;
            for (int o = tid; o < NOUT; o += 256) {
                const int l = o & 63;
                const int a = R == 8 ? 0 : (o >> 6) % NACC;
                const int pj = R == 8 ? (o >> 6) : (o >> 6) / NACC;
                const int row = l & 15;
                const int j = a * 16 + (l >> 4) * 4;
                if (row < t.n_rows && j < R) {
                    f32x4 s;
                    if (R == 8) {
                        s = red[0][pj][0][l] + red[0][pj][1][l + 32];
                        s += red[1][pj][0][l] + red[1][pj][1][l + 32];
                        s += red[2][pj][0][l] + red[2][pj][1][l + 32];
                        s += red[3][pj][0][l] + red[3][pj][1][l + 32];
                    } else {
                        s = red[0][pj][a][l];
                        s += red[1][pj][a][l];
                        s += red[2][pj][a][l];
                        s += red[3][pj][a][l];
                    }
                    st16f(p.v[pj] + ((int64_t)part * p.P + t.row0 + row) * R + j, s);
                }
            }
            __syncthreads();
        }
    }
}

template <int R, int NPROJ>
hipError_t launch_rn(const ShrinkParams &p, hipStream_t s)
{
    if (p.build) {
        if (p.wave_per_tile || p.seg.P > kInlineMaxRows || p.seg.n_adapters * (int64_t)p.seg.n_experts > kInlineMaxKeys)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL((shrink16_kernel<R, NPROJ, true, false, true>), dim3(p.grid), dim3(256), 0, s, p,
                           p.tiles, p.units, p.counts);
    } else if (p.wave_per_tile)
        hipLaunchKernelGGL((shrink16_kernel<R, NPROJ, true, true>), dim3(p.grid), dim3(256), 0, s, p,
                           p.tiles, p.units, p.counts);
    else if (p.x_stream)       // large inputs that are read once: streamed, as whole lines where a step is 256 bytes of a row
        hipLaunchKernelGGL((shrink16_kernel<R, NPROJ, true, false, false, true, (R <= 16)>), dim3(p.grid), dim3(256), 0,
                           s, p, p.tiles, p.units, p.counts);
    else
        hipLaunchKernelGGL((shrink16_kernel<R, NPROJ, true, false>), dim3(p.grid), dim3(256), 0, s, p,
                           p.tiles, p.units, p.counts);
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const ShrinkParams &p, hipStream_t s)
{
    switch (p.n_fused) {
    case 1: return launch_rn<R, 1>(p, s);
    case 2: return launch_rn<R, 2>(p, s);
    case 3: return launch_rn<R, 3>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

int inline_build_max_rows() { return kInlineMaxRows; }
int inline_build_max_keys() { return kInlineMaxKeys; }

hipError_t launch_shrink_decode(const ShrinkParams &p, hipStream_t s)
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
