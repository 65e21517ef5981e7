// Expand with fused scale-and-accumulate for batches with long segments (tiles of up to 32
// rows): y[row] += scale * v[row] * B
// (App. A.2.2 "expand phase"; Sec. 2.2: the update is added to the base output; Fig. 7b:
// final addition of the two outputs).
//
// Work item = (group of consecutive row tiles, projection, group of 128-column chunks).
// Every wave of the workgroup owns one chunk of the chunk group and keeps that chunk's packed
// B in MFMA operand registers for as long as the tiles it walks over belong to the same
// (adapter, expert): with the long segments of a prefill batch B is read once per tile
// group instead of once per tile, and the kernel's traffic is the read-modify-write of y.
// Per tile the workgroup adds the K parts of v in a fixed order, applies the adapter's
// scale, and stages the result in LDS as two bf16 planes hi + lo (hi = v truncated to bf16,
// lo = the rounded remainder), so the MFMA sees v to about 16 mantissa bits although its
// operands are bf16.  The column permutation baked into the packed B leaves each lane with
// eight consecutive output columns of a row, so the y access is one 16-byte load and one
// 16-byte store per lane with 16 lanes covering 256 contiguous bytes of a row.
#include <type_traits>

#include "expand_common.h"
#include "lora_internal.h"

namespace lora {

namespace {

template <int R, bool F32>
__global__ __launch_bounds__(256, 2) void expand_kernel(ExpandParams p)
{
    using Tile = ExpandTile<R>;
    constexpr int KS = Tile::KS;                  // MFMA K steps over the rank
    constexpr int TR = kTileRows;
    constexpr int SUB = TR / 16;
    constexpr int LD = R + 8;                     // padded LDS row (bf16 elements)
    constexpr int ESZ = F32 ? 4 : 2;
    __shared__ __attribute__((aligned(16))) uint16_t v_hi[TR][LD];
    __shared__ __attribute__((aligned(16))) uint16_t v_lo[TR][LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, i16 = lane & 15;
    const int n_tiles = p.counts[2];
    const int n_chunks = p.n_chunks[0], h_out = p.h_out[0];          // equal for all projections here
    const int cgroups = (n_chunks + p.waves - 1) / p.waves;         // chunk groups of a row
    const int tgroups = (n_tiles + p.tile_group - 1) / p.tile_group;
    const int per_tgroup = p.n_fused * cgroups;
    const int n_items = tgroups * per_tgroup;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tg = item / per_tgroup;
        const int rem = item - tg * per_tgroup;
        const int pj = rem / cgroups;
        const int cg = rem - pj * cgroups;
        const int chunk = cg * p.waves + wave;
        const bool chunk_ok = chunk < n_chunks;                    // wave-uniform
        const int col = chunk * kColChunk + i16 * 8;               // first of this lane's 8 columns
        const bool col_ok = chunk_ok && col < h_out;
        const float *vsrc = p.v[pj];
        char *ybase = static_cast<char *>(p.y[pj]);

        typename Tile::B b;
        int b_key = -1;                                            // key whose B is in registers

        const int t_end = min((tg + 1) * p.tile_group, n_tiles);
        for (int ti = tg * p.tile_group; ti < t_end; ++ti) {
            const lora_tile t = p.tiles[ti];
            const Unit unit = p.units[(int64_t)t.key * p.n_proj + p.proj0 + pj];

            // destination rows of this lane (issued before the staging so that their latency
            // overlaps with it)
            char *yrow[SUB][4];
            bool rok[SUB][4];
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = sub * 16 + g * 4 + i;
                    rok[sub][i] = col_ok && r < t.n_rows;
                    const int dst = p.perm[t.row0 + min(r, t.n_rows - 1)];
                    yrow[sub][i] = ybase + ((int64_t)dst * p.ldy[pj] + (col_ok ? col : 0)) * ESZ;
                }

            // ---- stage scale * sum_parts(v) as hi/lo bf16 planes -------------------------
            for (int o = tid; o < TR * (R / 4); o += blockDim.x) {
                const int row = o / (R / 4);
                const int j = (o - row * (R / 4)) * 4;
                f32x4 s = {0.f, 0.f, 0.f, 0.f};
                if (row < t.n_rows) {
                    const float *src = vsrc + ((int64_t)(t.row0 + row)) * R + j;
                    for (int part = 0; part < p.n_parts; ++part)
                        s += ld16f(src + (int64_t)part * p.P * R);
                    s *= unit.scale;
                }
                unsigned hi[4];
                float lo[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned u = __float_as_uint(s[q]) & 0xFFFF0000u;
                    hi[q] = u >> 16;
                    lo[q] = s[q] - __uint_as_float(u);
                }
                *reinterpret_cast<u32x2 *>(&v_hi[row][j]) =
                    u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
                *reinterpret_cast<u32x2 *>(&v_lo[row][j]) =
                    u32x2{pack_bf16_rne(lo[0], lo[1]), pack_bf16_rne(lo[2], lo[3])};
            }
            __syncthreads();

            if (chunk_ok) {
                if (t.key != b_key) {                              // wave-uniform
                    Tile::template load_b<false>(unit.B, chunk, lane, b);
                    b_key = t.key;
                }
                // base output of both sub-tiles first, so that all of the tile's y is in flight
                // at once: MFMA result register i of sub-tile s holds row 16*s + 4*g + i; rows
                // beyond the tile read the tile's first row and are not stored
                u32x4 yv[SUB][4][F32 ? 2 : 1];
#pragma unroll
                for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                        for (int q = 0; q < (F32 ? 2 : 1); ++q) yv[sub][i][q] = ld16<false>(yrow[sub][i] + 16 * q);

#pragma unroll
                for (int sub = 0; sub < SUB; ++sub) {
                    // v operand of the sub-tile: row i16, this lane group's K values
                    const int row = sub * 16 + i16;
                    typename Tile::A a;
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        const int jb = Tile::jbase(g, ks);
                        typedef typename Tile::vec vec;
                        const vec vh = *reinterpret_cast<const vec *>(&v_hi[row][jb]);
                        const vec vl = *reinterpret_cast<const vec *>(&v_lo[row][jb]);
                        a.hi[ks] = (R == 8 && g >= 2) ? vl : vh;
                        a.lo[ks] = vl;
                    }
                    f32x4 acc[8];
                    Tile::mma(a, b, acc);

                    // y += delta: lane owns columns col .. col+7 of rows 4*g + i
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (F32) {
                            u32x4 o0, o1;
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                o0[q] = __float_as_uint(__uint_as_float(yv[sub][i][0][q]) + acc[q][i]);
                                o1[q] = __float_as_uint(__uint_as_float(yv[sub][i][F32 ? 1 : 0][q]) + acc[4 + q][i]);
                            }
                            if (rok[sub][i]) {
                                st16<false>(yrow[sub][i], o0);
                                st16<false>(yrow[sub][i] + 16, o1);
                            }
                        } else {
                            u32x4 o;
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                const unsigned u = yv[sub][i][0][q];
                                const float f0 = __uint_as_float(u << 16) + acc[2 * q][i];
                                const float f1 = __uint_as_float(u & 0xFFFF0000u) + acc[2 * q + 1][i];
                                o[q] = pack_bf16_rne(f0, f1);
                            }
                            if (rok[sub][i]) st16<false>(yrow[sub][i], o);
                        }
                    }
                }
            }
            __syncthreads();
        }
    }
}

template <int R>
hipError_t launch_r(const ExpandParams &p, hipStream_t s)
{
    const dim3 block(p.waves * 64);
    if (p.out_f32)
        hipLaunchKernelGGL((expand_kernel<R, true>), dim3(p.grid), block, 0, s, p);
    else
        hipLaunchKernelGGL((expand_kernel<R, false>), dim3(p.grid), block, 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_expand(const ExpandParams &p, hipStream_t s)
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
