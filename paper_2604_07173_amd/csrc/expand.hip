// Expand with fused scale-and-accumulate: y[row] += scale * v[row] * B
// (App. A.2.2 "expand phase"; Sec. 2.2: the update is added to the base output; Fig. 7b:
// final addition of the two outputs).
//
// Work item = (row tile, projection, column slice).  The workgroup first adds the K parts
// of the tile's v in a fixed order, applies the adapter's scale, and stages the result in
// LDS as two bf16 planes hi + lo (hi = v truncated to bf16, lo = the rounded remainder), so
// the MFMA sees v to about 16 mantissa bits although its operands are bf16.  Then every
// wave walks over its 128-column chunks of the slice: it loads the chunk's packed B (16
// bytes per lane, contiguous per wave) into operand registers once, and for each 16-row
// sub-tile runs the MFMAs and read-modify-writes y.  The column permutation baked into the
// packed B leaves each lane with eight consecutive output columns of a row, so the y access
// is one 16-byte load and one 16-byte store per lane with 16 lanes covering 256 contiguous
// bytes of a row.  B is read exactly once per (tile, chunk).
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
    __shared__ __attribute__((aligned(16))) uint16_t v_hi[TR][LD];
    __shared__ __attribute__((aligned(16))) uint16_t v_lo[TR][LD];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, i16 = lane & 15;
    const int n_tiles = p.counts[2];
    const int per_tile = p.n_fused * p.n_slices;
    const int n_items = n_tiles * per_tile;
    const int groups = (p.n_chunks + p.waves - 1) / p.waves;        // chunk groups of a row
    const int groups_per_slice = (groups + p.n_slices - 1) / p.n_slices;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile_ix = item / per_tile;
        const int rem = item - tile_ix * per_tile;
        const int pj = rem / p.n_slices;
        const int slice = rem - pj * p.n_slices;
        const lora_tile t = p.tiles[tile_ix];
        const int nsub = (t.n_rows + 15) >> 4;
        const Unit unit = p.units[(int64_t)t.key * p.n_proj + p.proj0 + pj];
        const uint16_t *Bp = unit.B;
        const float *vsrc = p.v[pj];

        // ---- stage scale * sum_parts(v) as hi/lo bf16 planes -----------------------------
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
            float rem[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned u = __float_as_uint(s[q]) & 0xFFFF0000u;
                hi[q] = u >> 16;
                rem[q] = s[q] - __uint_as_float(u);
            }
            *reinterpret_cast<u32x2 *>(&v_hi[row][j]) = u32x2{hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16)};
            *reinterpret_cast<u32x2 *>(&v_lo[row][j]) = u32x2{pack_bf16_rne(rem[0], rem[1]), pack_bf16_rne(rem[2], rem[3])};
        }
        __syncthreads();

        // destination rows of this lane: MFMA result register i holds row 4*g + i
        int drow[SUB][4];
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int r = sub * 16 + g * 4 + i;
                drow[sub][i] = r < t.n_rows ? p.perm[t.row0 + r] : -1;
            }

        const int cg_end = min((slice + 1) * groups_per_slice, groups);
        for (int cg = slice * groups_per_slice; cg < cg_end; ++cg) {
            const int chunk = cg * p.waves + wave;
            if (chunk >= p.n_chunks) continue;                 // wave-uniform
            const int col = chunk * kColChunk + i16 * 8;       // first of this lane's 8 columns
            const bool col_ok = col < p.h_out;

            // packed B of the chunk -> operand registers
            typename Tile::B b;
            Tile::template load_b<false>(Bp, chunk, lane, b);

#pragma unroll
            for (int sub = 0; sub < SUB; ++sub) {
                if (sub >= nsub) break;
                // base output of this lane's rows (issued before the MFMAs)
                u32x4 yv[4][F32 ? 2 : 1];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool ok = col_ok && drow[sub][i] >= 0;
                    if (F32) {
                        const float *yp = static_cast<const float *>(p.y[pj]) + (int64_t)drow[sub][i] * p.ldy + col;
                        yv[i][0] = ok ? ld16<false>(yp) : zero4;
                        yv[i][F32 ? 1 : 0] = ok ? ld16<false>(yp + 4) : zero4;
                    } else {
                        const uint16_t *yp = static_cast<const uint16_t *>(p.y[pj]) + (int64_t)drow[sub][i] * p.ldy + col;
                        yv[i][0] = ok ? ld16<false>(yp) : zero4;
                    }
                }

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
                    if (!(col_ok && drow[sub][i] >= 0)) continue;
                    if (F32) {
                        float *yp = static_cast<float *>(p.y[pj]) + (int64_t)drow[sub][i] * p.ldy + col;
                        f32x4 o0, o1;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            o0[q] = __uint_as_float(yv[i][0][q]) + acc[q][i];
                            o1[q] = __uint_as_float(yv[i][F32 ? 1 : 0][q]) + acc[4 + q][i];
                        }
                        st16<false>(yp, __builtin_bit_cast(u32x4, o0));
                        st16<false>(yp + 4, __builtin_bit_cast(u32x4, o1));
                    } else {
                        uint16_t *yp = static_cast<uint16_t *>(p.y[pj]) + (int64_t)drow[sub][i] * p.ldy + col;
                        u32x4 o;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const unsigned u = yv[i][0][q];
                            const float f0 = __uint_as_float(u << 16) + acc[2 * q][i];
                            const float f1 = __uint_as_float(u & 0xFFFF0000u) + acc[2 * q + 1][i];
                            o[q] = pack_bf16_rne(f0, f1);
                        }
                        st16<false>(yp, o);
                    }
                }
            }
        }
        __syncthreads();
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
