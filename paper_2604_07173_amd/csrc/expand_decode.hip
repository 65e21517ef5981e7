// Expand for decode batches (tiles of at most 16 rows): y[row] += scale * v[row] * B, with
// every wave working on its own, no LDS and no barriers.
//
// Work item (per wave) = (row tile, projection, slice of 128-column chunks).  Prologue: the
// wave adds the K parts of the tile's v in a fixed order, applies the adapter's scale and
// splits the result into bf16 hi + lo planes held in MFMA operand registers (hi = v
// truncated to bf16, lo = the rounded remainder, so the product sees about 16 mantissa bits
// of v).  Main loop over the slice's chunks, software-pipelined two deep (the first two
// chunks' loads are issued before v is fetched): while chunk c is
// multiplied and written back, the packed B tile and the base-output rows of chunk c+1 are
// already in flight (B with nontemporal loads: it is read once; y with ordinary accesses:
// read-modify-write runs faster through the L2).  All loads in the loop are unconditional and the loop is specialised
// on the number of row quads, so the code is straight-line and the hardware counters let
// the next chunk's loads stay outstanding across the current chunk's compute.
//
// Row placement: tile row r sits in MFMA row slot (r % 4) * 4 + r / 4, so result register i
// of lane group g is row 4*i + g.  A tile of n rows then needs only ceil(n / 4) y loads and
// stores per chunk, each with all four lane groups busy (16 lanes cover 256 contiguous
// bytes of a row), instead of four quarter-empty ones.  B is streamed exactly once per
// (tile, chunk); after the eight MFMAs of a chunk a lane owns eight consecutive output
// columns of each of its rows.
#include <type_traits>

#include "expand_common.h"
#include "lora_internal.h"

namespace lora {

namespace {

// OVW: the output rows are written, not updated: the base output counts as zero and is never
// read (used when the update goes to a buffer of its own rather than into base rows).
template <int R, bool F32, int NI, bool OVW>
struct ExpandWave {
    using Tile = ExpandTile<R>;
    static constexpr int KS = Tile::KS;
    static constexpr int NY = F32 ? 2 : 1;
    static constexpr int ESZ = F32 ? 4 : 2;

    struct YBuf {
        u32x4 r[NI][NY];
    };

    int lane, g, i16, h_out;
    const uint16_t *Bp;
    char *yrow[NI];          // y rows of result registers 0..NI-1 (a valid row even if unused)
    bool rok[NI];            // whether result register i belongs to a row of the tile
    typename Tile::A a;

    __device__ inline void load(int c, typename Tile::B &b, YBuf &y) const
    {
        Tile::template load_b<true>(Bp, c, lane, b);
        const int col = c * kColChunk + i16 * 8;
        const int colc = col < h_out ? col : 0;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int q = 0; q < NY; ++q)
                y.r[i][q] = OVW ? u32x4{0u, 0u, 0u, 0u} : ld16<false>(yrow[i] + (int64_t)colc * ESZ + 16 * q);
    }

    __device__ inline void compute_store(int c, const typename Tile::B &b, const YBuf &y) const
    {
        f32x4 acc[8];
        Tile::mma(a, b, acc);
        const int col = c * kColChunk + i16 * 8;
        const bool col_ok = col < h_out;
        // the sums are formed for every lane; only the store itself is predicated
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            char *yp = yrow[i] + (int64_t)col * ESZ;
            const bool ok = col_ok && rok[i];
            if (F32) {
                u32x4 o0, o1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    o0[q] = __float_as_uint(__uint_as_float(y.r[i][0][q]) + acc[q][i]);
                    o1[q] = __float_as_uint(__uint_as_float(y.r[i][NY - 1][q]) + acc[4 + q][i]);
                }
                if (ok) {
                    st16<false>(yp, o0);
                    st16<false>(yp + 16, o1);
                }
            } else {
                u32x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned u = y.r[i][0][q];
                    const float f0 = __uint_as_float(u << 16) + acc[2 * q][i];
                    const float f1 = __uint_as_float(u & 0xFFFF0000u) + acc[2 * q + 1][i];
                    o[q] = pack_bf16_rne(f0, f1);
                }
                if (ok) st16<false>(yp, o);
            }
        }
    }

    // chunks in flight (three or four for the small rank-8 chunks measured no faster)
    static constexpr int D = 2;

    struct Stage {
        typename Tile::B b;
        YBuf y;
    };

    // issue the loads of the first D chunks of [c0, c1) (a slice shorter than D repeats its
    // last chunk; the repeats are never used)
    __device__ inline void prefetch(int c0, int c1, Stage (&st)[D]) const
    {
#pragma unroll
        for (int k = 0; k < D; ++k) load(min(c0 + k, c1 - 1), st[k].b, st[k].y);
    }

    // chunks [c0, c1) after prefetch(): D in flight; every load in the loop body is
    // unconditional
    __device__ inline void run(int c0, int c1, Stage (&st)[D]) const
    {
        int c = c0;
        for (; c + D < c1; c += D) {
#pragma unroll
            for (int k = 0; k < D; ++k) {
                compute_store(c + k, st[k].b, st[k].y);
                load(min(c + k + D, c1 - 1), st[k].b, st[k].y);
            }
        }
#pragma unroll
        for (int k = 0; k < D; ++k)
            if (c + k < c1) compute_store(c + k, st[k].b, st[k].y);      // wave-uniform
    }
};

template <int R, bool F32, int NI, bool OVW>
__device__ inline void expand_item(const ExpandParams &p, const lora_tile &t, const Unit &unit, int pj,
                                   int c0, int c1, int lane)
{
    using Tile = ExpandTile<R>;
    constexpr int KS = Tile::KS, KV = Tile::KV, ESZ = F32 ? 4 : 2;
    ExpandWave<R, F32, NI, OVW> w;
    w.lane = lane;
    w.g = lane >> 4;
    w.i16 = lane & 15;
    w.h_out = p.h_out[pj];
    w.Bp = unit.B;
    const float scale = unit.scale;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int r = 4 * i + w.g;                       // row of result register i
        w.rok[i] = r < t.n_rows;
        const int dst = p.perm[t.row0 + min(r, t.n_rows - 1)];
        w.yrow[i] = static_cast<char *>(p.y[pj]) + (int64_t)dst * p.ldy[pj] * ESZ;
    }

    // the first chunks' weights and base output: in flight while v is fetched
    typename ExpandWave<R, F32, NI, OVW>::Stage st[ExpandWave<R, F32, NI, OVW>::D];
    w.prefetch(c0, c1, st);

    // v operand: this lane's row slot i16 holds tile row (i16 % 4) * 4 + i16 / 4
    {
        const int row = (w.i16 & 3) * 4 + (w.i16 >> 2);
        const bool valid = row < t.n_rows;
        const float *vrow = p.v[pj] + (int64_t)(t.row0 + (valid ? row : 0)) * R;
        const int64_t part_stride = (int64_t)p.P * R;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int jb = Tile::jbase(w.g, ks);
            float s[KV];
#pragma unroll
            for (int q = 0; q < KV; ++q) s[q] = 0.f;
            for (int part = 0; part < p.n_parts; ++part) {
#pragma unroll
                for (int h = 0; h < KV / 4; ++h) {
                    const f32x4 x = ld16f(vrow + part * part_stride + jb + 4 * h);
#pragma unroll
                    for (int q = 0; q < 4; ++q) s[4 * h + q] += x[q];
                }
            }
#pragma unroll
            for (int q = 0; q < KV; ++q) s[q] = valid ? s[q] * scale : 0.f;
            Tile::make_a(s, w.g, ks, w.a);
        }
    }
    w.run(c0, c1, st);
}

// tiles, units and counts are passed again as restrict-qualified kernel arguments: with a
// wave-uniform index the compiler then reads them through the scalar cache, which shortens
// the dependent chain tile -> unit -> first data load.
template <int R, bool F32, bool OVW>
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
        switch ((t.n_rows + 3) >> 2) {              // wave-uniform
        case 1: expand_item<R, F32, 1, OVW>(p, t, unit, pj, c0, c1, lane); break;
        case 2: expand_item<R, F32, 2, OVW>(p, t, unit, pj, c0, c1, lane); break;
        case 3: expand_item<R, F32, 3, OVW>(p, t, unit, pj, c0, c1, lane); break;
        default: expand_item<R, F32, 4, OVW>(p, t, unit, pj, c0, c1, lane); break;
        }
    }
}

template <int R>
hipError_t launch_r(const ExpandParams &p, hipStream_t s)
{
    const dim3 block(p.waves * 64);
    if (p.out_f32)
        hipLaunchKernelGGL((expand16_kernel<R, true, false>), dim3(p.grid), block, 0, s, p, p.tiles, p.units, p.counts);
    else if (p.overwrite)
        hipLaunchKernelGGL((expand16_kernel<R, false, true>), dim3(p.grid), block, 0, s, p, p.tiles, p.units, p.counts);
    else
        hipLaunchKernelGGL((expand16_kernel<R, false, false>), dim3(p.grid), block, 0, s, p, p.tiles, p.units, p.counts);
    return hipGetLastError();
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
