// Expand with fused scale-and-accumulate for batches with long segments (tiles of up to 32
// rows): y[row] += scale * v[row] * B
// (App. A.2.2 "expand phase"; Sec. 2.2: the update is added to the base output; Fig. 7b:
// final addition of the two outputs).
//
// With long segments the traffic is the read-modify-write of y; B is small and stays in the
// L2.  Two launches:
//
// 1. operand images: one wave per 16-row sub-tile adds the K parts of v in a fixed order,
//    applies the adapter's scale and writes the sub-tile's MFMA operand exactly as the lanes
//    of the second kernel want it: two bf16 planes hi + lo (hi = v truncated to bf16, lo =
//    the rounded remainder, so the product sees about 16 mantissa bits of v), 64 lanes x 8
//    or 16 bytes per plane and K step.  This is done once per sub-tile instead of once per
//    (sub-tile, column chunk).
//
// 2. the product: every wave works on its own, no LDS and no barriers.  Work item (per
//    wave) = (group of kLongGroup consecutive tiles, projection, 128-column chunk).  The
//    wave keeps the chunk's packed B in MFMA operand registers for as long as the tiles
//    belong to the same (adapter, expert) and walks over the group's 16-row sub-tiles,
//    software-pipelined three deep: while sub-tile q is multiplied and written back, the
//    operand image and the base-output rows of sub-tile q+1 are in flight, and the row
//    indices of sub-tile q+2 are being fetched.  All loads are unconditional (rows beyond a
//    tile re-read a valid row and are not stored), so the code is straight-line.
//
// The base-output rows are read and written with nontemporal accesses: every byte of y is touched
// once, and keeping it out of the caches leaves them to the B tiles and operand images that many
// waves share (prefill workload: 250 -> 229 us; in the decode kernel, where a tile's rows are few
// and B is the larger stream, the same change costs 5 %).
//
// Row placement as in the decode kernel: tile row r of a sub-tile sits in MFMA row slot
// (r % 4) * 4 + r / 4, so result register i of lane group g is row 4*i + g and each y
// access of a wave covers four rows x 256 contiguous bytes.
#include <type_traits>

#include "expand_common.h"
#include "lora_internal.h"

namespace lora {

namespace {

constexpr int kLongGroup = 4;        // tiles one wave item walks over (128 rows)

// vec elements of one sub-tile's operand image
template <int R>
__host__ __device__ constexpr int image_vecs()
{
    return ExpandTile<R>::KS * 2 * 64;
}

template <int R>
__global__ __launch_bounds__(256) void operand_image_kernel(ExpandParams p,
                                                            const lora_tile *__restrict__ tiles,
                                                            const Unit *__restrict__ units,
                                                            const int32_t *__restrict__ counts)
{
    using Tile = ExpandTile<R>;
    typedef typename Tile::vec vec;
    constexpr int KS = Tile::KS, KV = Tile::KV;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 4, i16 = lane & 15;
    const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wave), nw = gridDim.x * 4;
    const int n_slots = counts[2] * 2;                 // 16-row sub-tiles, two per tile
    const int64_t part_stride = (int64_t)p.P * R;

    for (int s = gw; s < n_slots * p.n_fused; s += nw) {
        const int pj = s / n_slots;
        const int slot = s - pj * n_slots;
        const lora_tile t = tiles[slot >> 1];
        const float scale = units[(int64_t)t.key * p.n_proj + p.proj0 + pj].scale;
        const int row = (slot & 1) * 16 + (i16 & 3) * 4 + (i16 >> 2);
        const bool valid = row < t.n_rows;
        const float *vrow = p.v[pj] + (int64_t)(t.row0 + (valid ? row : 0)) * R;
        LORA_GLOBAL vec *img = (LORA_GLOBAL vec *)p.img[pj] + (int64_t)slot * image_vecs<R>();
        typename Tile::A a;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int jb = Tile::jbase(g, ks);
            float sum[KV];
#pragma unroll
            for (int q = 0; q < KV; ++q) sum[q] = 0.f;
            for (int part = 0; part < p.n_parts; ++part) {
#pragma unroll
                for (int h = 0; h < KV / 4; ++h) {
                    const f32x4 x = ld16f(vrow + part * part_stride + jb + 4 * h);
#pragma unroll
                    for (int q = 0; q < 4; ++q) sum[4 * h + q] += x[q];
                }
            }
#pragma unroll
            for (int q = 0; q < KV; ++q) sum[q] = valid ? sum[q] * scale : 0.f;
            Tile::make_a(sum, g, ks, a);
            img[(ks * 2 + 0) * 64 + lane] = a.hi[ks];
            img[(ks * 2 + 1) * 64 + lane] = a.lo[ks];
        }
    }
}

template <int R, bool F32>
struct LongWave {
    using Tile = ExpandTile<R>;
    typedef typename Tile::vec vec;
    static constexpr int KS = Tile::KS;
    static constexpr int NY = F32 ? 2 : 1;
    static constexpr int ESZ = F32 ? 4 : 2;
    static constexpr int NSLOT = 2 * kLongGroup;

    struct Rows {                 // stage 1: where the sub-tile's rows live
        char *y[4];
        bool ok[4];
    };
    struct Data {                 // stage 2: the sub-tile's operand and base output
        typename Tile::A a;
        u32x4 y[4][NY];
    };

    int lane, g, i16;
    const int32_t *perm;
    char *ybase;                  // y + this lane's first column
    int64_t ld_bytes;
    bool col_ok;
    const LORA_GLOBAL vec *img;
    lora_tile tl[kLongGroup];
    int tix[kLongGroup];
    bool live[kLongGroup];

    __device__ inline void rows_of(int q, Rows &r) const
    {
        const int k = q >> 1, sub = q & 1;
        const int n = live[k] ? tl[k].n_rows : 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = sub * 16 + 4 * i + g;
            r.ok[i] = col_ok && row < n;
            const int dst = perm[tl[k].row0 + min(row, tl[k].n_rows - 1)];
            r.y[i] = ybase + (int64_t)dst * ld_bytes;
        }
    }

    __device__ inline void load(int q, const Rows &r, Data &d) const
    {
        const int k = q >> 1, sub = q & 1;
        const LORA_GLOBAL vec *im = img + (int64_t)(tix[k] * 2 + sub) * image_vecs<R>();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            d.a.hi[ks] = im[(ks * 2 + 0) * 64 + lane];
            d.a.lo[ks] = im[(ks * 2 + 1) * 64 + lane];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int h = 0; h < NY; ++h) d.y[i][h] = ld16<true>(r.y[i] + 16 * h);     // touched once: nontemporal
    }

    __device__ inline void compute_store(const Rows &r, const Data &d, const typename Tile::B &b) const
    {
        f32x4 acc[8];
        Tile::mma(d.a, b, acc);
        // the sums are formed for every lane; only the store itself is predicated
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (F32) {
                u32x4 o0, o1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    o0[q] = __float_as_uint(__uint_as_float(d.y[i][0][q]) + acc[q][i]);
                    o1[q] = __float_as_uint(__uint_as_float(d.y[i][NY - 1][q]) + acc[4 + q][i]);
                }
                if (r.ok[i]) {
                    st16<true>(r.y[i], o0);
                    st16<true>(r.y[i] + 16, o1);
                }
            } else {
                u32x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned u = d.y[i][0][q];
                    const float f0 = __uint_as_float(u << 16) + acc[2 * q][i];
                    const float f1 = __uint_as_float(u & 0xFFFF0000u) + acc[2 * q + 1][i];
                    o[q] = pack_bf16_rne(f0, f1);
                }
                if (r.ok[i]) st16<true>(r.y[i], o);
            }
        }
    }
};

template <int R, bool F32>
__global__ __launch_bounds__(256, 2) void expand_long_kernel(ExpandParams p,
                                                             const lora_tile *__restrict__ tiles,
                                                             const Unit *__restrict__ units,
                                                             const int32_t *__restrict__ counts)
{
    using Wave = LongWave<R, F32>;
    using Tile = ExpandTile<R>;
    constexpr int NSLOT = Wave::NSLOT;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gw = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + wave), nw = gridDim.x * 4;
    const int n_tiles = counts[2];
    const int n_groups = (n_tiles + kLongGroup - 1) / kLongGroup;
    const int per_group = p.slice0[p.n_fused];                    // chunks of all projections
    const int n_items = n_groups * per_group;

    for (int item = gw; item < n_items; item += nw) {
        const int tg = item / per_group;
        const int rem = item - tg * per_group;
        const int pj = (rem >= p.slice0[1] ? 1 : 0) + (p.n_fused > 2 && rem >= p.slice0[2] ? 1 : 0);
        const int chunk = rem - p.slice0[pj];

        Wave w;
        w.lane = lane;
        w.g = lane >> 4;
        w.i16 = lane & 15;
        w.perm = p.perm;
        const int col = chunk * kColChunk + w.i16 * 8;
        w.col_ok = col < p.h_out[pj];
        w.ybase = static_cast<char *>(p.y[pj]) + (int64_t)(w.col_ok ? col : 0) * Wave::ESZ;
        w.ld_bytes = p.ldy[pj] * Wave::ESZ;
        w.img = (const LORA_GLOBAL typename Wave::vec *)p.img[pj];
#pragma unroll
        for (int k = 0; k < kLongGroup; ++k) {
            w.live[k] = tg * kLongGroup + k < n_tiles;
            w.tix[k] = min(tg * kLongGroup + k, n_tiles - 1);
            w.tl[k] = tiles[w.tix[k]];
        }

        typename Tile::B b;
        int b_key = w.tl[0].key;
        Tile::template load_b<false>(units[(int64_t)b_key * p.n_proj + p.proj0 + pj].B, chunk, lane, b);

        typename Wave::Rows rows[3];
        typename Wave::Data data[2];
        w.rows_of(0, rows[0]);
        w.rows_of(1, rows[1]);
        w.load(0, rows[0], data[0]);
#pragma unroll
        for (int q = 0; q < NSLOT; ++q) {
            if (q + 2 < NSLOT) w.rows_of(q + 2, rows[(q + 2) % 3]);
            if (q + 1 < NSLOT) w.load(q + 1, rows[(q + 1) % 3], data[(q + 1) & 1]);
            const int key = w.tl[q >> 1].key;
            if (key != b_key) {                                   // wave-uniform, rare
                b_key = key;
                Tile::template load_b<false>(units[(int64_t)key * p.n_proj + p.proj0 + pj].B, chunk, lane, b);
            }
            w.compute_store(rows[q % 3], data[q & 1], b);
        }
    }
}

template <int R>
hipError_t launch_r(const ExpandParams &p, hipStream_t s)
{
    hipLaunchKernelGGL((operand_image_kernel<R>), dim3(p.image_grid), dim3(256), 0, s, p, p.tiles,
                       p.units, p.counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (p.out_f32)
        hipLaunchKernelGGL((expand_long_kernel<R, true>), dim3(p.grid), dim3(256), 0, s, p, p.tiles,
                           p.units, p.counts);
    else
        hipLaunchKernelGGL((expand_long_kernel<R, false>), dim3(p.grid), dim3(256), 0, s, p, p.tiles,
                           p.units, p.counts);
    return hipGetLastError();
}

}  // namespace

size_t expand_image_bytes(int rank, int64_t n_tiles)
{
    const int ks = rank >= 32 ? rank / 32 : 1;
    const size_t vec_bytes = rank <= 16 ? 8 : 16;
    return (size_t)n_tiles * 2 * ks * 2 * 64 * vec_bytes;
}

int expand_long_group() { return kLongGroup; }

hipError_t launch_expand(const ExpandParams &p, hipStream_t s)
{
    if (p.grid <= 0) return hipSuccess;
    switch (p.rank) {
    case 16: return launch_r<16>(p, s);       // rank 8 always runs with 16-row tiles
    case 32: return launch_r<32>(p, s);
    case 64: return launch_r<64>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lora
