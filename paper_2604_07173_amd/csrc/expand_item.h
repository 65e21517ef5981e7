// The wave-level work of the decode expand (tiles of at most 16 rows), shared by the expand
// kernel and the kernel that runs shrink and expand in one launch: one wave adds scale * v * B
// to the rows of one tile over a run of 128-column chunks.
//
// Prologue: the wave adds the K parts of the tile's v in a fixed order, applies the adapter's
// scale and splits the result into bf16 hi + lo planes held in MFMA operand registers (hi = v
// truncated to bf16, lo = the rounded remainder, so the product sees about 16 mantissa bits of
// v).  Main loop over the chunks, software-pipelined two deep (the first two chunks' loads are
// issued before v is fetched): while chunk c is multiplied and written back, the packed B tile
// and the base-output rows of chunk c+1 are already in flight (B with nontemporal loads: it is
// read once; y with ordinary accesses: read-modify-write runs faster through the L2).  All loads
// in the loop are unconditional and the loop is specialised on the number of row quads, so the
// code is straight-line and the hardware counters let the next chunk's loads stay outstanding
// across the current chunk's compute.
//
// Row placement: tile row r sits in MFMA row slot (r % 4) * 4 + r / 4, so result register i of
// lane group g is row 4*i + g.  A tile of n rows then needs only ceil(n / 4) y loads and stores
// per chunk, each with all four lane groups busy (16 lanes cover 256 contiguous bytes of a row),
// instead of four quarter-empty ones.  B is streamed exactly once per (tile, chunk); after the
// eight MFMAs of a chunk a lane owns eight consecutive output columns of each of its rows.
#pragma once
#include <type_traits>

#include "expand_common.h"
#include "lora_internal.h"

namespace lora {

// OVW: the output rows are written, not updated: the base output counts as zero and is never
// read (used when the update goes to a buffer of its own rather than into base rows).
// YNT: the output rows are read and written with the streaming hint (for callers whose outputs
// are not in a cache when the call starts, or are too large to be).
template <int R, bool F32, int NI, bool OVW, bool YNT = false>
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
                y.r[i][q] = OVW ? u32x4{0u, 0u, 0u, 0u} : ld16<YNT>(yrow[i] + (int64_t)colc * ESZ + 16 * q);
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
                    st16<YNT>(yp, o0);
                    st16<YNT>(yp + 16, o1);
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
                if (ok) st16<YNT>(yp, o);
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

// vlds: null = v comes from the K parts in global memory (p.v[pj]); otherwise the tile's summed v
// already sits in LDS as [16][R] floats (the kernel that runs shrink and expand in one launch).
// perm_lds: null = the sorted order comes from p.perm; otherwise from LDS (the kernel that also
// builds the segments).
template <int R, bool F32, int NI, bool OVW, bool YNT = false>
__device__ inline void expand_item(const ExpandParams &p, const lora_tile &t, const Unit &unit, int pj,
                                   int c0, int c1, int lane, const float *vlds = nullptr,
                                   const uint16_t *perm_lds = nullptr)
{
    using Tile = ExpandTile<R>;
    constexpr int KS = Tile::KS, KV = Tile::KV, ESZ = F32 ? 4 : 2;
    ExpandWave<R, F32, NI, OVW, YNT> w;
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
        const int at = t.row0 + min(r, t.n_rows - 1);
        const int dst = perm_lds ? (int)perm_lds[at] : p.perm[at];       // wave-uniform choice
        w.yrow[i] = static_cast<char *>(p.y[pj]) + (int64_t)dst * p.ldy[pj] * ESZ;
    }

    // v operand: this lane's row slot i16 holds tile row (i16 % 4) * 4 + i16 / 4.  The loads of
    // the K parts (PB at a time) are issued before anything is added, and before the first
    // chunks' weights and base output, so that the wait for v leaves those in flight; a part
    // beyond the last re-reads the last one and counts as zero.  The parts are added in
    // ascending order.
    constexpr int PB = R <= 32 ? 4 : (F32 ? 1 : 2);              // parts per batch of loads (registers permitting)
    const int row = (w.i16 & 3) * 4 + (w.i16 >> 2);
    const bool valid = row < t.n_rows;
    const float *vrow = p.v[pj] + (int64_t)(t.row0 + (valid ? row : 0)) * R;
    const int64_t part_stride = (int64_t)p.P * R;
    auto load_v = [&](int part0, f32x4 (&buf)[PB][KS][KV / 4]) {
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const float *src = vrow + min(part0 + u, p.n_parts - 1) * part_stride;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int h = 0; h < KV / 4; ++h) buf[u][ks][h] = ld16f(src + Tile::jbase(w.g, ks) + 4 * h);
        }
    };
    float s[KS][KV];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
        for (int q = 0; q < KV; ++q) s[ks][q] = 0.f;
    auto add_v = [&](int part0, const f32x4 (&buf)[PB][KS][KV / 4]) {
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const bool in = part0 + u < p.n_parts;             // wave-uniform
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int h = 0; h < KV / 4; ++h)
#pragma unroll
                    for (int q = 0; q < 4; ++q) s[ks][4 * h + q] += in ? buf[u][ks][h][q] : 0.f;
        }
    };
    typename ExpandWave<R, F32, NI, OVW, YNT>::Stage st[ExpandWave<R, F32, NI, OVW, YNT>::D];
    if (vlds) {                                                  // wave-uniform
        w.prefetch(c0, c1, st);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int h = 0; h < KV / 4; ++h) {
                const f32x4 x = *reinterpret_cast<const f32x4 *>(vlds + (valid ? row : 0) * R +
                                                                 Tile::jbase(w.g, ks) + 4 * h);
#pragma unroll
                for (int q = 0; q < 4; ++q) s[ks][4 * h + q] = x[q];
            }
    } else if (p.n_parts == 1) {                                 // a single part: one load, no batch
        f32x4 one[KS][KV / 4];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int h = 0; h < KV / 4; ++h) one[ks][h] = ld16f(vrow + Tile::jbase(w.g, ks) + 4 * h);
        w.prefetch(c0, c1, st);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int h = 0; h < KV / 4; ++h)
#pragma unroll
                for (int q = 0; q < 4; ++q) s[ks][4 * h + q] = one[ks][h][q];
    } else {
        f32x4 vbuf[PB][KS][KV / 4];
        load_v(0, vbuf);
        w.prefetch(c0, c1, st);                                  // the first chunks' weights and base output
        add_v(0, vbuf);
        for (int part0 = PB; part0 < p.n_parts; part0 += PB) {
            load_v(part0, vbuf);
            add_v(part0, vbuf);
        }
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        float sc[KV];
#pragma unroll
        for (int q = 0; q < KV; ++q) sc[q] = valid ? s[ks][q] * scale : 0.f;
        Tile::make_a(sc, w.g, ks, w.a);
    }
    w.run(c0, c1, st);
}

// one wave, one tile, chunks [c0, c1) of projection pj; the specialisation on the number of row
// quads is picked here (wave-uniform)
template <int R, bool F32, bool OVW, bool YNT = false>
__device__ inline void expand_tile_chunks(const ExpandParams &p, const lora_tile &t, const Unit &unit,
                                          int pj, int c0, int c1, int lane, const float *vlds = nullptr,
                                          const uint16_t *perm_lds = nullptr)
{
    switch ((t.n_rows + 3) >> 2) {
    case 1: expand_item<R, F32, 1, OVW, YNT>(p, t, unit, pj, c0, c1, lane, vlds, perm_lds); break;
    case 2: expand_item<R, F32, 2, OVW, YNT>(p, t, unit, pj, c0, c1, lane, vlds, perm_lds); break;
    case 3: expand_item<R, F32, 3, OVW, YNT>(p, t, unit, pj, c0, c1, lane, vlds, perm_lds); break;
    default: expand_item<R, F32, 4, OVW, YNT>(p, t, unit, pj, c0, c1, lane, vlds, perm_lds); break;
    }
}

}  // namespace lora
