// Expand for decode batches (tiles of at most 16 rows): y[row] += scale * v[row] * B, with
// every wave working on its own, no LDS and no barriers.
//
// Work item (per wave) = (row tile, projection, slice of 128-column chunks).  Prologue: the
// wave adds the K parts of the tile's v in a fixed order, applies the adapter's scale and
// splits the result into bf16 hi + lo planes held in MFMA operand registers (hi = v
// truncated to bf16, lo = the rounded remainder, so the product sees about 16 mantissa bits
// of v).  Main loop over the slice's chunks, software-pipelined two deep: while chunk c is
// multiplied and written back, the packed B tile and the base-output rows of chunk c+1 are
// already in flight, so a wave always has loads outstanding.  B is streamed exactly once
// per (tile, chunk) with 16-byte loads, contiguous per wave; after the eight MFMAs of a
// chunk a lane owns eight consecutive output columns of four rows, so the read-modify-write
// of y is one 16-byte load and one 16-byte store per row and lane (16 lanes = 256
// contiguous bytes of a row).
#include "lora_device.h"
#include "lora_internal.h"

namespace lora {

namespace {

// eight fp32 values -> packed bf16 hi plane and lo plane
__device__ inline void split_hi_lo(const float (&s)[8], u32x4 &hi, u32x4 &lo)
{
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const unsigned h0 = __float_as_uint(s[2 * m]) & 0xFFFF0000u;
        const unsigned h1 = __float_as_uint(s[2 * m + 1]) & 0xFFFF0000u;
        hi[m] = (h0 >> 16) | h1;
        lo[m] = pack_bf16_rne(s[2 * m] - __uint_as_float(h0), s[2 * m + 1] - __uint_as_float(h1));
    }
}

template <int R, bool F32, bool NT>
struct ExpandWave {
    static constexpr int KS = R >= 32 ? R / 32 : 1;
    static constexpr int NY = F32 ? 2 : 1;

    const ExpandParams &p;
    int g, i16;
    const uint16_t *Bp;
    char *yrow[4];          // y rows of result registers 0..3 (a valid row even if unused)
    bool rok[4];            // whether result register i belongs to a row of the tile
    u32x4 a_hi[KS], a_lo[KS];

    __device__ ExpandWave(const ExpandParams &pp) : p(pp) {}

    // All loads are unconditional (rows beyond the tile read the tile's first row, columns
    // beyond h_out read column 0; neither is stored), which keeps the loop free of branches
    // so that the loads of the next chunk stay in flight while this one is computed.
    __device__ inline void load(int c, u32x4 (&b)[8][KS], u32x4 (&yv)[4][NY]) const
    {
#pragma unroll
        for (int blk = 0; blk < 8; ++blk)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                int64_t off;
                if (R >= 32) off = (((((int64_t)c * 8 + blk) * KS + ks) * 4 + g) * 16 + i16) * 8;
                else if (R == 16) off = ((((int64_t)c * 8 + blk) * 2 + (g & 1)) * 16 + i16) * 8;
                else off = (((int64_t)c * 8 + blk) * 16 + i16) * 8;
                b[blk][ks] = ld16<NT>(Bp + off);
            }
        const int col = c * kColChunk + i16 * 8;
        const int colc = col < p.h_out ? col : 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const char *yp = yrow[i] + (int64_t)colc * (F32 ? 4 : 2);
#pragma unroll
            for (int q = 0; q < NY; ++q) yv[i][q] = ld16<NT>(yp + 16 * q);
        }
    }

    __device__ inline void compute_store(int c, const u32x4 (&b)[8][KS], const u32x4 (&yv)[4][NY]) const
    {
        f32x4 acc[8];
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
            acc[blk] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                acc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    as_bf16x8(a_hi[ks]), as_bf16x8(b[blk][ks]), acc[blk], 0, 0, 0);
                if (R >= 32)
                    acc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        as_bf16x8(a_lo[ks]), as_bf16x8(b[blk][ks]), acc[blk], 0, 0, 0);
            }
        }
        const int col = c * kColChunk + i16 * 8;
        const bool col_ok = col < p.h_out;
        // the sums are formed for every lane; only the store itself is predicated
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            char *yp = yrow[i] + (int64_t)col * (F32 ? 4 : 2);
            const bool ok = col_ok && rok[i];
            if (F32) {
                u32x4 o0, o1;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    o0[q] = __float_as_uint(__uint_as_float(yv[i][0][q]) + acc[q][i]);
                    o1[q] = __float_as_uint(__uint_as_float(yv[i][NY - 1][q]) + acc[4 + q][i]);
                }
                if (ok) {
                    st16<NT>(yp, o0);
                    st16<NT>(yp + 16, o1);
                }
            } else {
                u32x4 o;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const unsigned u = yv[i][0][q];
                    const float f0 = __uint_as_float(u << 16) + acc[2 * q][i];
                    const float f1 = __uint_as_float(u & 0xFFFF0000u) + acc[2 * q + 1][i];
                    o[q] = pack_bf16_rne(f0, f1);
                }
                if (ok) st16<NT>(yp, o);
            }
        }
    }
};

template <int R, bool F32, bool NT>
__global__ __launch_bounds__(256) void expand16_kernel(ExpandParams p)
{
    constexpr int KS = R >= 32 ? R / 32 : 1;
    constexpr int NY = F32 ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wpb = blockDim.x >> 6;
    const int gw = blockIdx.x * wpb + wave, nw = gridDim.x * wpb;
    const int n_tiles = p.counts[2];
    const int per_tile = p.n_fused * p.n_slices;
    const int n_items = n_tiles * per_tile;
    const int cps = (p.n_chunks + p.n_slices - 1) / p.n_slices;   // chunks per slice

    ExpandWave<R, F32, NT> w(p);
    w.g = lane >> 4;
    w.i16 = lane & 15;

    for (int item = gw; item < n_items; item += nw) {
        const int tile_ix = item / per_tile;
        const int rem = item - tile_ix * per_tile;
        const int pj = rem / p.n_slices;
        const int slice = rem - pj * p.n_slices;
        const int c0 = slice * cps, c1 = min(c0 + cps, p.n_chunks);
        if (c0 >= c1) continue;
        const lora_tile t = p.tiles[tile_ix];
        const Unit *unit = p.units + ((int64_t)t.key * p.n_proj + p.proj0 + pj);
        w.Bp = unit->B;
        const float scale = unit->scale;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = w.g * 4 + i;
            w.rok[i] = r < t.n_rows;
            const int dst = p.perm[t.row0 + min(r, t.n_rows - 1)];
            w.yrow[i] = static_cast<char *>(p.y[pj]) + (int64_t)dst * p.ldy * (F32 ? 4 : 2);
        }

        // ---- v operand: sum of the K parts, scaled, as hi/lo bf16 planes ------------------
        {
            const bool valid = w.i16 < t.n_rows;
            const float *vrow = p.v[pj] + (int64_t)(t.row0 + w.i16) * R;
            const int64_t part_stride = (int64_t)p.P * R;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int jb = R >= 32 ? ks * 32 + w.g * 8 : (R == 16 ? (w.g & 1) * 8 : 0);
                float s[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) s[q] = 0.f;
                if (valid) {
                    for (int part = 0; part < p.n_parts; ++part) {
                        const f32x4 x0 = ld16f(vrow + part * part_stride + jb);
                        const f32x4 x1 = ld16f(vrow + part * part_stride + jb + 4);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            s[q] += x0[q];
                            s[4 + q] += x1[q];
                        }
                    }
#pragma unroll
                    for (int q = 0; q < 8; ++q) s[q] *= scale;
                }
                u32x4 hi, lo;
                split_hi_lo(s, hi, lo);
                const u32x4 zero4 = {0u, 0u, 0u, 0u};
                if (R >= 32) {
                    w.a_hi[ks] = hi;
                    w.a_lo[ks] = lo;
                } else if (R == 16) {
                    w.a_hi[ks] = w.g < 2 ? hi : lo;      // K = 32: hi of 16 entries, then lo
                    w.a_lo[ks] = zero4;
                } else {
                    w.a_hi[ks] = w.g == 0 ? hi : (w.g == 1 ? lo : zero4);   // hi, lo, zeros
                    w.a_lo[ks] = zero4;
                }
            }
        }

        // ---- chunks of the slice, two in flight ------------------------------------------
        // steady state: every load in the loop body is unconditional
        u32x4 b0[8][KS], y0[4][NY], b1[8][KS], y1[4][NY];
        w.load(c0, b0, y0);
        int c = c0;
        for (; c + 2 < c1; c += 2) {
            w.load(c + 1, b1, y1);
            w.compute_store(c, b0, y0);
            w.load(c + 2, b0, y0);
            w.compute_store(c + 1, b1, y1);
        }
        if (c + 1 < c1) {
            w.load(c + 1, b1, y1);
            w.compute_store(c, b0, y0);
            w.compute_store(c + 1, b1, y1);
        } else {
            w.compute_store(c, b0, y0);
        }
    }
}

template <int R, bool F32>
hipError_t launch_rf(const ExpandParams &p, hipStream_t s)
{
    const dim3 block(p.waves * 64);
    if (p.nontemporal)
        hipLaunchKernelGGL((expand16_kernel<R, F32, true>), dim3(p.grid), block, 0, s, p);
    else
        hipLaunchKernelGGL((expand16_kernel<R, F32, false>), dim3(p.grid), block, 0, s, p);
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const ExpandParams &p, hipStream_t s)
{
    return p.out_f32 ? launch_rf<R, true>(p, s) : launch_rf<R, false>(p, s);
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
