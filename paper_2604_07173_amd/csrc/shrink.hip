// Shrink: v = gather(x) * A for every row tile (App. A.2.2 "shrink phase"; Sec. 2.2 x A).
//
// Work item = (row tile of one segment, K part).  A workgroup of four waves takes one item;
// each wave owns a quarter of the part's K range, streams that slice of the packed A once
// (one 16-byte load per lane = one contiguous 1 KiB per wave) straight into MFMA operand
// registers and multiplies it with up to 32 gathered x rows.  The rank index sits on the M
// side of v_mfma_f32_16x16x32_bf16 and the rows on the N side, so a lane ends up with four
// consecutive rank entries of one row.  The four waves' partial sums are added through LDS
// in a fixed order and stored as this part's slice of v; lora_expand adds the parts, again
// in a fixed order, so results are bit-identical run to run.
//
// Ranks 16, 32 and 64; rank-8 pools always use the 16-row-tile kernels.
//
// With two fused projections (the MoE gate and up matrices) the gathered x operand is
// loaded once and used for both.
#include "lora_device.h"
#include "lora_internal.h"

namespace lora {

namespace {

template <int R, int NPROJ>
__global__ __launch_bounds__(256, 2) void shrink_kernel(ShrinkParams p)
{
    constexpr int NB = R / 16;                            // 16-wide blocks of the rank index
    constexpr int KB = R == 16 ? 8 : (R == 32 ? 4 : 2);   // K blocks loaded per step
    constexpr int SUB = kTileRows / 16;                   // 16-row sub-tiles per tile
    __shared__ f32x4 red[4][NPROJ][SUB][NB][64];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, i16 = lane & 15;
    const int n_tiles = p.counts[2];
    const int n_items = n_tiles * p.n_parts;
    const int kblocks = (p.h_in + kKBlock - 1) / kKBlock;
    const int kb_per_wave = (p.kb_per_part + 3) >> 2;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile_ix = item / p.n_parts;
        const int part = item - tile_ix * p.n_parts;
        const lora_tile t = p.tiles[tile_ix];
        const int nsub = (t.n_rows + 15) >> 4;

        const uint16_t *Ap[NPROJ];
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
            Ap[pj] = p.units[(int64_t)t.key * p.n_proj + p.proj0 + pj].A;

        // gathered input rows: lane (i16, g) reads x[row i16 of the sub-tile][8*g ...]
        const uint16_t *xp[SUB];
        bool rv[SUB];
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub) {
            const int r = sub * 16 + i16;
            rv[sub] = r < t.n_rows;
            xp[sub] = p.x;
            if (rv[sub]) {
                int s = p.perm[t.row0 + r];
                if (p.src_row) s = p.src_row[s];
                xp[sub] = p.x + (int64_t)s * p.ldx + g * 8;
            }
        }

        const int part_end = min((part + 1) * p.kb_per_part, kblocks);
        const int kb_begin = part * p.kb_per_part + wave * kb_per_wave;
        const int kb_end = min(kb_begin + kb_per_wave, part_end);

        f32x4 acc[NPROJ][SUB][NB];
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) acc[pj][sub][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

        for (int kb0 = kb_begin; kb0 < kb_end; kb0 += KB) {
            u32x4 w[NPROJ][KB][NB];
            u32x4 xv[SUB][KB];
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const int kb = kb0 + u;
                const bool k_ok = kb < kb_end;
#pragma unroll
                for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        w[pj][u][nb] = zero4;
                        if (k_ok)
                            w[pj][u][nb] = ld16<false>(
                                Ap[pj] + (((int64_t)kb * NB + nb) * 64 + lane) * 8);
                    }
                const bool c_ok = k_ok && (kb * kKBlock + g * 8 < p.h_in);
#pragma unroll
                for (int sub = 0; sub < SUB; ++sub) {
                    xv[sub][u] = zero4;
                    if (c_ok && rv[sub])
                        xv[sub][u] = ld16<false>(xp[sub] + kb * kKBlock);
                }
            }
#pragma unroll
            for (int u = 0; u < KB; ++u)
#pragma unroll
                for (int sub = 0; sub < SUB; ++sub) {
                    if (sub < nsub) {
#pragma unroll
                        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
                                acc[pj][sub][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    as_bf16x8(w[pj][u][nb]), as_bf16x8(xv[sub][u]),
                                    acc[pj][sub][nb], 0, 0, 0);
                    }
                }
        }

        // add the four waves' partial sums in a fixed order and store this part of v
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) red[wave][pj][sub][nb][lane] = acc[pj][sub][nb];
        __syncthreads();
        constexpr int NOUT = NPROJ * SUB * NB * 64;
        for (int o = tid; o < NOUT; o += 256) {
            const int l = o & 63;
            int rest = o >> 6;
            const int nb = rest % NB;
            rest /= NB;
            const int sub = rest % SUB;
            const int pj = rest / SUB;
            const int row = sub * 16 + (l & 15);
            const int j = nb * 16 + (l >> 4) * 4;
            if (row < t.n_rows && j < R) {
                f32x4 s = red[0][pj][sub][nb][l];
                s += red[1][pj][sub][nb][l];
                s += red[2][pj][sub][nb][l];
                s += red[3][pj][sub][nb][l];
                float *dst = p.v[pj] + ((int64_t)part * p.P + t.row0 + row) * R + j;
                st16f(dst, s);
            }
        }
        __syncthreads();
    }
}

template <int R>
hipError_t launch_r(const ShrinkParams &p, hipStream_t s)
{
    if (p.n_fused == 2)
        hipLaunchKernelGGL((shrink_kernel<R, 2>), dim3(p.grid), dim3(256), 0, s, p);
    else
        hipLaunchKernelGGL((shrink_kernel<R, 1>), dim3(p.grid), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_shrink(const ShrinkParams &p, hipStream_t s)
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
