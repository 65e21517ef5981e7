// Shrink for decode batches (tiles of at most 16 rows): v = gather(x) * A.
//
// Work item = (row tile, K part); a workgroup of four waves takes one item and each wave
// owns a quarter of the part's K range.  A wave streams its slice of the packed A (and of
// the second fused projection's A) with 16-byte loads that are contiguous per wave, two
// steps in flight (software pipeline: the loads of step s+1 are issued before the MFMAs of
// step s), and multiplies it with the tile's gathered x rows.  The rank index sits on the M
// side of v_mfma_f32_16x16x32_bf16 and the rows on the N side, so a lane ends up with four
// consecutive rank entries of one row.  The four waves' sums are added through LDS in a
// fixed order and stored as this part's slice of v.
#include "lora_device.h"
#include "lora_internal.h"

namespace lora {

namespace {

template <int R, int NPROJ, bool NT>
struct ShrinkWave {
    static constexpr int NB = R >= 16 ? R / 16 : 1;
    static constexpr int KB = R <= 16 ? 4 : (R == 32 ? 2 : 1);

    int lane, g, i16, h_in;
    const uint16_t *Ap[NPROJ];
    const uint16_t *xp;      // this lane's x row (a valid row even if the lane's row is not)
    bool row_ok;
    f32x4 acc[NPROJ][NB];

    // All loads are unconditional: a K-block beyond the wave's range re-reads the last valid
    // block and a row beyond the tile re-reads the tile's first row; both are then replaced
    // by zeros with selects.  No branches, so the next step's loads stay in flight.
    __device__ inline void load(int kb0, int kb_end, u32x4 (&w)[NPROJ][KB][NB], u32x4 (&xv)[KB]) const
    {
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            const bool k_ok = kb0 + u < kb_end;
            const int kb = k_ok ? kb0 + u : kb_end - 1;
#pragma unroll
            for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    u32x4 t;
                    if (R >= 16) t = ld16<NT>(Ap[pj] + (((int64_t)kb * NB + nb) * 64 + lane) * 8);
                    else t = ld16<NT>(Ap[pj] + ((int64_t)kb * 32 + g * 8 + (i16 & 7)) * 8);
                    w[pj][u][nb] = (k_ok && (R >= 16 || i16 < 8)) ? t : zero4;
                }
            const bool c_ok = kb * kKBlock + g * 8 < h_in;
            const u32x4 t = ld16<false>(xp + (c_ok ? kb * kKBlock + g * 8 : 0));
            xv[u] = (k_ok && row_ok && c_ok) ? t : zero4;
        }
    }

    __device__ inline void mma(const u32x4 (&w)[NPROJ][KB][NB], const u32x4 (&xv)[KB])
    {
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[pj][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        as_bf16x8(w[pj][u][nb]), as_bf16x8(xv[u]), acc[pj][nb], 0, 0, 0);
    }
};

// tiles, units and counts are passed again as restrict-qualified kernel arguments: with a
// workgroup-uniform index the compiler then reads them through the scalar cache, which
// shortens the dependent chain tile -> unit -> first data load.
template <int R, int NPROJ, bool NT>
__global__ __launch_bounds__(256, 2) void shrink16_kernel(ShrinkParams p,
                                                          const lora_tile *__restrict__ tiles,
                                                          const Unit *__restrict__ units,
                                                          const int32_t *__restrict__ counts)
{
    using Wave = ShrinkWave<R, NPROJ, NT>;
    constexpr int NB = Wave::NB, KB = Wave::KB;
    __shared__ f32x4 red[4][NPROJ][NB][64];

    const int tid = threadIdx.x, wave = tid >> 6;
    Wave w;
    w.lane = tid & 63;
    w.g = w.lane >> 4;
    w.i16 = w.lane & 15;
    w.h_in = p.h_in;
    const int n_tiles = counts[2];
    const int n_items = n_tiles * p.n_parts;
    const int kblocks = (p.h_in + kKBlock - 1) / kKBlock;
    const int kb_per_wave = (p.kb_per_part + 3) >> 2;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int tile_ix = item / p.n_parts;
        const int part = item - tile_ix * p.n_parts;
        const lora_tile t = tiles[tile_ix];
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
            w.Ap[pj] = units[(int64_t)t.key * p.n_proj + p.proj0 + pj].A;
        w.row_ok = w.i16 < t.n_rows;
        {
            int s = p.perm[t.row0 + min(w.i16, t.n_rows - 1)];
            if (p.src_row) s = p.src_row[s];
            w.xp = p.x + (int64_t)s * p.ldx;
        }
        const int part_end = min((part + 1) * p.kb_per_part, kblocks);
        const int kb_begin = part * p.kb_per_part + wave * kb_per_wave;
        const int kb_end = min(kb_begin + kb_per_wave, part_end);
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) w.acc[pj][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

        if (kb_begin < kb_end) {
            u32x4 w0[NPROJ][KB][NB], x0[KB], w1[NPROJ][KB][NB], x1[KB];
            w.load(kb_begin, kb_end, w0, x0);
            for (int kb0 = kb_begin; kb0 < kb_end; kb0 += 2 * KB) {
                const bool has1 = kb0 + KB < kb_end;
                if (has1) w.load(kb0 + KB, kb_end, w1, x1);
                w.mma(w0, x0);
                if (has1) {
                    if (kb0 + 2 * KB < kb_end) w.load(kb0 + 2 * KB, kb_end, w0, x0);
                    w.mma(w1, x1);
                }
            }
        }

        // add the four waves' sums in a fixed order and store this part of v
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) red[wave][pj][nb][w.lane] = w.acc[pj][nb];
        __syncthreads();
        constexpr int NOUT = NPROJ * NB * 64;
        for (int o = tid; o < NOUT; o += 256) {
            const int l = o & 63;
            const int nb = (o >> 6) % NB;
            const int pj = (o >> 6) / NB;
            const int row = l & 15;
            const int j = nb * 16 + (l >> 4) * 4;
            if (row < t.n_rows && j < R) {
                f32x4 s = red[0][pj][nb][l];
                s += red[1][pj][nb][l];
                s += red[2][pj][nb][l];
                s += red[3][pj][nb][l];
                float *dst = p.v[pj] + ((int64_t)part * p.P + t.row0 + row) * R + j;
                st16f(dst, s);
            }
        }
        __syncthreads();
    }
}

template <int R, int NPROJ>
hipError_t launch_rn(const ShrinkParams &p, hipStream_t s)
{
    if (p.nontemporal)
        hipLaunchKernelGGL((shrink16_kernel<R, NPROJ, true>), dim3(p.grid), dim3(256), 0, s, p, p.tiles, p.units, p.counts);
    else
        hipLaunchKernelGGL((shrink16_kernel<R, NPROJ, false>), dim3(p.grid), dim3(256), 0, s, p, p.tiles, p.units, p.counts);
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const ShrinkParams &p, hipStream_t s)
{
    return p.n_fused == 2 ? launch_rn<R, 2>(p, s) : launch_rn<R, 1>(p, s);
}

}  // namespace

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
