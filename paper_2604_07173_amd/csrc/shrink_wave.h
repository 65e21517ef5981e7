// The wave-level work of the decode shrink (tiles of at most 16 rows), shared by the shrink
// kernel and the kernel that runs shrink and expand in one launch: one wave multiplies a run of
// K units of the packed A (of up to three projections that read the same input) with the
// gathered x rows of one tile.
//
// A wave streams its slice of the packed A with 16-byte loads that are contiguous per wave, two
// steps in flight (the loads of step s+1 are issued before the MFMAs of step s; all loads are
// unconditional so the loop is branch-free and the hardware counters keep them outstanding).
// The rank index sits on the M side of v_mfma_f32_16x16x32_bf16 and the rows on the N side, so a
// lane ends up with four consecutive rank entries of one row.
//
// Rank 8: a packed block holds 64 K values (two 32-deep halves side by side in the 16 M rows),
// is multiplied once with each half's x values, and rows 0..7 of the first product plus rows
// 8..15 of the second give the eight rank entries.
#pragma once
#include "lora_device.h"
#include "lora_internal.h"

namespace lora {

// NT: the packed A is loaded with the streaming hint (it is read once).  XNT: so are the x rows
// (for inputs too large to stay in a cache until anyone reads them again).
//
// LINES (ranks 8 and 16, where a step covers 128 K values = 256 bytes of a row): the x rows are
// fetched as whole cache lines - instruction q reads rows 4q .. 4q+3 of the tile, 256 contiguous
// bytes each - and turned into the MFMA operand layout (16 rows on the lane index, 64 bytes of a
// row per operand) through 4 KiB of LDS owned by the wave, the 16-byte column of a row stored
// at column (col xor row) so that the row-wise writes and the operand-wise reads both touch every
// bank once.  Fetched in the operand layout directly, an instruction reads 16 rows x 64 bytes:
// half a line per row, and the other half by the next instruction.
template <int R, int NPROJ, bool NT, bool XNT = false, bool LINES = false>
struct ShrinkWave {
    static constexpr int NB = R >= 16 ? R / 16 : 1;            // weight tiles per K unit
    static constexpr int XN = R == 8 ? 2 : 1;                  // x operands per K unit
    static constexpr int NACC = R == 8 ? 2 : NB;               // accumulators per projection
    static constexpr int KU = R == 8 ? 64 : 32;                // K values per unit
    static constexpr int KB = R <= 16 ? (R == 8 ? 2 : 4) : (R == 32 ? 2 : 1);   // units per step
    static_assert(!LINES || KB * KU == 128, "whole-line rows: a step is 256 bytes of a row");

    int lane, g, i16, h_in;
    const uint16_t *Ap[NPROJ];
    const uint16_t *xp;      // this lane's x row (a valid row even if the lane's row is not)
    const uint16_t *xq[LINES ? 4 : 1];   // LINES: rows 4q + lane / 16 of the tile (valid rows likewise)
    u32x4 *xt;               // LINES: the wave's 4 KiB of LDS
    bool row_ok;
    f32x4 acc[NPROJ][NACC];

    struct Step {
        u32x4 w[NPROJ][KB][NB];
        u32x4 x[KB][XN];
    };

    // All loads are unconditional: a K unit beyond the wave's range re-reads the last valid
    // unit and a row beyond the tile re-reads the tile's first row; both are then replaced
    // by zeros with selects.  No branches, so the next step's loads stay in flight.
    __device__ inline void load(int kb0, int kb_end, Step &s) const
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
                    const u32x4 t = ld16<NT>(Ap[pj] + (((int64_t)kb * NB + nb) * 64 + lane) * 8);
                    s.w[pj][u][nb] = k_ok ? t : zero4;
                }
            if constexpr (!LINES) {
#pragma unroll
                for (int h = 0; h < XN; ++h) {
                    const int c = kb * KU + h * 32 + g * 8;
                    const bool c_ok = c < h_in;
                    const u32x4 t = ld16<XNT>(xp + (c_ok ? c : 0));
                    s.x[u][h] = (k_ok && row_ok && c_ok) ? t : zero4;
                }
            }
        }
        if constexpr (LINES) {
            // lane (g, i16) of instruction q: row 4q + g, K values kb0 * KU + 8 * i16 .. + 7; what
            // lies beyond the range or the row is replaced by zeros after the transposition
            const int c = kb0 * KU + i16 * 8;
            const bool ok = kb0 + i16 / (KU / 8) < kb_end && c < h_in;
#pragma unroll
            for (int q = 0; q < 4; ++q) (&s.x[0][0])[q] = ld16<XNT>(xq[q] + (ok ? c : 0));
        }
    }

    // LINES: the step's rows through LDS into operand order; everything the MFMAs must not see
    // (rows beyond the tile, K beyond the range) becomes zero here
    __device__ inline void to_operands(int kb0, int kb_end, Step &s) const
    {
        const u32x4 zero4 = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = 4 * q + g;
            xt[row * 16 + (i16 ^ row)] = (&s.x[0][0])[q];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int h = 0; h < XN; ++h) {
                const int piece = (u * KU + h * 32) / 8 + g;
                const u32x4 t = xt[i16 * 16 + (piece ^ i16)];
                const bool ok = kb0 + u < kb_end && row_ok && (kb0 + u) * KU + h * 32 + g * 8 < h_in;
                s.x[u][h] = ok ? t : zero4;
            }
        __builtin_amdgcn_wave_barrier();
    }

    __device__ inline void mma(const Step &s)
    {
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int pj = 0; pj < NPROJ; ++pj) {
                if (R == 8) {
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        acc[pj][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(s.w[pj][u][0]), as_bf16x8(s.x[u][h]), acc[pj][h], 0, 0, 0);
                } else {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[pj][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            as_bf16x8(s.w[pj][u][nb]), as_bf16x8(s.x[u][0]), acc[pj][nb], 0, 0, 0);
                }
            }
    }

    // K units kb_begin, kb_begin + stride, ... below kb_end in steps of KB units (stride = KB:
    // the contiguous range [kb_begin, kb_end)), two steps in flight
    __device__ inline void run(int kb_begin, int kb_end, int stride = KB)
    {
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int a = 0; a < NACC; ++a) acc[pj][a] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (kb_begin >= kb_end) return;
        Step s0, s1;
        load(kb_begin, kb_end, s0);
        int kb0 = kb_begin;
        for (; kb0 + 2 * stride < kb_end; kb0 += 2 * stride) {
            load(kb0 + stride, kb_end, s1);
            if constexpr (LINES) to_operands(kb0, kb_end, s0);
            mma(s0);
            load(kb0 + 2 * stride, kb_end, s0);
            if constexpr (LINES) to_operands(kb0 + stride, kb_end, s1);
            mma(s1);
        }
        if (kb0 + stride < kb_end) {
            load(kb0 + stride, kb_end, s1);
            if constexpr (LINES) to_operands(kb0, kb_end, s0);
            mma(s0);
            if constexpr (LINES) to_operands(kb0 + stride, kb_end, s1);
            mma(s1);
        } else {
            if constexpr (LINES) to_operands(kb0, kb_end, s0);
            mma(s0);
        }
    }
};

}  // namespace lora
