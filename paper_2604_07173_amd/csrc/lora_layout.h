// Packed (re-tiled) storage of a unit's A and B inside the pool slab.
//
// The kernels feed v_mfma_f32_16x16x32_bf16, whose two bf16 operands want, per lane
// l = 16*g + i (g = 0..3, i = 0..15), eight consecutive K elements 8*g .. 8*g+7 of
// row/column i.  Storing the matrices so that lane l's eight values are contiguous and
// consecutive lanes are adjacent lets one 16-byte load per lane fetch an operand with the
// whole wave reading one contiguous 1 KiB block.
//
// Shrink operand, A[h_in][rank] (K = input index c, M = rank index j):
//   rank >= 16: block (kb = c/32, nb = j/16) of 64 lanes x 8 values;
//               lane 16*g + (j%16) holds c = 32*kb + 8*g + t, t = 0..7.
//   rank == 8 : block q of 64 lanes x 8 values covers 64 K values: lane 16*g + 8*half + j
//               holds c = 64*q + 32*half + 8*g + t, so that no lane of the 1 KiB block is
//               idle; the kernel multiplies the block twice, once with the x values of each
//               half, and keeps rows 0..7 of the first product and rows 8..15 of the second.
//   K is padded with zeros to a multiple of 32 (rank 8: 64).
//
// Expand operand, B[rank][h_out] (K = rank index j, N = output column d):
//   columns are grouped in chunks of 128; inside a chunk the MFMA column slot n = 0..15 of
//   sub-block blk = 0..7 is output column 8*n + blk, so that after the eight MFMAs of a
//   chunk a lane owns eight consecutive output columns of a row (one 16-byte access).
//   rank >= 32 (v_mfma_f32_16x16x32_bf16): K steps of 32, ks = j/32; within a step lane
//     group gl = (j%32)/8 holds t = j%8; a sub-block is 64 lanes x 16 bytes per K step.
//   rank <= 16 (v_mfma_f32_16x16x16_bf16, four K values per lane): lane group gl = j/4
//     holds t = j%4; the 8-byte operands of sub-blocks 2q and 2q+1 of a lane are adjacent, so
//     a wave reads a pair of sub-blocks with one 16-byte load per lane (rank 16: 1 KiB
//     contiguous, no two lanes read the same bytes).
//   Columns are padded with zeros to a multiple of 128.
#pragma once
#include <stdint.h>

#ifndef LORA_HD
#define LORA_HD __host__ __device__ inline
#endif

namespace lora {

// K values per packed block of the shrink operand
LORA_HD int packA_kunit(int rank) { return rank == 8 ? 64 : 32; }

LORA_HD int64_t packA_index(int c, int j, int rank)
{
    const int g = (c & 31) >> 3, t = c & 7;
    if (rank == 8) {
        const int q = c >> 6, half = (c >> 5) & 1;
        return (((int64_t)q * 64) + g * 16 + half * 8 + j) * 8 + t;
    }
    const int kb = c >> 5;
    const int NB = rank >> 4, nb = j >> 4, n = j & 15;
    return ((((int64_t)kb * NB + nb) * 64) + g * 16 + n) * 8 + t;
}

LORA_HD int64_t packB_index(int j, int d, int rank)
{
    const int chunk = d >> 7, dd = d & 127, n = dd >> 3, blk = dd & 7;
    if (rank <= 16) {
        // sub-blocks in pairs: a lane's operands of sub-blocks 2q and 2q+1 are adjacent
        const int G = rank >> 2, gl = j >> 2, t = j & 3;
        return ((((((int64_t)chunk * 4 + (blk >> 1)) * G + gl) * 16) + n) * 2 + (blk & 1)) * 4 + t;
    }
    const int KS = rank >> 5;
    const int ks = j >> 5, gl = (j & 31) >> 3, t = j & 7;
    return ((((((int64_t)chunk * 8 + blk) * KS + ks) * 4 + gl) * 16) + n) * 8 + t;
}

}  // namespace lora
