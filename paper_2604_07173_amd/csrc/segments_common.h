// Device helpers shared by the segment builders (segments.hip: one workgroup, everything in
// LDS; segments_large.hip: several workgroups for long batches): workgroup scans, the ballot
// match that ranks equal digits inside a wave, and the key of a row.
#pragma once
#include "lora_internal.h"

namespace lora {

constexpr int kSegThreads = 1024;
constexpr int kSegWaves = kSegThreads / 64;
constexpr int kSegBins = 256;

// inclusive prefix sum over the 64 lanes on the cross-lane data path (no LDS round trips):
// shifts inside the rows of 16 lanes, then lane 15 of a row added to the next row (rows 1
// and 3), then lane 31 added to rows 2 and 3.  A lane without a source adds 0.
__device__ inline unsigned wave_incl_sum(unsigned x)
{
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, false);   // row_shr:1
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, false);   // row_shr:2
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, false);   // row_shr:4
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, false);   // row_shr:8
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false);   // row_bcast:15
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false);   // row_bcast:31
    return x;
}

// exclusive prefix sum over the workgroup, plus the total
__device__ inline __noinline__ int block_excl_sum(int v, int *total, volatile int *wave_sums)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int inc = (int)wave_incl_sum((unsigned)v);
    __syncthreads();
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    // wave totals: lane k of the first 16 fetches total k, scalar reads of the lanes add them
    const int mine = wave_sums[lane & (kSegWaves - 1)];
    int tot = 0, base = 0;
#pragma unroll
    for (int k = 0; k < kSegWaves; ++k) {
        const int t = __builtin_amdgcn_readlane(mine, k);
        tot += t;
        base += k < w ? t : 0;
    }
    *total = tot;
    return base + inc - v;
}

// exclusive prefix sums of two values over the workgroup, plus their totals; one barrier
template <int NW = kSegWaves>
__device__ inline void block_excl_sum2(unsigned a, unsigned b, volatile unsigned (*wave_sums)[2],
                                       unsigned *a_before, unsigned *b_before, unsigned *a_total,
                                       unsigned *b_total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const unsigned ia = wave_incl_sum(a), ib = wave_incl_sum(b);
    if (lane == 63) {
        wave_sums[w][0] = ia;
        wave_sums[w][1] = ib;
    }
    __syncthreads();
    const unsigned ma = wave_sums[lane & (NW - 1)][0], mb = wave_sums[lane & (NW - 1)][1];
    unsigned ta = 0, tb = 0, ba = 0, bb = 0;
#pragma unroll
    for (int k = 0; k < NW; ++k) {
        const unsigned xa = (unsigned)__builtin_amdgcn_readlane((int)ma, k);
        const unsigned xb = (unsigned)__builtin_amdgcn_readlane((int)mb, k);
        ta += xa;
        tb += xb;
        ba += k < w ? xa : 0u;
        bb += k < w ? xb : 0u;
    }
    *a_before = ba + ia - a;
    *b_before = bb + ib - b;
    *a_total = ta;
    *b_total = tb;
}

// Lanes of the wave whose digit equals mine (restricted to valid lanes), as two 32-bit
// halves.  Per digit bit that can be set: one ballot, then keep the lanes whose bit equals mine.
struct Match {
    unsigned lo, hi;
};

__device__ inline __noinline__ Match match_digit(unsigned digit, bool valid, int nbits)
{
    const unsigned long long v = __ballot(valid);
    Match m = {(unsigned)v, (unsigned)(v >> 32)};
#pragma unroll 1
    for (int b = 0; b < nbits; ++b) {
        const unsigned bit = (digit >> b) & 1u;
        const unsigned long long bal = __ballot(valid && bit);
        const unsigned same = 0u - bit;                  // all ones if my bit is set
        m.lo &= ~((unsigned)bal ^ same);                 // bit ? bal : ~bal
        m.hi &= ~((unsigned)(bal >> 32) ^ same);
    }
    return m;
}

// number of lanes below mine in the mask
__device__ inline unsigned lanes_below(Match m)
{
    return __builtin_amdgcn_mbcnt_hi(m.hi, __builtin_amdgcn_mbcnt_lo(m.lo, 0u));
}

constexpr unsigned kNoKey = 0xFFFFFFFFu;               // row without adapter: left out of the order

// key of a row from its ids, or kNoKey; ids that are neither valid nor -1 are reported in `bad`
__device__ inline unsigned row_key(const SegParams &p, int a, int e, unsigned &bad)
{
    const bool a_ok = a >= 0 && a < p.n_adapters;
    const bool e_ok = e >= 0 && e < p.n_experts;
    const bool ok = a_ok && e_ok;
    if (a != -1 && !ok)
        bad |= (a_ok ? 0u : (unsigned)LORA_STATUS_BAD_ADAPTER) |
               (e_ok ? 0u : (unsigned)LORA_STATUS_BAD_EXPERT);
    return ok ? (unsigned)a * (unsigned)p.n_experts + (unsigned)e : kNoKey;
}

}  // namespace lora
