// Segment builder: stable counting sort of the batch rows by key = adapter * E + expert,
// then segment boundaries and row tiles.  One workgroup of 1024 threads does the whole job
// out of LDS (a batch has at most 16384 rows and the result feeds kernels that run right
// after it, so latency matters, not bandwidth; gfx950 has 160 KiB of LDS per workgroup).
//
// LDS holds key[row] for the whole batch and two 16-bit row-index arrays that the radix
// passes (8 key bits each, least significant first) ping-pong between; the keys never move.
//
// Stability without order-defining atomics: in every pass wave w owns the contiguous
// positions [w*CH, (w+1)*CH) of the current order; it walks them 64 at a time in order,
// ranks equal digits inside a group of 64 by lane order (ballot match) and keeps a running
// per-digit count of its own; an exclusive scan over (digit, wave) in digit-major order
// turns the counts into start positions.  Equal keys therefore keep their original order
// and the output is unique, hence bit-identical run to run.
#include "lora_internal.h"

namespace lora {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kBins = 256;

__device__ inline int block_excl_scan(int v, int *total, volatile int *wave_sums)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < kWaves; ++k) {
        int s = wave_sums[k];
        if (k < w) base += s;
        tot += s;
    }
    *total = tot;
    return base + inc - v;
}

// lanes of the wave whose digit equals mine (restricted to valid lanes)
__device__ inline unsigned long long match_digit(unsigned digit, bool valid)
{
    unsigned long long m = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
        const bool bit = (digit >> b) & 1u;
        const unsigned long long bal = __ballot(valid && bit);
        m &= bit ? bal : ~bal;
    }
    return m;
}

__global__ __launch_bounds__(kThreads) void segments_kernel(SegParams p)
{
    __shared__ unsigned hist[kWaves][kBins];
    __shared__ int wave_sums[kWaves];
    __shared__ unsigned status_bits;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int P = p.P;
    const int P_pad = (P + 63) & ~63;
    unsigned *key_of = reinterpret_cast<unsigned *>(dyn_lds);                    // [P_pad]
    uint16_t *order[2] = {reinterpret_cast<uint16_t *>(key_of + P_pad),          // [P_pad] each
                          reinterpret_cast<uint16_t *>(key_of + P_pad) + P_pad};
    const unsigned n_keys = (unsigned)p.n_adapters * (unsigned)p.n_experts;      // sentinel key
    const int items = (P + kThreads - 1) / kThreads;       // 64-row groups per wave
    const int wave_base = w * items * 64;
    const unsigned long long lt_mask = (1ull << lane) - 1ull;

    if (tid == 0) status_bits = 0;
    __syncthreads();

    // ---- key of every row --------------------------------------------------------------
    int n_active = 0;
    unsigned bad = 0;
#pragma unroll 4
    for (int i = tid; i < P; i += kThreads) {
        const int a = p.adapter_id[i];
        const int e = p.expert_id ? p.expert_id[i] : 0;
        unsigned k = n_keys;
        if (a != -1) {
            const bool a_ok = a >= 0 && a < p.n_adapters;
            const bool e_ok = e >= 0 && e < p.n_experts;
            if (a_ok && e_ok) {
                k = (unsigned)a * (unsigned)p.n_experts + (unsigned)e;
                ++n_active;
            } else {
                bad |= (a_ok ? 0u : (unsigned)LORA_STATUS_BAD_ADAPTER) |
                       (e_ok ? 0u : (unsigned)LORA_STATUS_BAD_EXPERT);
            }
        }
        key_of[i] = k;
    }
    if (bad) atomicOr(&status_bits, bad);   // OR is order-independent
    int P_act;
    block_excl_scan(n_active, &P_act, wave_sums);   // its barriers also publish key_of

    // ---- radix passes over the row order ----------------------------------------------
    for (int pass = 0; pass < p.passes; ++pass) {
        const int shift = 8 * pass;
        const bool last = pass == p.passes - 1;
        const uint16_t *src = order[(pass + 1) & 1];   // unused in pass 0 (identity order)
        uint16_t *dst = order[pass & 1];

        for (int b = tid; b < kWaves * kBins; b += kThreads) (&hist[0][0])[b] = 0;
        __syncthreads();

        volatile unsigned *my_hist = hist[w];
        // count
        for (int g = 0; g < items; ++g) {
            const int i = wave_base + g * 64 + lane;
            const bool valid = i < P;
            const unsigned row = valid ? (pass == 0 ? (unsigned)i : (unsigned)src[i]) : 0u;
            const unsigned digit = valid ? (key_of[row] >> shift) & 255u : 0u;
            const unsigned long long m = match_digit(digit, valid);
            if (valid && (m & lt_mask) == 0) my_hist[digit] += (unsigned)__popcll(m);
        }
        __syncthreads();

        // exclusive scan over (digit, wave), digit-major: thread t owns digit t/4 and waves
        // 4*(t%4) .. 4*(t%4)+3
        {
            const int bin = tid >> 2, w0 = (tid & 3) * 4;
            const unsigned c0 = hist[w0][bin], c1 = hist[w0 + 1][bin], c2 = hist[w0 + 2][bin],
                           c3 = hist[w0 + 3][bin];
            int tot;
            const unsigned base = (unsigned)block_excl_scan((int)(c0 + c1 + c2 + c3), &tot, wave_sums);
            hist[w0][bin] = base;
            hist[w0 + 1][bin] = base + c0;
            hist[w0 + 2][bin] = base + c0 + c1;
            hist[w0 + 3][bin] = base + c0 + c1 + c2;
        }
        __syncthreads();

        // scatter
        for (int g = 0; g < items; ++g) {
            const int i = wave_base + g * 64 + lane;
            const bool valid = i < P;
            const unsigned row = valid ? (pass == 0 ? (unsigned)i : (unsigned)src[i]) : 0u;
            const unsigned digit = valid ? (key_of[row] >> shift) & 255u : 0u;
            const unsigned long long m = match_digit(digit, valid);
            if (valid) {
                const unsigned pos = my_hist[digit] + (unsigned)__popcll(m & lt_mask);
                dst[pos] = (uint16_t)row;
                if (last) p.perm[pos] = (int32_t)row;
            }
            __builtin_amdgcn_wave_barrier();
            if (valid && (m & lt_mask) == 0) my_hist[digit] += (unsigned)__popcll(m);
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
    }
    const uint16_t *sorted = order[(p.passes - 1) & 1];

    // ---- segment boundaries: thread t owns sorted positions t*items .. t*items+items-1 ---
    const int i0 = tid * items;
    int n_flag = 0;
    {
        unsigned prev = (i0 > 0 && i0 - 1 < P_act) ? key_of[sorted[i0 - 1]] : 0xFFFFFFFFu;
        for (int q = 0; q < items; ++q) {
            const int i = i0 + q;
            if (i >= P_act) break;
            const unsigned k = key_of[sorted[i]];
            n_flag += (i == 0 || k != prev) ? 1 : 0;
            prev = k;
        }
    }
    int S;
    int sidx = block_excl_scan(n_flag, &S, wave_sums);
    {
        unsigned prev = (i0 > 0 && i0 - 1 < P_act) ? key_of[sorted[i0 - 1]] : 0xFFFFFFFFu;
        for (int q = 0; q < items; ++q) {
            const int i = i0 + q;
            if (i >= P_act) break;
            const unsigned k = key_of[sorted[i]];
            if (i == 0 || k != prev) {
                p.seg_start[sidx] = i;
                p.seg_key[sidx] = (int32_t)k;
                ++sidx;
            }
            prev = k;
        }
    }
    if (tid == 0) p.seg_start[S] = P_act;
    __syncthreads();   // seg_start / seg_key written above are read below by other threads

    // ---- tiles: thread t owns segments t*items .. ; a tile never crosses a segment -------
    const int TR = p.tile_rows;
    int n_my_tiles = 0;
    for (int q = 0; q < items; ++q) {
        const int s = i0 + q;
        if (s >= S) break;
        n_my_tiles += (p.seg_start[s + 1] - p.seg_start[s] + TR - 1) / TR;
    }
    int n_tiles;
    int tix = block_excl_scan(n_my_tiles, &n_tiles, wave_sums);
    for (int q = 0; q < items; ++q) {
        const int s = i0 + q;
        if (s >= S) break;
        const int b = p.seg_start[s], e = p.seg_start[s + 1], k = p.seg_key[s];
        for (int r0 = b; r0 < e; r0 += TR) {
            lora_tile t;
            t.key = k;
            t.row0 = r0;
            t.n_rows = min(TR, e - r0);
            t.seg = s;
            p.tiles[tix++] = t;
        }
    }
    if (tid == 0) {
        p.counts[0] = S;
        p.counts[1] = P_act;
        p.counts[2] = n_tiles;
        p.counts[3] = 0;
        p.status[0] = status_bits;
    }
}

}  // namespace

size_t segments_lds_bytes(int P)
{
    const size_t P_pad = ((size_t)P + 63) & ~(size_t)63;
    return P_pad * 4 + 2 * P_pad * 2;
}

hipError_t launch_segments(const SegParams &p, hipStream_t s)
{
    const size_t dyn = segments_lds_bytes(p.P);
    if (dyn > 48 * 1024) {
        // ask once for the largest dynamic LDS size this kernel is ever launched with
        static hipError_t attr = hipFuncSetAttribute(
            reinterpret_cast<const void *>(segments_kernel),
            hipFuncAttributeMaxDynamicSharedMemorySize, (int)segments_lds_bytes(LORA_MAX_ROWS));
        if (attr != hipSuccess) return attr;
    }
    hipLaunchKernelGGL(segments_kernel, dim3(1), dim3(kThreads), dyn, s, p);
    return hipGetLastError();
}

}  // namespace lora
