// Segment builder: stable counting sort of the batch rows by key = adapter * E + expert,
// then segment boundaries and row tiles.  One workgroup of 1024 threads does the whole job
// out of LDS (a batch has at most 16384 rows and the result feeds kernels that run right
// after it, so latency matters, not bandwidth; gfx950 has 160 KiB of LDS per workgroup).
// Global memory is only read for the ids and only written for the results.
//
// LDS holds key[row] for the whole batch and two 16-bit row-index arrays that the radix
// passes (8 key bits each, least significant first) ping-pong between; the keys never move.
//
// Stability without order-defining atomics: in every pass wave w owns the contiguous
// positions [w*CH, (w+1)*CH) of the current order; it walks them 64 at a time in order,
// ranks equal digits inside a group of 64 by lane order (ballot match) and keeps a running
// per-digit count of its own (LDS adds whose only effect is a sum, so their order does not
// matter); an exclusive scan over (digit, wave) in digit-major order turns the counts into
// start positions.  Equal keys therefore keep their original order and the output is
// unique, hence bit-identical run to run.
//
// Boundaries and tiles: thread t owns `items` consecutive sorted positions and keeps the
// boundary flags of its positions as a bit mask; three block scans (count of boundaries,
// last boundary before, first boundary after) give every position its segment index, start
// and end without reading anything back from global memory.
#include "lora_internal.h"

namespace lora {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kBins = 256;
constexpr int kMaxItems = LORA_MAX_ROWS / kThreads;   // positions per thread, fits a 32-bit mask
static_assert(kMaxItems <= 32, "boundary flags are kept in a 32-bit mask");

struct ScanLds {
    int sum[kWaves];
    int mx[kWaves];
    int mn[kWaves];
};

// exclusive prefix sum over the workgroup, plus the total
__device__ __noinline__ int block_excl_sum(int v, int *total, volatile int *wave_sums)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int inc = v;
#pragma unroll 1
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) wave_sums[w] = inc;
    __syncthreads();
    // wave totals: lane k < 16 fetches total k, a wave reduction does the rest
    const int mine = lane < kWaves ? wave_sums[lane] : 0;
    int tot = mine, base = lane < w ? mine : 0;
#pragma unroll 1
    for (int o = 8; o > 0; o >>= 1) {
        tot += __shfl_xor(tot, o, 64);
        base += __shfl_xor(base, o, 64);
    }
    tot = __shfl(tot, 0, 64);
    base = __shfl(base, 0, 64);
    *total = tot;
    return base + inc - v;
}

// three scans with one pair of barriers: exclusive sum of `cnt` (and total), exclusive
// running max of `last` over earlier threads, exclusive running min of `first` over later
// threads
__device__ inline void block_scan3(int cnt, int last, int first, ScanLds *s,
                                   int *cnt_before, int *cnt_total, int *last_before,
                                   int *first_after)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int isum = cnt, imax = last, imin = first;
#pragma unroll 1
    for (int o = 1; o < 64; o <<= 1) {
        const int a = __shfl_up(isum, o, 64), b = __shfl_up(imax, o, 64);
        const int c = __shfl_down(imin, o, 64);
        if (lane >= o) {
            isum += a;
            imax = max(imax, b);
        }
        if (lane + o < 64) imin = min(imin, c);
    }
    __syncthreads();
    if (lane == 63) {
        s->sum[w] = isum;
        s->mx[w] = imax;
    }
    if (lane == 0) s->mn[w] = imin;
    __syncthreads();
    // lane k < 16 fetches wave k's values; a 16-lane butterfly combines them
    const bool in = lane < kWaves;
    const int a = in ? s->sum[lane] : 0, b = in ? s->mx[lane] : -1, c = in ? s->mn[lane] : 0x7FFFFFFF;
    int tot = a, base = lane < w ? a : 0, mx = lane < w ? b : -1, mn = lane > w ? c : 0x7FFFFFFF;
#pragma unroll 1
    for (int o = 8; o > 0; o >>= 1) {
        tot += __shfl_xor(tot, o, 64);
        base += __shfl_xor(base, o, 64);
        mx = max(mx, __shfl_xor(mx, o, 64));
        mn = min(mn, __shfl_xor(mn, o, 64));
    }
    tot = __shfl(tot, 0, 64);
    base = __shfl(base, 0, 64);
    mx = __shfl(mx, 0, 64);
    mn = __shfl(mn, 0, 64);
    // exclusive within the wave: take the neighbour's inclusive value
    const int pmax = __shfl_up(imax, 1, 64), nmin = __shfl_down(imin, 1, 64);
    *cnt_before = base + isum - cnt;
    *cnt_total = tot;
    *last_before = lane > 0 ? max(mx, pmax) : mx;
    *first_after = lane < 63 ? min(mn, nmin) : mn;
}

// Lanes of the wave whose digit equals mine (restricted to valid lanes), as two 32-bit
// halves.  Per digit bit that can be set: one ballot, then keep the lanes whose bit equals mine.
struct Match {
    unsigned lo, hi;
};

__device__ __noinline__ Match match_digit(unsigned digit, bool valid, int nbits)
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

__global__ __launch_bounds__(kThreads) void segments_kernel(SegParams p)
{
    __shared__ unsigned hist[kWaves][kBins];
    __shared__ ScanLds scan;
    __shared__ unsigned status_bits;
    __shared__ int n_active_total;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int P = p.P;
    const int P_pad = (P + 63) & ~63;
    unsigned *key_of = reinterpret_cast<unsigned *>(dyn_lds);                    // [P_pad]
    uint16_t *order[2] = {reinterpret_cast<uint16_t *>(key_of + P_pad),          // [P_pad] each
                          reinterpret_cast<uint16_t *>(key_of + P_pad) + P_pad};
    const unsigned n_keys = (unsigned)p.n_adapters * (unsigned)p.n_experts;
    constexpr unsigned kNoKey = 0xFFFFFFFFu;               // row without adapter: dropped by pass 0
    const int items = (P + kThreads - 1) / kThreads;       // 64-row groups per wave
    const int wave_base = w * items * 64;
    const bool park = n_keys <= 0x10000u;                  // room for a 16-bit rank above the key
    const unsigned key_mask = park ? 0xFFFFu : 0xFFFFFFFFu;

    if (tid == 0) {
        status_bits = 0;
        n_active_total = 0;
    }
    for (int b = tid; b < kWaves * kBins; b += kThreads) (&hist[0][0])[b] = 0;
    __syncthreads();

    // ---- key of every row (independent loads, four in flight per thread) -----------------
    {
        int n_active = 0;
        unsigned bad = 0;
#pragma unroll 1
        for (int i = tid; i < P; i += kThreads) {
            const int a = p.adapter_id[i];
            const int e = p.expert_id ? p.expert_id[i] : 0;
            const bool a_ok = a >= 0 && a < p.n_adapters;
            const bool e_ok = e >= 0 && e < p.n_experts;
            const bool none = a == -1;
            const bool ok = a_ok && e_ok;
            key_of[i] = ok ? (unsigned)a * (unsigned)p.n_experts + (unsigned)e : kNoKey;
            n_active += ok ? 1 : 0;
            if (!none && !ok)
                bad |= (a_ok ? 0u : (unsigned)LORA_STATUS_BAD_ADAPTER) |
                       (e_ok ? 0u : (unsigned)LORA_STATUS_BAD_EXPERT);
        }
        if (bad) atomicOr(&status_bits, bad);          // OR and + are order-independent
#pragma unroll 1
        for (int o = 32; o > 0; o >>= 1) n_active += __shfl_xor(n_active, o, 64);
        if (lane == 0 && n_active) atomicAdd(&n_active_total, n_active);
    }
    __syncthreads();
    const int P_act = n_active_total;

    // ---- radix passes over the row order ----------------------------------------------
    for (int pass = 0; pass < p.passes; ++pass) {
        const int shift = 8 * pass;
        const int nbits = min(8, p.key_bits - shift);      // digit bits that can be set
        const bool last = pass == p.passes - 1;
        const int n_in = pass == 0 ? P : P_act;            // pass 0 leaves the rows without adapter out
        const uint16_t *src = order[(pass + 1) & 1];   // unused in pass 0 (identity order)
        uint16_t *dst = order[pass & 1];
        unsigned *my_hist = hist[w];

        // count: rank of every element among the equal digits of its wave; when keys fit
        // 16 bits the rank is parked in the upper half of the key word for the scatter
#pragma unroll 1
        for (int g = 0; g < items; ++g) {
            const int i = wave_base + g * 64 + lane;
            const bool in = i < n_in;
            const unsigned row = in ? (pass == 0 ? (unsigned)i : (unsigned)src[i]) : 0u;
            const unsigned kfull = in ? key_of[row] : kNoKey;
            const bool val = in && (pass != 0 || kfull != kNoKey);
            const unsigned k = val ? kfull & key_mask : 0u;
            const unsigned dig = (k >> shift) & 255u;
            const Match m = match_digit(dig, val, nbits);
            const unsigned below = lanes_below(m);
            // every lane reads the digit's running count before the leader advances it; LDS
            // operations of one wave execute in program order
            const unsigned first = *(volatile unsigned *)&my_hist[dig];
            if (val && park) key_of[row] = k | ((first + below) << 16);
            __builtin_amdgcn_wave_barrier();
            if (val && below == 0) my_hist[dig] = first + __popc(m.lo) + __popc(m.hi);
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
        // exclusive scan over (digit, wave), digit-major: thread t owns digit t/4 and waves
        // 4*(t%4) .. 4*(t%4)+3
        {
            const int bin = tid >> 2, w0 = (tid & 3) * 4;
            const unsigned c0 = hist[w0][bin], c1 = hist[w0 + 1][bin], c2 = hist[w0 + 2][bin],
                           c3 = hist[w0 + 3][bin];
            int tot;
            const unsigned base = (unsigned)block_excl_sum((int)(c0 + c1 + c2 + c3), &tot, scan.sum);
            hist[w0][bin] = base;
            hist[w0 + 1][bin] = base + c0;
            hist[w0 + 2][bin] = base + c0 + c1;
            hist[w0 + 3][bin] = base + c0 + c1 + c2;
        }
        __syncthreads();
        // scatter: position = start of (digit, wave) + rank within it
#pragma unroll 1
        for (int g = 0; g < items; ++g) {
            const int i = wave_base + g * 64 + lane;
            const bool in = i < n_in;
            const unsigned row = in ? (pass == 0 ? (unsigned)i : (unsigned)src[i]) : 0u;
            const unsigned kfull = in ? key_of[row] : kNoKey;
            const bool val = in && (pass != 0 || kfull != kNoKey);
            const unsigned kw = val ? kfull : 0u;
            const unsigned dig = ((kw & key_mask) >> shift) & 255u;
            unsigned pos;
            if (park) {
                pos = my_hist[dig] + (kw >> 16);
            } else {
                const Match m = match_digit(dig, val, nbits);
                const unsigned below = lanes_below(m);
                const unsigned first = *(volatile unsigned *)&my_hist[dig];
                pos = first + below;
                __builtin_amdgcn_wave_barrier();
                if (val && below == 0) my_hist[dig] = first + __popc(m.lo) + __popc(m.hi);
                __builtin_amdgcn_wave_barrier();
            }
            if (val) {
                dst[pos] = (uint16_t)row;
                if (last) p.perm[pos] = (int32_t)row;
            }
        }
        __syncthreads();
        if (!last) {
            for (int b = tid; b < kWaves * kBins; b += kThreads) (&hist[0][0])[b] = 0;
            __syncthreads();
        }
    }
    const uint16_t *sorted = order[(p.passes - 1) & 1];

    // ---- segment boundaries of my positions as a bit mask --------------------------------
    const int i0 = tid * items;
    unsigned F = 0;
    {
        unsigned prev = (i0 > 0 && i0 - 1 < P_act) ? (key_of[sorted[i0 - 1]] & key_mask) : 0xFFFFFFFFu;
        for (int q = 0; q < items; ++q) {
            const int i = i0 + q;
            if (i >= P_act) break;
            const unsigned k = key_of[sorted[i]] & key_mask;
            if (i == 0 || k != prev) F |= 1u << q;
            prev = k;
        }
    }
    const int my_last = F ? i0 + 31 - __clz(F) : -1;
    const int my_first = F ? i0 + __ffs(F) - 1 : 0x7FFFFFFF;
    int seg_before, S, start_before, next_after;
    block_scan3(__popc(F), my_last, my_first, &scan, &seg_before, &S, &start_before, &next_after);
    next_after = min(next_after, P_act);

    // ---- segment records and tile starts -------------------------------------------------
    const int TR = p.tile_rows;       // a power of two
    unsigned T = 0;                   // tile starts among my positions
    {
        int sidx = seg_before;
        int seg_begin = start_before;
        for (int q = 0; q < items; ++q) {
            const int i = i0 + q;
            if (i >= P_act) break;
            if (F & (1u << q)) {
                seg_begin = i;
                p.seg_start[sidx] = i;
                p.seg_key[sidx] = (int32_t)(key_of[sorted[i]] & key_mask);
                ++sidx;
            }
            if (((i - seg_begin) & (TR - 1)) == 0) T |= 1u << q;
        }
    }
    if (tid == 0) p.seg_start[S] = P_act;
    int n_tiles;
    int tix = block_excl_sum(__popc(T), &n_tiles, scan.sum);
    for (unsigned rest = T; rest; rest &= rest - 1) {
        const int q = __ffs(rest) - 1;
        const int i = i0 + q;
        const unsigned above = q >= 31 ? 0u : F & (0xFFFFFFFEu << q);      // boundaries after i
        const int seg_end = above ? i0 + __ffs(above) - 1 : next_after;
        lora_tile t;
        t.key = (int32_t)(key_of[sorted[i]] & key_mask);
        t.row0 = i;
        t.n_rows = min(TR, seg_end - i);
        t.seg = seg_before + __popc(F & (0xFFFFFFFFu >> (31 - q))) - 1;
        p.tiles[tix++] = t;
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
