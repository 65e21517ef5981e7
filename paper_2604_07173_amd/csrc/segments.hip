// Segment builder: stable counting sort of the batch rows by key = adapter * E + expert,
// then segment boundaries and row tiles (App. A.2.2: rows of one adapter are aggregated so its
// weights are read once; Sec. 2.3: per (adapter, expert) in MoE layers).  One workgroup of
// 1024 threads does the whole job out of LDS (a batch has at most 16384 rows and the result
// feeds kernels that run right after it, so latency matters, not bandwidth; gfx950 has
// 160 KiB of LDS per workgroup).  Global memory is only read for the ids and only written for
// the results.  One CU issues one wave instruction per four cycles and SIMD, so the time of
// either path below is essentially its instruction count.
//
// Two paths with identical results (rows ordered by key, original order inside a key):
//
// * Radix path (segments_kernel; long segments, or key spaces too large for LDS counters).
//   LDS holds key[row] for the whole batch and two 16-bit row-index arrays that the radix
//   passes (8 key bits each, least significant first) ping-pong between; the keys never move.
//   Stability without order-defining atomics: in every pass wave w owns the contiguous
//   positions [w*CH, (w+1)*CH) of the current order; it walks them 64 at a time in order,
//   ranks equal digits inside a group of 64 by lane order (ballot match) and keeps a running
//   per-digit count of its own (LDS adds whose only effect is a sum, so their order does not
//   matter); an exclusive scan over (digit, wave) in digit-major order turns the counts into
//   start positions.  With a single pass (at most 256 keys) the scanned histogram already is
//   the segment table.  Otherwise thread t owns `items` consecutive sorted positions and keeps
//   the boundary flags of its positions as a bit mask; three block scans (count of
//   boundaries, last boundary before, first boundary after) give every position its segment
//   index, start and end without reading anything back from global memory.
//
// * Counting path (segments_bucket_kernel; many short segments): described at the kernel.
#include <cstdlib>

#include "segments_common.h"

namespace lora {

namespace {

constexpr int kThreads = kSegThreads;
constexpr int kWaves = kSegWaves;
constexpr int kBins = kSegBins;
constexpr int kMaxItems = LORA_MAX_ROWS / kThreads;   // positions per thread, fits a 32-bit mask
static_assert(kMaxItems <= 32, "boundary flags are kept in a 32-bit mask");

struct ScanLds {
    int sum[kWaves];
    int mx[kWaves];
    int mn[kWaves];
    unsigned two[kWaves][2];
};

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

// key_of[i] for all rows; `each(i, key)` is called once per row.  The id loads of up to eight
// rows are issued before the first is used (the ids come from HBM; one round trip per row
// would otherwise dominate large batches).
template <int NT = kThreads, class F>
__device__ inline void all_row_keys(const SegParams &p, unsigned *key_of, unsigned &bad, F each)
{
    constexpr int U = 8;
    const int tid = threadIdx.x;
#pragma unroll 1
    for (int i0 = tid; i0 < p.P; i0 += U * NT) {
        int a[U], e[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u * NT;
            a[u] = -1;
            e[u] = 0;
            if (i < p.P) {
                a[u] = p.adapter_id[i];
                if (p.expert_id) e[u] = p.expert_id[i];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = i0 + u * NT;
            if (i < p.P) {
                const unsigned k = row_key(p, a[u], e[u], bad);
                key_of[i] = k;
                each(i, k);
            }
        }
    }
}

// The radix path, whole: keys, passes, boundaries, tiles, counts.
__device__ __forceinline__ void radix_body(const SegParams &p)
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
        all_row_keys(p, key_of, bad, [&](int, unsigned k) { n_active += k != kNoKey ? 1 : 0; });
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
                if (p.passes > 1) dst[pos] = (uint16_t)row;       // one pass: nothing reads the order back
                if (last) p.perm[pos] = (int32_t)row;
            }
        }
        __syncthreads();
        if (!last) {
            for (int b = tid; b < kWaves * kBins; b += kThreads) (&hist[0][0])[b] = 0;
            __syncthreads();
        }
    }
    const int TR = p.tile_rows;       // a power of two

    // ---- one pass (at most 256 keys): the scanned histogram already is the segment table ----
    if (p.passes == 1) {
        __shared__ unsigned bin_tile0[kBins];     // first tile of the key (exclusive prefix)
        __shared__ unsigned bin_seg[kBins];       // segment index of the key
        const int tr_shift = 31 - __clz(TR);
        unsigned start = 0, n = 0;
        if (tid < kBins) {
            start = hist[0][tid];                                  // wave 0's start = the key's start
            n = (tid + 1 < kBins ? hist[0][tid + 1] : (unsigned)P_act) - start;
        }
        const unsigned my_tiles = (n + TR - 1) >> tr_shift;
        unsigned seg_before, tile_before, S, n_tiles;
        block_excl_sum2(n ? 1u : 0u, my_tiles, scan.two, &seg_before, &tile_before, &S, &n_tiles);
        if (tid < kBins) {
            bin_tile0[tid] = tile_before;
            bin_seg[tid] = seg_before;
            if (n) {
                p.seg_start[seg_before] = (int32_t)start;
                p.seg_key[seg_before] = tid;
            }
        }
        __syncthreads();
        // tiles, one per thread and turn: the key of tile ti is the last one whose first tile
        // is not beyond ti (an empty key shares its first tile with the next key, which wins)
#pragma unroll 1
        for (unsigned ti = tid; ti < n_tiles; ti += kThreads) {
            int key = 0;
#pragma unroll
            for (int step = kBins / 2; step > 0; step >>= 1)
                if (bin_tile0[key + step] <= ti) key += step;
            const unsigned kstart = hist[0][key];
            const unsigned kend = key + 1 < kBins ? hist[0][key + 1] : (unsigned)P_act;
            const unsigned r = (ti - bin_tile0[key]) << tr_shift;
            lora_tile t;
            t.key = key;
            t.row0 = (int32_t)(kstart + r);
            t.n_rows = (int32_t)min((unsigned)TR, kend - kstart - r);
            t.seg = (int32_t)bin_seg[key];
            p.tiles[ti] = t;
        }
        if (tid == 0) {
            p.seg_start[S] = P_act;
            p.counts[0] = (int32_t)S;
            p.counts[1] = P_act;
            p.counts[2] = (int32_t)n_tiles;
            p.counts[3] = 0;
            p.status[0] = status_bits;
        }
        return;
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

__global__ __launch_bounds__(kThreads) void segments_kernel(SegParams p)
{
    radix_body(p);
}

// ---- bucket path ---------------------------------------------------------------------------
// For batches of many short segments (decode): one LDS counter per key instead of radix
// passes over the key bits.
//   1. count the rows of every key with LDS adds (a sum: the order of the adds is immaterial);
//   2. thread t owns a contiguous range of keys: an exclusive scan over the counts gives
//      every key its start; the keys that occur are the segments, so they are listed in LDS
//      and the segment records and tiles are then written one segment per thread;
//   3. every row takes a place inside its key's range with a fetching LDS add; which place
//      depends on the order the adds execute in, so
//   4. every row is re-ranked inside its bucket by the number of rows of the bucket with a
//      smaller row index: the final order is by (key, row index), unique, hence bit-identical
//      run to run and identical to the stable sort of the radix path.
// Step 4 costs bucket length per row; if one key holds more than kMaxBucket rows the
// workgroup drops this attempt and runs the radix path (a workgroup-uniform decision).
//
// Longer batches are launched with several workgroups.  Step 1 and the sums of step 2 are
// repeated by every one of them (a workgroup cannot hand anything to another inside a launch,
// and repeating costs no time); the list of segments with the keys' starts, the segment records
// and tiles, step 3 and step 4 are shared out by segment index: workgroup g of G takes the
// segments [S g / G, S (g + 1) / G), which are a contiguous range of keys and of sorted
// positions.  Measured on the fine-grained MoE shapes (8192 rows, 32768 keys), kernel time in a
// rocprofv3 trace: one workgroup 17.1 us, eight workgroups 13.6 us (the steps that every
// workgroup repeats are about 6 us of it).  If the radix path has to run, workgroup 0 runs it.
//
// Two 16-bit counters share a 32-bit LDS word (a batch has at most 16384 rows, so neither
// half overflows and positions fit 16 bits).  The words are skewed by one word per
// thread-owned range so that the threads' range walks hit different banks.
constexpr int kMaxBucket = 256;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// SHIFT = log2 of the counter words a thread owns (1 .. 32 words: up to 65536 keys); a
// compile-time constant so that a thread's words live in registers between the scan and the
// passes that need them again, and every loop over them is unrolled with its LDS reads in
// flight together.
template <int NT, int SHIFT>
__global__ __launch_bounds__(NT) void segments_bucket_kernel(SegParams p)
{
    constexpr int WPT = 1 << SHIFT;                   // counter words per thread
    constexpr int n_cnt = (NT << SHIFT) + NT;         // counter words incl. the skew
    constexpr int NW = NT / 64;
    constexpr bool kFallback = NT == kThreads;        // the radix path is written for kThreads
    __shared__ unsigned wave_sums[NW][2];
    __shared__ unsigned status_bits;
    __shared__ int n_active_total;
    __shared__ unsigned longest;
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int G = gridDim.x, wg = blockIdx.x;         // workgroups that share steps 2b to 4
    const int P = p.P;
    const int P_pad = (P + 63) & ~63;
    unsigned *key_of = reinterpret_cast<unsigned *>(dyn_lds);           // [P_pad]
    unsigned *cnt = key_of + P_pad;                                     // [n_cnt]
    unsigned *tmp = cnt + n_cnt;                                        // [P_pad] row | key << 16
    unsigned *seglist = tmp;               // key | first tile << 16 per segment, before tmp is used
    auto slot = [&](unsigned word) { return word + (SHIFT ? word >> SHIFT : 0u); };
    auto half_of = [&](unsigned key) { return (cnt[slot(key >> 1)] >> ((key & 1u) * 16u)) & 0xFFFFu; };

    if (tid == 0) {
        status_bits = 0;
        n_active_total = 0;
        longest = 0;
    }
#pragma unroll
    for (int j = 0; j < WPT + 1; ++j) cnt[tid + j * NT] = 0;
    __syncthreads();

    // ---- 1. keys and counts --------------------------------------------------------------
    {
        int n_active = 0;
        unsigned bad = 0;
        all_row_keys<NT>(p, key_of, bad, [&](int, unsigned k) {
            if (k != kNoKey) {
                ++n_active;
                atomicAdd(&cnt[slot(k >> 1)], 1u << ((k & 1u) * 16u));
            }
        });
        if (bad) atomicOr(&status_bits, bad);
#pragma unroll 1
        for (int o = 32; o > 0; o >>= 1) n_active += __shfl_xor(n_active, o, 64);
        if (lane == 0 && n_active) atomicAdd(&n_active_total, n_active);
    }
    __syncthreads();

    // ---- 2. scan over the keys; segments and tiles ----------------------------------------
    const int TR = p.tile_rows;                       // a power of two
    const int tr_shift = 31 - __clz(TR);
    const unsigned w0 = (unsigned)tid << SHIFT;       // my counter words: w0 .. w0 + WPT - 1
    unsigned rs_before, rs_total, t_before, t_total;  // rows | segments << 16, and tiles
    unsigned cw[WPT];                                 // my words (two 16-bit counts each)
    unsigned segs_mine;                               // occupied keys among mine
    {
        unsigned rows = 0, tiles = 0, mx = 0, segs = 0;
#pragma unroll
        for (int j = 0; j < WPT; ++j) cw[j] = cnt[slot(w0 + j)];
#pragma unroll
        for (int j = 0; j < WPT; ++j) {
            const unsigned lo = cw[j] & 0xFFFFu, hi = cw[j] >> 16;
            rows += lo + hi;
            tiles += ((lo + TR - 1) >> tr_shift) + ((hi + TR - 1) >> tr_shift);
            mx = max(mx, max(lo, hi));
            segs += (lo ? 1u : 0u) + (hi ? 1u : 0u);
        }
        segs_mine = segs;
        if (kFallback && mx > kMaxBucket) atomicMax(&longest, mx);
        // a batch has at most 16384 rows, so rows and segments share a word
        block_excl_sum2<NW>(rows | (segs << 16), tiles, wave_sums, &rs_before, &t_before, &rs_total,
                        &t_total);
    }
    if constexpr (kFallback) {
        if (longest > kMaxBucket) {    // same value in every thread: read after the scan's barrier
            __syncthreads();
            if (wg == 0) radix_body(p);               // every workgroup has seen the same counts
            return;
        }
    }
    const int P_act = (int)(rs_total & 0xFFFFu);
    const int S = (int)(rs_total >> 16);
    const int n_tiles = (int)t_total;
    // From here on workgroup wg takes the segments [s0, s1), i.e. the keys [key_lo, key_hi) and the
    // sorted positions [pos_lo, pos_hi); up to here every workgroup has done the same.
    const int s0 = (int)((int64_t)S * wg / G), s1 = (int)((int64_t)S * (wg + 1) / G);
    // Only the threads whose keys lie in or next to that range go on: the others' segments are
    // listed, and their keys' counts turned into starts, by the workgroups that need them.
    const int seg_first = (int)(rs_before >> 16);
    if (seg_first <= s1 && seg_first + (int)segs_mine >= s0) {
        // list of the occupied keys with the first tile of each, and the start of every key in
        // place of its count (all from the words in registers: nothing is read back)
        int sidx = (int)(rs_before >> 16);
        unsigned tix = t_before;
        unsigned at = rs_before & 0xFFFFu;
#pragma unroll
        for (int j = 0; j < WPT; ++j) {
            const unsigned lo = cw[j] & 0xFFFFu, hi = cw[j] >> 16;
            if (cw[j]) {                               // most words of a large key space are empty
                if (lo) {
                    seglist[sidx++] = (w0 + j) * 2 | (tix << 16);
                    tix += (lo + TR - 1) >> tr_shift;
                }
                if (hi) {
                    seglist[sidx++] = ((w0 + j) * 2 + 1) | (tix << 16);
                    tix += (hi + TR - 1) >> tr_shift;
                }
            }
            cnt[slot(w0 + j)] = at | ((at + lo) << 16);
            at += lo + hi;
        }
    }
    __syncthreads();
    const unsigned key_lo = s0 < S ? seglist[s0] & 0xFFFFu : 0x10000u;
    const unsigned key_hi = s1 < S ? seglist[s1] & 0xFFFFu : 0x10000u;
    const int pos_lo = s0 < S ? (int)half_of(key_lo) : P_act;
    const int pos_hi = s1 < S ? (int)half_of(key_hi) : P_act;
    // segment records and tiles, one segment per thread and turn
#pragma unroll 1
    for (int sidx = s0 + tid; sidx < s1; sidx += NT) {
        const unsigned me = seglist[sidx];
        const unsigned next = seglist[min(sidx + 1, S - 1)];
        const int key = (int)(me & 0xFFFFu);
        const int pos = (int)half_of(me & 0xFFFFu);
        const int n = (sidx + 1 < S ? (int)half_of(next & 0xFFFFu) : P_act) - pos;
        int tix = (int)(me >> 16);
        p.seg_start[sidx] = pos;
        p.seg_key[sidx] = key;
#pragma unroll 1
        for (int r = 0; r < n; r += TR) {
            lora_tile t;
            t.key = key;
            t.row0 = pos + r;
            t.n_rows = min(TR, n - r);
            t.seg = sidx;
            p.tiles[tix++] = t;
        }
    }
    __syncthreads();

    // ---- 3. a place in the key's range for every row --------------------------------------
    // four rows per turn: their key reads, fetching adds and stores overlap
#pragma unroll 1
    for (int i0 = tid; i0 < P; i0 += 4 * NT) {
        unsigned k[4], old[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            k[u] = i0 + u * NT < P ? key_of[i0 + u * NT] : kNoKey;
            if (k[u] < key_lo || k[u] >= key_hi) k[u] = kNoKey;     // another workgroup's key
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k[u] != kNoKey) old[u] = atomicAdd(&cnt[slot(k[u] >> 1)], 1u << ((k[u] & 1u) * 16u));
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (k[u] != kNoKey)
                tmp[(old[u] >> ((k[u] & 1u) * 16u)) & 0xFFFFu] = (unsigned)(i0 + u * NT) | (k[u] << 16);
    }
    // filler around this workgroup's positions: step 4 reads aligned groups of four words
    if (tid < 4 && (pos_lo & ~3) + tid < pos_lo) tmp[(pos_lo & ~3) + tid] = 0xFFFFFFFFu;
    if (tid >= 4 && tid < 8 && pos_hi + tid - 4 < ((pos_hi + 3) & ~3)) tmp[pos_hi + tid - 4] = 0xFFFFFFFFu;
    __syncthreads();

    // ---- 4. order inside the bucket by row index -------------------------------------------
    // after step 3 a key's counter holds the end of its range = the start of the next key's
    // The bucket is read in aligned groups of four words; words of other keys (and the
    // filler around the workgroup's positions) fall outside [key << 16, mine) and count as not
    // smaller.
#pragma unroll 1
    for (int pos = pos_lo + tid; pos < pos_hi; pos += NT) {
        const unsigned mine = tmp[pos];
        const unsigned k = mine >> 16, row = mine & 0xFFFFu, base = mine & 0xFFFF0000u;
        const int e = (int)half_of(k);
        // the key before this workgroup's first one is another's: its counter still holds its start
        const int b = k == key_lo ? pos_lo : (int)half_of(k - 1);
        int rank = 0;
#pragma unroll 1
        for (int j = b & ~3; j < e; j += 4) {
            const u32x4 t = *reinterpret_cast<const u32x4 *>(tmp + j);
            rank += (t[0] - base < row ? 1 : 0) + (t[1] - base < row ? 1 : 0) +
                    (t[2] - base < row ? 1 : 0) + (t[3] - base < row ? 1 : 0);
        }
        p.perm[b + rank] = (int32_t)row;
    }
    if (tid == 0 && wg == 0) {
        p.seg_start[S] = P_act;
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

// log2 of the counter words a thread of the bucket path owns
static int bucket_shift_of(unsigned n_keys)
{
    const unsigned n_words = (n_keys + 1) / 2;
    int shift = 0;
    while (((unsigned)kThreads << shift) < n_words) ++shift;
    return shift;
}

// dynamic LDS of the bucket path (it may fall back to the radix path inside the kernel)
static size_t bucket_lds_bytes(int P, unsigned n_keys)
{
    const size_t P_pad = ((size_t)P + 63) & ~(size_t)63;
    const size_t n_cnt = ((size_t)kThreads << bucket_shift_of(n_keys)) + kThreads;
    const size_t need = P_pad * 4 + n_cnt * 4 + P_pad * 4;
    return need > segments_lds_bytes(P) ? need : segments_lds_bytes(P);
}

constexpr size_t kBucketLdsMax = 140 * 1024;
constexpr int kBucketWorkgroups = 8;

template <int NT, int SHIFT>
static hipError_t launch_bucket(const SegParams &p, size_t dyn, hipStream_t s)
{
    static hipError_t attr = hipFuncSetAttribute(
        reinterpret_cast<const void *>(segments_bucket_kernel<NT, SHIFT>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)kBucketLdsMax);
    if (attr != hipSuccess) return attr;
    // the counting and the scan over the keys are done by every workgroup, the rest is shared out
    const int wgs = std::max(1, std::min(kBucketWorkgroups, p.P / 1024));
    hipLaunchKernelGGL((segments_bucket_kernel<NT, SHIFT>), dim3(wgs), dim3(NT), dyn, s, p);
    return hipGetLastError();
}

hipError_t launch_segments(const SegParams &p_in, void *ws, hipStream_t s)
{
    SegParams p = p_in;
    // long batches of few keys: several workgroups (segments_large.hip)
    if (segments_large_handles(p)) return launch_segments_large(p, ws, s);
    // short segments on average and counters that fit LDS beside the radix path's static
    // arrays: bucket path
    const unsigned n_keys = (unsigned)p.n_adapters * (unsigned)p.n_experts;
    // LORA_SEGMENT_PATH=radix forces the radix path (both give the same result)
    static const bool force_radix = [] {
        const char *e = getenv("LORA_SEGMENT_PATH");
        return e && e[0] == 'r';
    }();
    // one radix pass (at most 256 keys) is as fast as the counting path and has no bucket
    // limit: prefer it once there are enough rows per key for long buckets to be likely
    const bool radix_is_cheap = p.passes == 1 && (int64_t)p.P >= 8 * (int64_t)n_keys;
    if (!force_radix && !radix_is_cheap && (int64_t)p.P < 64 * (int64_t)n_keys && n_keys <= 0x10000u &&
        bucket_lds_bytes(p.P, n_keys) <= kBucketLdsMax) {
        const size_t dyn = bucket_lds_bytes(p.P, n_keys);
        const int shift = bucket_shift_of(n_keys);
        switch (shift) {
        case 0: return launch_bucket<kThreads, 0>(p, dyn, s);
        case 1: return launch_bucket<kThreads, 1>(p, dyn, s);
        case 2: return launch_bucket<kThreads, 2>(p, dyn, s);
        case 3: return launch_bucket<kThreads, 3>(p, dyn, s);
        case 4: return launch_bucket<kThreads, 4>(p, dyn, s);
        default: return launch_bucket<kThreads, 5>(p, dyn, s);
        }
    }
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
