// Segment builder for long batches: the stable counting sort of segments.hip spread over
// several workgroups (App. A.2.2: rows that share an adapter are aggregated; Sec. 2.3: per
// (adapter, expert)).  Same results, bit for bit: rows ordered by key = adapter * E + expert,
// original order inside a key, rows without adapter left out.
//
// A batch is cut into chunks of kChunk consecutive rows, one workgroup each.  Stability needs no
// order-defining atomic: inside a workgroup, wave w owns the contiguous positions
// [w * 128, (w + 1) * 128) of the chunk, walks them 64 at a time in order and ranks equal digits
// inside a group of 64 by lane order (ballot match); a position in the sorted order is then
//   start of the digit + rows of that digit in earlier chunks + in earlier waves of the chunk
//   + in earlier groups of the wave + lanes below in the group.
// Nothing in that sum depends on the order in which anything executed.
//
// Per pass of 8 key bits, two launches (a launch boundary is the only hand-off between
// workgroups, so nothing ever waits inside a kernel):
//   count:   every workgroup counts the digits of its chunk -> wg_hist[chunk][256]
//   scatter: every workgroup sums wg_hist over the chunks (totals, and the rows of earlier
//            chunks), scans the 256 totals, recounts its own chunk wave by wave and writes its
//            rows to their positions.
// Up to 256 keys take one pass, and the scanned totals then are the segment table: every
// workgroup knows it, workgroup 0 writes the segment records and the counts, and the tiles are
// dealt out over all workgroups.  Larger key spaces take one pass per 8 key bits (a pass reads
// the rows in the order the previous one left them) and then two launches that find the segment
// boundaries in the sorted keys:
//   heads:  every workgroup marks the positions of its chunk whose key differs from the one
//           before (segment heads) and writes how many there are, the first and the last, and
//           how many tiles start at or behind the chunk's first head
//   bounds: every workgroup scans those chunk records (segments and tiles of earlier chunks,
//           the last head before the chunk, the first head behind it) and writes the segment
//           records and tiles of its chunk.
#include <string.h>

#include "segments_common.h"

namespace lora {

namespace {

constexpr int kChunk = 2048;                        // rows per workgroup
// Shorter batches stay with the single workgroup.  Measured on MI355X, 8 and 256 keys: one
// workgroup takes 9.5 / 10.8 us at 4096 rows, 10.9 / 13.6 at 6144, 12.8 / 16.5 at 8192 and
// 20.7 / 28.1 at 16384; the two launches here take 10.0-11.8 us at every one of those sizes.
constexpr int kLargeMinRows = 5120;
constexpr int kGroups = kChunk / kSegThreads;       // 64-row groups per wave
static_assert(kGroups * kSegThreads == kChunk, "a chunk is whole groups of every wave");

struct Group64 {                                    // what a lane keeps of a row between the passes over its groups
    unsigned row;
    unsigned dig;
    unsigned rank;                                  // equal digits before it in its wave
    bool val;
};

// Digits of this workgroup's chunk: fills hist[wave][digit] with the counts per wave and leaves
// in g[] every lane's rows with their rank inside the wave.  PASS0: rows come in batch order
// and their keys from the ids (and are written to key_g for later passes); otherwise rows come
// from order_in and keys from key_g.
template <bool PASS0>
__device__ inline void count_chunk(const LargeSegParams &q, unsigned (*hist)[kSegBins], Group64 (&g)[kGroups],
                                   unsigned &bad, int &n_active)
{
    const SegParams &p = q.p;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int n_in = PASS0 ? p.P : (int)q.header[0];
    const int shift = 8 * q.pass;
    const int nbits = min(8, p.key_bits - shift);
    unsigned *my_hist = hist[w];
    int a[kGroups], e[kGroups];
    unsigned kk[kGroups];
#pragma unroll
    for (int u = 0; u < kGroups; ++u) {             // all loads of the wave's groups first
        const int pos = blockIdx.x * kChunk + (w * kGroups + u) * 64 + lane;
        const bool in = pos < n_in;
        a[u] = -1;
        e[u] = 0;
        kk[u] = kNoKey;
        g[u].row = (unsigned)pos;
        if (PASS0) {
            if (in) {
                a[u] = p.adapter_id[pos];
                if (p.expert_id) e[u] = p.expert_id[pos];
            }
        } else if (in) {
            g[u].row = q.order_in[pos];
            kk[u] = q.key_g[g[u].row];
        }
    }
#pragma unroll
    for (int u = 0; u < kGroups; ++u) {
        const int pos = blockIdx.x * kChunk + (w * kGroups + u) * 64 + lane;
        const bool in = pos < n_in;
        unsigned key = kk[u];
        if (PASS0) {
            key = in ? row_key(p, a[u], e[u], bad) : kNoKey;
            if (in && q.key_g) q.key_g[pos] = key;
        }
        const bool val = in && key != kNoKey;
        n_active += val ? 1 : 0;
        const unsigned dig = val ? (key >> shift) & 255u : 0u;
        const Match m = match_digit(dig, val, nbits);
        const unsigned below = lanes_below(m);
        // every lane reads the digit's running count before the leader advances it; LDS
        // operations of one wave execute in program order
        const unsigned first = *(volatile unsigned *)&my_hist[dig];
        __builtin_amdgcn_wave_barrier();
        if (val && below == 0) my_hist[dig] = first + __popc(m.lo) + __popc(m.hi);
        __builtin_amdgcn_wave_barrier();
        g[u].dig = dig;
        g[u].rank = first + below;
        g[u].val = val;
    }
}

template <bool PASS0>
__global__ __launch_bounds__(kSegThreads) void seg_large_count_kernel(LargeSegParams q)
{
    __shared__ unsigned hist[kSegWaves][kSegBins];
    __shared__ unsigned status_bits;
    __shared__ int n_active_total;
    const int tid = threadIdx.x, lane = tid & 63;
    if (tid == 0) {
        status_bits = 0;
        n_active_total = 0;
    }
    for (int b = tid; b < kSegWaves * kSegBins; b += kSegThreads) (&hist[0][0])[b] = 0;
    __syncthreads();
    Group64 g[kGroups];
    unsigned bad = 0;
    int n_active = 0;
    count_chunk<PASS0>(q, hist, g, bad, n_active);
    if (PASS0) {
        if (bad) atomicOr(&status_bits, bad);      // OR and + are order-independent
#pragma unroll 1
        for (int o = 32; o > 0; o >>= 1) n_active += __shfl_xor(n_active, o, 64);
        if (lane == 0 && n_active) atomicAdd(&n_active_total, n_active);
    }
    __syncthreads();
    if (tid < kSegBins) {
        unsigned s = 0;
#pragma unroll
        for (int w = 0; w < kSegWaves; ++w) s += hist[w][tid];
        q.wg_hist[(size_t)blockIdx.x * kSegBins + tid] = s;
    }
    if (PASS0 && tid == 0) {
        q.wg_info[2 * blockIdx.x] = (unsigned)n_active_total;
        q.wg_info[2 * blockIdx.x + 1] = status_bits;
    }
}

// FINAL: this pass completes the order (rows go to perm); with a single pass the scanned totals
// are the segment table, written here too.
template <bool PASS0, bool FINAL>
__global__ __launch_bounds__(kSegThreads) void seg_large_scatter_kernel(LargeSegParams q)
{
    __shared__ unsigned hist[kSegWaves][kSegBins];
    __shared__ unsigned key_start[kSegBins + 1];     // start of every digit in the sorted order
    __shared__ unsigned bin_tile0[kSegBins];         // single pass: first tile of the key
    __shared__ unsigned bin_seg[kSegBins];           // single pass: segment index of the key
    __shared__ int scan_sums[kSegWaves];
    __shared__ unsigned scan_two[kSegWaves][2];
    const SegParams &p = q.p;
    const int tid = threadIdx.x;
    const int w = tid >> 6;
    for (int b = tid; b < kSegWaves * kSegBins; b += kSegThreads) (&hist[0][0])[b] = 0;
    __syncthreads();
    Group64 g[kGroups];
    unsigned bad = 0;
    int n_active = 0;
    count_chunk<PASS0>(q, hist, g, bad, n_active);

    // totals of every digit over all chunks, and the rows of earlier chunks
    unsigned tot = 0, before = 0;
    if (tid < kSegBins) {
        const unsigned *col = q.wg_hist + tid;
        int c = 0;
#pragma unroll 1
        for (; c + 4 <= q.G; c += 4) {               // four loads in flight
            const unsigned h0 = col[(size_t)c * kSegBins], h1 = col[(size_t)(c + 1) * kSegBins],
                           h2 = col[(size_t)(c + 2) * kSegBins], h3 = col[(size_t)(c + 3) * kSegBins];
            tot += h0 + h1 + h2 + h3;
            before += (c < (int)blockIdx.x ? h0 : 0u) + (c + 1 < (int)blockIdx.x ? h1 : 0u) +
                      (c + 2 < (int)blockIdx.x ? h2 : 0u) + (c + 3 < (int)blockIdx.x ? h3 : 0u);
        }
        for (; c < q.G; ++c) {
            const unsigned h = col[(size_t)c * kSegBins];
            tot += h;
            before += c < (int)blockIdx.x ? h : 0u;
        }
    }
    int P_act;
    const unsigned start = (unsigned)block_excl_sum((int)tot, &P_act, scan_sums);   // barriers inside
    if (tid < kSegBins) key_start[tid] = start;
    if (tid == 0) key_start[kSegBins] = (unsigned)P_act;
    __syncthreads();                                 // every wave's counts of this chunk are in hist
    if (tid < kSegBins) {
        // start of (digit, wave) = start of the digit + earlier chunks + earlier waves
        unsigned acc = start + before;
#pragma unroll
        for (int k = 0; k < kSegWaves; ++k) {
            const unsigned c = hist[k][tid];
            hist[k][tid] = acc;
            acc += c;
        }
    }
    __syncthreads();
    int32_t *dst = FINAL ? p.perm : reinterpret_cast<int32_t *>(q.order_out);
#pragma unroll
    for (int u = 0; u < kGroups; ++u)
        if (g[u].val) dst[hist[w][g[u].dig] + g[u].rank] = (int32_t)g[u].row;
    if (!FINAL) {
        if (blockIdx.x == 0 && tid == 0) q.header[0] = (unsigned)P_act;     // rows of the next pass
        return;
    }
    if (p.passes != 1) return;                       // boundaries come from the sorted keys

    // ---- single pass: the scanned totals are the segment table -------------------------------
    const int TR = p.tile_rows;                      // a power of two
    const int tr_shift = 31 - __clz(TR);
    const unsigned my_tiles = (tot + TR - 1) >> tr_shift;
    unsigned seg_before, tile_before, S, n_tiles;
    block_excl_sum2(tot ? 1u : 0u, my_tiles, scan_two, &seg_before, &tile_before, &S, &n_tiles);
    if (tid < kSegBins) {
        bin_tile0[tid] = tile_before;
        bin_seg[tid] = seg_before;
        if (tot && blockIdx.x == 0) {
            p.seg_start[seg_before] = (int32_t)start;
            p.seg_key[seg_before] = tid;
        }
    }
    __syncthreads();
    // tiles, dealt out over all workgroups: the key of tile ti is the last one whose first tile
    // is not beyond ti (an empty key shares its first tile with the next key, which wins)
#pragma unroll 1
    for (unsigned ti = blockIdx.x * kSegThreads + tid; ti < n_tiles; ti += gridDim.x * kSegThreads) {
        int key = 0;
#pragma unroll
        for (int step = kSegBins / 2; step > 0; step >>= 1)
            if (bin_tile0[key + step] <= ti) key += step;
        const unsigned kstart = key_start[key], kend = key_start[key + 1];
        const unsigned r = (ti - bin_tile0[key]) << tr_shift;
        lora_tile t;
        t.key = key;
        t.row0 = (int32_t)(kstart + r);
        t.n_rows = (int32_t)min((unsigned)TR, kend - kstart - r);
        t.seg = (int32_t)bin_seg[key];
        p.tiles[ti] = t;
    }
    if (blockIdx.x == 0 && tid == 0) {
        unsigned status = 0;
        for (int c = 0; c < q.G; ++c) status |= q.wg_info[2 * c + 1];
        p.seg_start[S] = P_act;
        p.counts[0] = (int32_t)S;
        p.counts[1] = P_act;
        p.counts[2] = (int32_t)n_tiles;
        p.counts[3] = 0;
        p.status[0] = status;
    }
}

// ---- several passes: segment boundaries from the sorted keys ----------------------------------

constexpr unsigned kNone = 0xFFFFFFFFu;
constexpr int kPosPerThread = kChunk / kSegThreads;  // consecutive positions of a thread
static_assert(kPosPerThread == 2, "the head scan below is written for two positions per thread");

struct Heads {                                      // a thread's two consecutive sorted positions
    unsigned pos0;
    unsigned key[2];
    bool in[2], head[2];
    unsigned ord[2];                                // heads of the chunk up to and including the position
};

// Marks the segment heads of this workgroup's chunk of the sorted order, numbers them and lists
// their positions in head_pos[].  n = rows in the order.
__device__ inline void chunk_heads(const LargeSegParams &q, unsigned n, Heads &h, unsigned *head_pos,
                                   int *scan_sums, int *n_heads)
{
    const int tid = threadIdx.x;
    h.pos0 = (unsigned)blockIdx.x * kChunk + 2u * tid;
    h.in[0] = h.pos0 < n;
    h.in[1] = h.pos0 + 1 < n;
    const int32_t *perm = q.p.perm;
    const bool has_prev = h.in[0] && h.pos0 > 0;
    const int32_t rp = has_prev ? perm[h.pos0 - 1] : 0;
    const int32_t r0 = h.in[0] ? perm[h.pos0] : 0;
    const int32_t r1 = h.in[1] ? perm[h.pos0 + 1] : 0;
    const unsigned kp = has_prev ? q.key_g[rp] : kNoKey;
    h.key[0] = h.in[0] ? q.key_g[r0] : kNoKey;
    h.key[1] = h.in[1] ? q.key_g[r1] : kNoKey;
    h.head[0] = h.in[0] && (!has_prev || h.key[0] != kp);
    h.head[1] = h.in[1] && h.key[1] != h.key[0];
    const int mine = (h.head[0] ? 1 : 0) + (h.head[1] ? 1 : 0);
    const int before = block_excl_sum(mine, n_heads, scan_sums);            // barriers inside
    h.ord[0] = (unsigned)before + (h.head[0] ? 1u : 0u);
    h.ord[1] = h.ord[0] + (h.head[1] ? 1u : 0u);
    if (h.head[0]) head_pos[h.ord[0] - 1] = h.pos0;
    if (h.head[1]) head_pos[h.ord[1] - 1] = h.pos0 + 1;
    __syncthreads();
}

// chunk record: {heads, first head, last head, tiles that start at or behind the first head}
__global__ __launch_bounds__(kSegThreads) void seg_large_heads_kernel(LargeSegParams q)
{
    __shared__ unsigned head_pos[kChunk];
    __shared__ int scan_sums[kSegWaves];
    const unsigned n = q.header[0];
    const unsigned tr_mask = (unsigned)q.p.tile_rows - 1u;                  // a power of two
    Heads h;
    int n_heads;
    chunk_heads(q, n, h, head_pos, scan_sums, &n_heads);
    int tiles = 0;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (h.in[j] && h.ord[j] >= 1 && ((h.pos0 + j - head_pos[h.ord[j] - 1]) & tr_mask) == 0) ++tiles;
    int n_tiles;
    block_excl_sum(tiles, &n_tiles, scan_sums);
    if (threadIdx.x == 0) {
        unsigned *rec = q.chunk_info + 4 * (size_t)blockIdx.x;
        rec[0] = (unsigned)n_heads;
        rec[1] = n_heads ? head_pos[0] : kNone;
        rec[2] = n_heads ? head_pos[n_heads - 1] : kNone;
        rec[3] = (unsigned)n_tiles;
    }
}

// inclusive prefix maximum over the workgroup
__device__ inline unsigned block_incl_max(unsigned v, volatile unsigned *wave_max)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned up = (unsigned)__shfl_up((int)v, o, 64);
        if (lane >= o) v = max(v, up);
    }
    __syncthreads();
    if (lane == 63) wave_max[w] = v;
    __syncthreads();
    unsigned base = 0;
    for (int k = 0; k < w; ++k) base = max(base, wave_max[k]);
    return max(v, base);
}

__global__ __launch_bounds__(kSegThreads) void seg_large_bounds_kernel(LargeSegParams q)
{
    __shared__ unsigned head_pos[kChunk];
    __shared__ int scan_sums[kSegWaves];
    __shared__ unsigned scan_two[kSegWaves][2];
    __shared__ unsigned wave_max[kSegWaves];
    __shared__ unsigned mine_of[6];     // this chunk: segments before, tiles before, last head before, first head behind; S, tiles
    const SegParams &p = q.p;
    const int tid = threadIdx.x;
    const unsigned n = q.header[0];
    const int TR = p.tile_rows;
    const int tr_shift = 31 - __clz(TR);
    const unsigned tr_mask = (unsigned)TR - 1u;

    // ---- the chunk records: thread c looks at chunk c and, for the scan from the right, at
    // chunk G-1-c (at most kSegThreads chunks: LORA_MAX_ROWS_LONG / kChunk)
    const bool have = tid < q.G;
    const unsigned *rec = q.chunk_info + 4 * (size_t)(have ? tid : 0);
    const unsigned heads_c = have ? rec[0] : 0u, first_c = have ? rec[1] : kNone, last_c = have ? rec[2] : kNone,
                   tiles_c = have ? rec[3] : 0u;
    const unsigned first_r = have ? q.chunk_info[4 * (size_t)(q.G - 1 - tid) + 1] : kNone;
    // last head in chunks before c: positions + 1, so that 0 means none
    const unsigned incl_last = block_incl_max(last_c == kNone ? 0u : last_c + 1u, wave_max);
    const unsigned up_last = (unsigned)__shfl_up((int)incl_last, 1, 64);
    __syncthreads();
    if ((tid & 63) == 63) wave_max[tid >> 6] = incl_last;
    __syncthreads();
    const unsigned carry1 = (tid & 63) ? up_last : (tid ? wave_max[(tid >> 6) - 1] : 0u);   // exclusive
    // tiles of chunk c = those behind its first head + those between its start and that head,
    // which continue the segment of the last head before the chunk
    unsigned pre = 0;
    if (have && carry1) {
        const unsigned lo = (unsigned)tid * kChunk;
        const unsigned hi = min(min(first_c, lo + (unsigned)kChunk), n);
        if (hi > lo) {
            const unsigned a = lo - (carry1 - 1u), b = hi - (carry1 - 1u);
            pre = ((b + tr_mask) >> tr_shift) - ((a + tr_mask) >> tr_shift);
        }
    }
    unsigned seg_before, tile_before, S, n_tiles;
    __syncthreads();
    block_excl_sum2(heads_c, tiles_c + pre, scan_two, &seg_before, &tile_before, &S, &n_tiles);
    // first head in chunks behind chunk G-1-tid, as n - position so that a maximum finds it
    const unsigned incl_first = block_incl_max(first_r == kNone ? 0u : n - first_r, wave_max);
    const unsigned up_first = (unsigned)__shfl_up((int)incl_first, 1, 64);
    __syncthreads();
    if ((tid & 63) == 63) wave_max[tid >> 6] = incl_first;
    __syncthreads();
    const unsigned behind = (tid & 63) ? up_first : (tid ? wave_max[(tid >> 6) - 1] : 0u);   // exclusive
    if (tid == (int)blockIdx.x) {
        mine_of[0] = seg_before;
        mine_of[1] = tile_before;
        mine_of[2] = carry1;
    }
    if (have && q.G - 1 - tid == (int)blockIdx.x) mine_of[3] = n - behind;  // n if no head follows
    if (tid == 0) {
        mine_of[4] = S;
        mine_of[5] = n_tiles;
    }
    __syncthreads();
    const unsigned my_seg0 = mine_of[0], my_tile0 = mine_of[1], my_carry1 = mine_of[2], my_next = mine_of[3];

    // ---- this chunk's segment records and tiles --------------------------------------------------
    Heads h;
    int n_heads;
    chunk_heads(q, n, h, head_pos, scan_sums, &n_heads);
    bool th[2];
    unsigned start[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        start[j] = h.ord[j] >= 1 ? head_pos[h.ord[j] - 1] : my_carry1 - 1u;   // a position without a head before it has a carry
        th[j] = h.in[j] && ((h.pos0 + j - start[j]) & tr_mask) == 0;
    }
    int tiles_total;
    const int tiles_before = block_excl_sum((th[0] ? 1 : 0) + (th[1] ? 1 : 0), &tiles_total, scan_sums);
    unsigned ti = my_tile0 + (unsigned)tiles_before;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const unsigned pos = h.pos0 + j;
        const unsigned seg = my_seg0 + h.ord[j] - 1u;
        if (h.head[j] && seg < (unsigned)p.P) {              // never beyond the caller's arrays
            p.seg_start[seg] = (int32_t)pos;
            p.seg_key[seg] = (int32_t)h.key[j];
        }
        if (th[j] && ti < (unsigned)p.P) {
            const unsigned end = (int)h.ord[j] < n_heads ? head_pos[h.ord[j]] : my_next;
            lora_tile t;
            t.key = (int32_t)h.key[j];
            t.row0 = (int32_t)pos;
            t.n_rows = (int32_t)min((unsigned)TR, end - pos);
            t.seg = (int32_t)seg;
            p.tiles[ti] = t;
        }
        ti += th[j] ? 1u : 0u;
    }
    if (blockIdx.x == 0 && tid == 0) {
        unsigned status = 0;
        for (int c = 0; c < q.G; ++c) status |= q.wg_info[2 * c + 1];
        p.seg_start[mine_of[4]] = (int32_t)n;
        p.counts[0] = (int32_t)mine_of[4];
        p.counts[1] = (int32_t)n;
        p.counts[2] = (int32_t)mine_of[5];
        p.counts[3] = 0;
        p.status[0] = status;
    }
}

}  // namespace

static int segments_large_chunks(int P) { return (P + kChunk - 1) / kChunk; }
// One pass (at most 256 keys) and a batch long enough for two launches of many workgroups to
// beat one launch of a single workgroup; or a batch beyond what a single workgroup holds.
bool segments_large_handles(const SegParams &p)
{
    return (p.passes == 1 && p.P >= kLargeMinRows) || p.P > LORA_MAX_ROWS;
}

int segments_large_launches(const SegParams &p) { return p.passes == 1 ? 2 : 2 * p.passes + 2; }

namespace {
struct LargeLayout {
    size_t hist, info, chunk_info, key, order[2], total;
};
LargeLayout large_layout(int P)
{
    const size_t G = (size_t)segments_large_chunks(P);
    LargeLayout L;
    size_t o = 256;                                   // header
    L.hist = o, o += align_up(G * kSegBins * sizeof(unsigned), 256);
    L.info = o, o += align_up(G * 2 * sizeof(unsigned), 256);
    L.chunk_info = o, o += align_up(G * 4 * sizeof(unsigned), 256);
    // keys and two row orders: only batches beyond a single workgroup can need several passes here
    const size_t rows = P > LORA_MAX_ROWS ? align_up((size_t)P * sizeof(unsigned), 256) : 0;
    L.key = o, o += rows;
    L.order[0] = o, o += rows;
    L.order[1] = o, o += rows;
    L.total = o;
    return L;
}
}  // namespace

size_t segments_large_ws_bytes(int P) { return large_layout(P).total; }

hipError_t launch_segments_large(const SegParams &p, void *ws, hipStream_t s)
{
    LargeSegParams q;
    memset(&q, 0, sizeof q);
    q.p = p;
    q.G = segments_large_chunks(p.P);
    if (q.G > kSegThreads) return hipErrorInvalidValue;        // the bounds kernel holds a chunk record per thread
    const LargeLayout L = large_layout(p.P);
    char *base = static_cast<char *>(ws);
    q.header = reinterpret_cast<unsigned *>(base);
    q.wg_hist = reinterpret_cast<unsigned *>(base + L.hist);
    q.wg_info = reinterpret_cast<unsigned *>(base + L.info);
    q.chunk_info = reinterpret_cast<unsigned *>(base + L.chunk_info);
    const dim3 grid(q.G), block(kSegThreads);
    hipError_t e;
    if (p.passes == 1) {
        q.pass = 0;
        hipLaunchKernelGGL((seg_large_count_kernel<true>), grid, block, 0, s, q);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL((seg_large_scatter_kernel<true, true>), grid, block, 0, s, q);
        return hipGetLastError();
    }
    if (p.P <= LORA_MAX_ROWS) return hipErrorInvalidValue;     // no room for keys and orders was asked for
    q.key_g = reinterpret_cast<unsigned *>(base + L.key);
    for (int pass = 0; pass < p.passes; ++pass) {
        const bool last = pass == p.passes - 1;
        q.pass = pass;
        q.order_in = pass ? reinterpret_cast<const unsigned *>(base + L.order[(pass - 1) & 1]) : nullptr;
        q.order_out = last ? nullptr : reinterpret_cast<unsigned *>(base + L.order[pass & 1]);
        if (pass == 0) {
            hipLaunchKernelGGL((seg_large_count_kernel<true>), grid, block, 0, s, q);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            hipLaunchKernelGGL((seg_large_scatter_kernel<true, false>), grid, block, 0, s, q);
        } else {
            hipLaunchKernelGGL((seg_large_count_kernel<false>), grid, block, 0, s, q);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            if (last)
                hipLaunchKernelGGL((seg_large_scatter_kernel<false, true>), grid, block, 0, s, q);
            else
                hipLaunchKernelGGL((seg_large_scatter_kernel<false, false>), grid, block, 0, s, q);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(seg_large_heads_kernel, grid, block, 0, s, q);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(seg_large_bounds_kernel, grid, block, 0, s, q);
    return hipGetLastError();
}

}  // namespace lora
