// C-ABI entry points: argument checks, pool bookkeeping, launch geometry.
// Every check that can be made on the host happens before the first HIP call, so a bad
// call costs nothing on the device and can be exercised on a machine without a GPU.
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "lora_internal.h"

using namespace lora;

namespace {

constexpr uint32_t kPoolMagic = 0x4C6F5241u;  // "LoRA"

thread_local std::string g_hip_error;

int hip_fail(hipError_t e)
{
    g_hip_error = hipGetErrorString(e);
    return LORA_ERR_HIP;
}

#define LORA_HIP(expr)                                  \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return hip_fail(e_);      \
    } while (0)

bool rank_ok(int r) { return r == 8 || r == 16 || r == 32 || r == 64; }
bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int env_int(const char *name, int dflt, int lo, int hi)
{
    const char *v = getenv(name);
    if (!v || !*v) return dflt;
    long x = strtol(v, nullptr, 10);
    if (x < lo || x > hi) return dflt;
    return (int)x;
}

// Work-split constants.  The library as shipped uses the defaults below, so workspace sizes
// and launch shapes depend only on the pool and the batch; a build with -DLORA_TUNING reads
// them from the environment instead (for parameter sweeps, never for the installed library).
int tune_int(const char *name, int dflt, int lo, int hi)
{
#ifdef LORA_TUNING
    return env_int(name, dflt, lo, hi);
#else
    (void)name;
    (void)lo;
    (void)hi;
    return dflt;
#endif
}

int cu_count()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

// Workspace of lora_moe_apply_static: one array per GPU, part of the loaded code object, so
// no call ever allocates it.  In host code the name below is only a handle for
// hipGetSymbolAddress; the address kernels and copies use is the one that call returns, looked
// up once per device with that device current and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = LORA_STATIC_WS_BYTES;

}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];

// address of `scratch` on the current device (resolved on the first call per device)
int static_scratch(void **out)
{
    int dev = -1;
    LORA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return LORA_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        LORA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return LORA_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LORA_OK;
}

}  // namespace

struct lora_pool {
    uint32_t magic;
    lora_pool_desc d;
    std::vector<float> scale;
    std::vector<int32_t> arank;
    char *slab;
    size_t slab_bytes;
    size_t table_bytes;
    size_t unit_bytes;                    // all projections of one (layer, adapter, expert)
    size_t A_off[LORA_MAX_PROJ], A_bytes[LORA_MAX_PROJ];
    size_t B_off[LORA_MAX_PROJ], B_bytes[LORA_MAX_PROJ];
    std::vector<Unit> table;              // host mirror of the device table
    std::vector<hipEvent_t> ready;        // [adapter][layer], created at the first async load
    int act_policy;                       // LORA_ACT_*: cache hints of the activation streams

    size_t unit_base(int layer, int adapter, int expert) const
    {
        return table_bytes +
               (((size_t)layer * d.n_adapters + adapter) * d.n_experts + expert) * unit_bytes;
    }
    size_t table_index(int layer, int adapter, int expert, int proj) const
    {
        return (((size_t)layer * d.n_adapters + adapter) * d.n_experts + expert) * d.n_proj + proj;
    }
    const Unit *device_table() const { return reinterpret_cast<const Unit *>(slab); }
};

namespace {

int check_desc(const lora_pool_desc *d)
{
    if (!d) return LORA_ERR_INVALID_ARG;
    if (d->n_adapters < 1 || d->n_layers < 1 || d->n_experts < 1) return LORA_ERR_INVALID_ARG;
    if (d->n_proj < 1 || d->n_proj > LORA_MAX_PROJ) return LORA_ERR_INVALID_ARG;
    if (d->dtype != LORA_DTYPE_BF16) return LORA_ERR_INVALID_ARG;
    if (!rank_ok(d->rank)) return LORA_ERR_UNSUPPORTED_RANK;
    if ((int64_t)d->n_adapters * d->n_experts >= (int64_t)1 << 30) return LORA_ERR_TOO_LARGE;
    for (int i = 0; i < d->n_proj; ++i) {
        const lora_proj_desc &p = d->proj[i];
        if (p.h_in < 8 || p.h_out < 8 || (p.h_in % 8) || (p.h_out % 8)) return LORA_ERR_BAD_SHAPE;
    }
    if (d->adapter_rank)
        for (int a = 0; a < d->n_adapters; ++a)
            if (d->adapter_rank[a] < 1 || d->adapter_rank[a] > d->rank) return LORA_ERR_UNSUPPORTED_RANK;
    return LORA_OK;
}

struct Layout {
    size_t table_bytes, unit_bytes, total;
    size_t A_off[LORA_MAX_PROJ], A_bytes[LORA_MAX_PROJ], B_off[LORA_MAX_PROJ], B_bytes[LORA_MAX_PROJ];
};

Layout layout_of(const lora_pool_desc &d)
{
    Layout L;
    const size_t n_units = (size_t)d.n_layers * d.n_adapters * d.n_experts;
    L.table_bytes = align_up(n_units * d.n_proj * sizeof(Unit), 256);
    size_t off = 0;
    for (int i = 0; i < d.n_proj; ++i) {
        L.A_off[i] = off;
        L.A_bytes[i] = packed_A_bytes(d.proj[i].h_in, d.rank);
        off = align_up(off + L.A_bytes[i], 256);
        L.B_off[i] = off;
        L.B_bytes[i] = packed_B_bytes(d.proj[i].h_out, d.rank);
        off = align_up(off + L.B_bytes[i], 256);
    }
    L.unit_bytes = off;
    L.total = L.table_bytes + n_units * L.unit_bytes;
    return L;
}

int check_pool(const lora_pool *p)
{
    if (!p || p->magic != kPoolMagic) return LORA_ERR_NOT_REGISTERED;
    return LORA_OK;
}

int check_unit(const lora_pool *p, int adapter, int layer, int expert, int proj)
{
    if (adapter < 0 || adapter >= p->d.n_adapters || layer < 0 || layer >= p->d.n_layers ||
        expert < 0 || expert >= p->d.n_experts || proj < 0 || proj >= p->d.n_proj)
        return LORA_ERR_BAD_SHAPE;
    return LORA_OK;
}

// upper bound on the number of row tiles a batch of P rows can produce
int64_t tiles_upper_bound(const lora_pool *p, int P, int tile_rows)
{
    const int64_t keys = (int64_t)p->d.n_adapters * p->d.n_experts;
    return std::min<int64_t>(P, std::min<int64_t>(keys, P) + P / tile_rows);
}

// Rows per tile for a batch: decode batches (few rows per adapter/expert cell) get the
// 16-row tiles of the decode kernels, batches with long segments the 32-row tiles.
int pick_tile_rows(const lora_pool *p, int P)
{
    if (p->d.rank == 8) return kDecodeTileRows;      // the 32-row shrink has no rank-8 form
    // test switch, looked at on every call: segments remember the height they were built with and
    // every compute call checks it, so a change between two calls is an error, not a mismatch
    const int forced = env_int("LORA_TILE_ROWS", 0, 0, 32);
    if (forced == kTileRows || forced == kDecodeTileRows) return forced;
    // Measured crossovers on MI355X: Mixtral shapes at rank 16 (256 keys) at 8192 rows, llama shapes
    // at rank 16 (64 keys) between 8192 and 16384 rows, prefill shapes at rank 64 (8 keys) between
    // 1024 and 2048 rows: the long-segment kernels pay off from rows x rank = 2^17 on (their two
    // extra launches and 128-row work items need that much to amortise), if the segments are
    // long enough to fill 32-row tiles at all.
    const int64_t keys = (int64_t)p->d.n_adapters * p->d.n_experts;
    return ((int64_t)P >= 32 * keys && (int64_t)P * p->d.rank >= kLongMinRowsTimesRank) ? kTileRows : kDecodeTileRows;
}

struct KSplit {
    int n_parts, kb_per_part;
    bool wave_per_tile;
};

// How the K range of a shrink is cut into parts: enough work items to fill the chip when the
// batch has few tiles, and no part longer than kPartKBlocks K-blocks.  Depends only on the
// pool and P, so lora_shrink, lora_expand and lora_v_bytes agree.
KSplit ksplit_of(const lora_pool *p, int proj, int P)
{
    const int kblocks = kblocks_of(p->d.proj[proj].h_in, p->d.rank);
    if (pick_tile_rows(p, P) == kDecodeTileRows) {
        // decode: parts of about kb_target K-blocks, more of them when the batch has so few
        // tiles that the chip would not be filled otherwise, at most max_parts
        static const int kb_target = tune_int("LORA_DEC_KB_PER_PART", 32, 4, 4096);
        static const int max_parts = tune_int("LORA_DEC_MAX_PARTS", 8, 1, kMaxParts);
        static const int want_wgs = tune_int("LORA_DEC_SHRINK_ITEMS", 1024, 1, 1 << 20);
        const int64_t tub = std::max<int64_t>(1, tiles_upper_bound(p, P, kDecodeTileRows));
        // thousands of tiles over a short K range: one wave per tile, K not split at all
        static const int wpt = tune_int("LORA_DEC_WAVE_PER_TILE", -1, -1, 1);
        static const int wpt_tiles = tune_int("LORA_DEC_WAVE_PER_TILE_MIN_TILES", 4096, 1, 1 << 20);
        static const int wpt_k = tune_int("LORA_DEC_WAVE_PER_TILE_MAX_K", 4096, 32, 1 << 20);
        if (wpt == 1 || (wpt < 0 && tub >= wpt_tiles && p->d.proj[proj].h_in <= wpt_k)) {
            KSplit k;
            k.kb_per_part = kblocks;
            k.n_parts = 1;
            k.wave_per_tile = true;
            return k;
        }
        int n = std::max(1, (kblocks + kb_target - 1) / kb_target);
        n = std::max<int>(n, (int)std::min<int64_t>((want_wgs + tub - 1) / tub, kblocks / 4));
        n = std::min(std::max(n, 1), max_parts);
        int per = ((kblocks + n - 1) / n + 3) / 4 * 4;
        KSplit k;
        k.kb_per_part = per;
        k.n_parts = (kblocks + per - 1) / per;
        k.wave_per_tile = false;
        return k;
    }
    // long segments: work items are groups of tiles; enough K parts to fill the chip
    const int64_t tub = std::max<int64_t>(1, tiles_upper_bound(p, P, kTileRows));
    const int64_t groups = (tub + shrink_long_tiles() - 1) / shrink_long_tiles();
    static const int target = tune_int("LORA_SHRINK_ITEMS", 512, 1, 1 << 20);
    int want = (int)std::min<int64_t>((target + groups - 1) / groups, kMaxParts);
    int by_size = (kblocks + kPartKBlocks - 1) / kPartKBlocks;
    int n = std::max(want, by_size);
    n = std::min(n, std::max(1, kblocks / 4));
    n = std::min(n, kMaxParts);
    int per = (kblocks + n - 1) / n;
    per = (per + 3) / 4 * 4;
    KSplit k;
    k.kb_per_part = per;
    k.n_parts = (kblocks + per - 1) / per;
    k.wave_per_tile = false;
    return k;
}

// Segments are only meaningful together with the pool they were built for: the keys index that
// pool's table, and the kernel family and the workspace layout follow from (pool, P).
int check_segments(const lora_pool *pool, const lora_segments *s)
{
    if (!s) return LORA_ERR_INVALID_ARG;
    if (s->P < 0 || (s->tile_rows != kTileRows && s->tile_rows != kDecodeTileRows))
        return LORA_ERR_NOT_REGISTERED;
    if ((int64_t)s->n_keys != (int64_t)pool->d.n_adapters * pool->d.n_experts ||
        s->tile_rows != pick_tile_rows(pool, s->P))
        return LORA_ERR_NOT_REGISTERED;
    if (s->P > 0 && (!s->perm || !s->seg_start || !s->seg_key || !s->tiles || !s->counts || !s->status))
        return LORA_ERR_INVALID_ARG;
    return LORA_OK;
}

// A group of n consecutive projections proj0 .. proj0+n-1 that read the same input (same
// h_in): per projection its slice of the intermediate, its output and the output's stride.
struct Group {
    int proj0, n;
    float *v[kMaxFused];
    void *y[kMaxFused];
    int64_t ldy[kMaxFused];
    int overwrite;           // bf16 decode expand: write the update instead of adding it to y
};

// bytes of the K parts of one projection's intermediate
size_t parts_bytes(const lora_pool *pool, int n_parts, int P)
{
    return align_up((size_t)n_parts * std::max(P, 1) * pool->d.rank * sizeof(float), 256);
}

// launch parameters of the shrink of a group (decode kernels: complete; long kernels: all but
// the per-launch projection fields)
// Cache hints of the activation streams (the weights are always streamed: they are read once).
// x rows that every pair reads for itself (no gather through src_row) are read exactly once, so
// keeping them cacheable pays only while they are small against the memory-side cache: a quarter
// of it and more is streamed, so that it does not push out the output rows, which are read,
// written and read again by whatever runs next.  Output rows, and read-once input rows of any
// size, are streamed when the caller says its activations are not in a cache when a call starts
// (LORA_ACT_STREAMING); output rows also when one call's outputs exceed the memory-side cache
// anyway.  LORA_ACT_RESIDENT switches both off.
bool stream_x(const lora_pool *pool, const int32_t *src_row, int64_t x_bytes)
{
    static const int mb = tune_int("LORA_X_STREAM_MB", kStreamXMiB, 1, 1 << 20);
    if (pool->act_policy == LORA_ACT_RESIDENT || src_row) return false;
    if (pool->act_policy == LORA_ACT_STREAMING) return true;
    return x_bytes >= (int64_t)mb << 20;
}

bool stream_y(const lora_pool *pool, int64_t y_bytes)
{
    static const int mb = tune_int("LORA_Y_STREAM_MB", kStreamYMiB, 1, 1 << 20);
    if (pool->act_policy == LORA_ACT_RESIDENT) return false;
    return pool->act_policy == LORA_ACT_STREAMING || y_bytes >= (int64_t)mb << 20;
}

ShrinkParams shrink_params(const lora_pool *pool, int layer, const Group &g, const void *x, int64_t ldx,
                           const int32_t *src_row, const lora_segments *seg)
{
    const lora_proj_desc &pd = pool->d.proj[g.proj0];
    const KSplit ks = ksplit_of(pool, g.proj0, seg->P);
    ShrinkParams sp;
    memset(&sp, 0, sizeof sp);
    sp.units = pool->device_table() + pool->table_index(layer, 0, 0, 0);
    sp.n_proj = pool->d.n_proj;
    sp.x = static_cast<const uint16_t *>(x);
    sp.ldx = ldx;
    sp.src_row = src_row;
    sp.perm = seg->perm;
    sp.tiles = seg->tiles;
    sp.counts = seg->counts;
    sp.P = seg->P;
    sp.h_in = pd.h_in;
    sp.n_parts = ks.n_parts;
    sp.kb_per_part = ks.kb_per_part;
    sp.rank = pool->d.rank;
    const int64_t items = tiles_upper_bound(pool, seg->P, seg->tile_rows) * ks.n_parts;
    if (seg->tile_rows == kDecodeTileRows) {
        static const int per_cu = tune_int("LORA_DEC_SHRINK_WGS_PER_CU", 8, 1, 64);
        sp.proj0 = g.proj0;
        sp.n_fused = g.n;
        for (int j = 0; j < g.n; ++j) sp.v[j] = g.v[j];
        sp.wave_per_tile = ks.wave_per_tile;
        sp.x_stream = !ks.wave_per_tile && stream_x(pool, src_row, (int64_t)seg->P * pd.h_in * 2);
        const int64_t wgs = ks.wave_per_tile ? (items + 3) / 4 : items;
        sp.grid = (int)std::min<int64_t>(wgs, (int64_t)cu_count() * per_cu);
        return sp;
    }
    // 32-row tiles: work items are groups of tiles; at most two projections per launch
    static const int per_cu = tune_int("LORA_SHRINK_WGS_PER_CU", 2, 1, 64);
    const int64_t groups = (tiles_upper_bound(pool, seg->P, seg->tile_rows) + shrink_long_tiles() - 1) /
                           shrink_long_tiles();
    sp.grid = (int)std::min<int64_t>(groups * ks.n_parts, (int64_t)cu_count() * per_cu);
    return sp;
}

int do_shrink(const lora_pool *pool, int layer, const Group &g, const void *x, int64_t ldx,
              const int32_t *src_row, const lora_segments *seg, hipStream_t st,
              const SegParams *build = nullptr)
{
    ShrinkParams sp = shrink_params(pool, layer, g, x, ldx, src_row, seg);
    if (seg->tile_rows == kDecodeTileRows) {
        if (build) {
            // every workgroup sorts the batch before its first item: fewer, longer-lived workgroups
            static const int per_cu = tune_int("LORA_INLINE_BUILD_WGS_PER_CU", 4, 1, 64);
            sp.build = 1;
            sp.x_stream = 0;                      // at most 2048 rows: nothing to stream
            sp.seg = *build;
            sp.grid = (int)std::min<int64_t>(sp.grid, (int64_t)cu_count() * per_cu);
        }
        LORA_HIP(launch_shrink_decode(sp, st));
        return LORA_OK;
    }
    if (build) return LORA_ERR_INVALID_ARG;       // the caller checks inline_build_ok first
    for (int j = 0; j < g.n; j += 2) {
        sp.proj0 = g.proj0 + j;
        sp.n_fused = std::min(2, g.n - j);
        sp.v[0] = g.v[j];
        sp.v[1] = sp.n_fused == 2 ? g.v[j + 1] : nullptr;
        LORA_HIP(launch_shrink(sp, st));
    }
    return LORA_OK;
}

int expand_params(const lora_pool *pool, int layer, const Group &g, const lora_segments *seg,
                  int out_dtype, ExpandParams &ep);

int do_expand(const lora_pool *pool, int layer, const Group &g, const lora_segments *seg,
              int out_dtype, hipStream_t st)
{
    ExpandParams ep;
    expand_params(pool, layer, g, seg, out_dtype, ep);
    if (seg->tile_rows == kDecodeTileRows)
        LORA_HIP(launch_expand_decode(ep, st));
    else
        LORA_HIP(launch_expand(ep, st));
    return LORA_OK;
}

// launch parameters of the expand of a group
int expand_params(const lora_pool *pool, int layer, const Group &g, const lora_segments *seg,
                  int out_dtype, ExpandParams &ep)
{
    const KSplit ks = ksplit_of(pool, g.proj0, seg->P);
    memset(&ep, 0, sizeof ep);
    ep.units = pool->device_table() + pool->table_index(layer, 0, 0, 0);
    ep.n_proj = pool->d.n_proj;
    ep.n_parts = ks.n_parts;
    ep.P = seg->P;
    ep.perm = seg->perm;
    ep.tiles = seg->tiles;
    ep.counts = seg->counts;
    ep.out_f32 = out_dtype == LORA_DTYPE_F32;
    ep.rank = pool->d.rank;
    const int64_t tub = std::max<int64_t>(1, tiles_upper_bound(pool, seg->P, seg->tile_rows));
    if (seg->tile_rows == kDecodeTileRows) {
        // every wave works alone on wave items = (tile, projection, slice of 128-column chunks).
        // Chunks per item: an item should move about item_bytes (its prologue - row indices, v -
        // costs a few load latencies), but a small batch must still yield a few thousand items;
        // the grid holds several times more workgroups than are resident, so that the hardware
        // hands out items as waves finish and tiles of different heights balance out.
        static const int cpi_max = tune_int("LORA_DEC_CHUNKS_PER_ITEM", 8, 1, 4096);
        static const int item_bytes = tune_int("LORA_DEC_ITEM_BYTES", 12288, 1024, 1 << 24);
        static const int want_items = tune_int("LORA_DEC_EXPAND_ITEMS", 4096, 1, 1 << 22);
        static const int per_cu = tune_int("LORA_DEC_EXPAND_WGS_PER_CU", 16, 1, 64);
        ep.proj0 = g.proj0;
        ep.n_fused = g.n;
        ep.overwrite = g.overwrite && out_dtype == LORA_DTYPE_BF16;
        {
            int64_t y_bytes = 0;
            for (int j = 0; j < g.n; ++j)
                y_bytes += (int64_t)seg->P * pool->d.proj[g.proj0 + j].h_out * (ep.out_f32 ? 4 : 2);
            ep.y_stream = stream_y(pool, y_bytes);
        }
        int64_t chunks_per_tile = 0;
        for (int j = 0; j < g.n; ++j) chunks_per_tile += chunks_of(pool->d.proj[g.proj0 + j].h_out);
        const int64_t units = tub * chunks_per_tile;
        // bytes of one chunk of an average tile: its B plus the read-modify-write of its rows
        const double rows_per_tile = (double)seg->P / (double)tub;
        const double chunk_bytes = kColChunk * pool->d.rank * 2.0 +
                                   rows_per_tile * kColChunk * (out_dtype == LORA_DTYPE_F32 ? 8.0 : 4.0);
        // at least two chunks (the kernel keeps two in flight) unless the batch is so small
        // that single-chunk items are needed to occupy the chip
        int cpi = std::max(2, (int)std::lround(item_bytes / chunk_bytes));
        cpi = (int)std::max<int64_t>(1, std::min<int64_t>(std::min(cpi, cpi_max), units / want_items));
        ep.slice0[0] = 0;
        for (int j = 0; j < g.n; ++j) {
            ep.v[j] = g.v[j];
            ep.y[j] = g.y[j];
            ep.ldy[j] = g.ldy[j];
            ep.h_out[j] = pool->d.proj[g.proj0 + j].h_out;
            ep.n_chunks[j] = chunks_of(ep.h_out[j]);
            // no empty slice: a row is cut into n_slices pieces of cps = ceil(n_chunks / n_slices)
            // chunks; cps even, because the kernel keeps two chunks in flight with unconditional
            // loads and a piece of odd length costs it one chunk loaded twice
            const int want = std::max(1, (ep.n_chunks[j] + cpi - 1) / cpi);
            int cps = (ep.n_chunks[j] + want - 1) / want;
            if (cpi > 1) cps = std::min(ep.n_chunks[j], (cps + 1) & ~1);     // cpi 1: a small batch, items first
            ep.cps[j] = cps;
            ep.n_slices[j] = (ep.n_chunks[j] + cps - 1) / cps;
            ep.slice0[j + 1] = ep.slice0[j] + ep.n_slices[j];
        }
        for (int j = g.n; j < kMaxFused; ++j) ep.slice0[j + 1] = ep.slice0[g.n];
        ep.waves = 4;
        // with many rows per (adapter, expert) a segment spans several tiles: let neighbouring
        // waves take neighbouring tiles, so that they share the segment's B through the L2
        static const int tile_group = tune_int("LORA_DEC_EXPAND_TILE_GROUP", 0, 0, 4);
        const int64_t n_keys = (int64_t)pool->d.n_adapters * pool->d.n_experts;
        ep.tile_group = tile_group ? tile_group : (seg->P >= 8 * n_keys ? 2 : 1);
        const int64_t wave_items = (tub + ep.tile_group - 1) / ep.tile_group * ep.tile_group * ep.slice0[g.n];
        ep.grid = (int)std::min<int64_t>((wave_items + ep.waves - 1) / ep.waves,
                                         (int64_t)cu_count() * per_cu);
        return LORA_OK;
    }
    // long segments: operand images of the sub-tiles behind the K parts in each projection's
    // slice of the workspace, then wave items = (group of tiles, projection, 128-column chunk)
    static const int per_cu = tune_int("LORA_EXPAND_WGS_PER_CU", 32, 1, 64);
    ep.proj0 = g.proj0;
    ep.n_fused = g.n;
    ep.slice0[0] = 0;
    for (int j = 0; j < g.n; ++j) {
        ep.v[j] = g.v[j];
        ep.y[j] = g.y[j];
        ep.ldy[j] = g.ldy[j];
        ep.h_out[j] = pool->d.proj[g.proj0 + j].h_out;
        ep.n_chunks[j] = chunks_of(ep.h_out[j]);
        ep.n_slices[j] = ep.n_chunks[j];
        ep.slice0[j + 1] = ep.slice0[j] + ep.n_chunks[j];
        ep.img[j] = reinterpret_cast<char *>(g.v[j]) + parts_bytes(pool, ks.n_parts, seg->P);
    }
    for (int j = g.n; j < kMaxFused; ++j) ep.slice0[j + 1] = ep.slice0[g.n];
    ep.waves = 4;
    const int64_t groups = (tub + expand_long_group() - 1) / expand_long_group();
    const int64_t wave_items = groups * ep.slice0[g.n];
    ep.grid = (int)std::min<int64_t>((wave_items + 3) / 4, (int64_t)cu_count() * per_cu);
    ep.image_grid = (int)std::min<int64_t>((tub * 2 * g.n + 3) / 4, (int64_t)cu_count() * 8);
    return LORA_OK;
}

// Shrink and expand of a group as one launch (fused_decode.hip): every workgroup repeats the
// shrink of its tile and projection and expands a slice of the output columns, so the launch
// needs no hand-off between workgroups but reads A once per slice (from the L2 after the first).
// Worth it only for small decode batches with short inputs: few tiles (the repeated reads stay
// small against the bytes of B and y, and a second launch would cost more than it moves) and a
// K range that four waves get through quickly.  Returns false if the group is not eligible;
// otherwise fills the slicing of ep (n_slices, cps, slice0) and the grid.
bool fused_plan(const lora_pool *pool, const Group &g, const lora_segments *seg, int out_dtype,
                ShrinkParams *sp, ExpandParams *ep)
{
    static const int enabled = tune_int("LORA_FUSED", 1, 0, 1);
    static const int max_k = tune_int("LORA_FUSED_MAX_K", kFusedMaxK, 8, 1 << 20);
    static const int max_tiles = tune_int("LORA_FUSED_MAX_TILES", kFusedMaxTiles, 1, 1 << 20);
    static const int min_chunks = tune_int("LORA_FUSED_MIN_CHUNKS", kFusedMinChunks, 1, 1 << 20);
    static const int want_wgs = tune_int("LORA_FUSED_WGS", kFusedWorkgroups, 1, 1 << 20);
    if (!enabled || seg->tile_rows != kDecodeTileRows || out_dtype != LORA_DTYPE_BF16 || g.overwrite)
        return false;
    if (pool->d.proj[g.proj0].h_in > max_k) return false;
    {
        static const int max_chunks = tune_int("LORA_FUSED_MAX_CHUNKS", kFusedMaxChunks, 1, 1 << 20);
        int chunks = 0;
        for (int j = 0; j < g.n; ++j) chunks += chunks_of(pool->d.proj[g.proj0 + j].h_out);
        if (chunks > max_chunks) return false;
    }
    const int64_t tub = std::max<int64_t>(1, tiles_upper_bound(pool, seg->P, kDecodeTileRows));
    if (tub > max_tiles) return false;
    if (!sp || !ep) return true;
    // slices per projection: enough workgroups to occupy the chip, but at least min_chunks
    // chunks per slice (a workgroup repeats a whole shrink for them)
    int total_chunks = 0;
    for (int j = 0; j < g.n; ++j) total_chunks += chunks_of(pool->d.proj[g.proj0 + j].h_out);
    const double per_tile = std::max(1.0, (double)want_wgs / (double)tub);
    ep->slice0[0] = 0;
    for (int j = 0; j < g.n; ++j) {
        const int n = chunks_of(pool->d.proj[g.proj0 + j].h_out);
        int slices = (int)std::lround(per_tile * n / total_chunks);
        slices = std::max(1, std::min(slices, std::max(1, n / min_chunks)));
        int cps = (n + slices - 1) / slices;
        cps = std::min(n, (cps + 1) & ~1);                      // even: two chunks are in flight
        ep->cps[j] = cps;
        ep->n_slices[j] = (n + cps - 1) / cps;
        ep->slice0[j + 1] = ep->slice0[j] + ep->n_slices[j];
    }
    for (int j = g.n; j < kMaxFused; ++j) ep->slice0[j + 1] = ep->slice0[g.n];
    sp->n_parts = 1;
    sp->kb_per_part = kblocks_of(pool->d.proj[g.proj0].h_in, pool->d.rank);
    ep->n_parts = 1;
    sp->grid = (int)std::min<int64_t>(tub * ep->slice0[g.n], (int64_t)cu_count() * 8);
    return true;
}

// Can the shrink of this group sort the batch itself (segments_inline.h) instead of waiting for
// a launch of the segment builder?  Small decode batches of at most 256 keys, on the K-split
// shrink kernel or on the kernel that runs shrink and expand as one launch (the whole call of a
// small batch is then a single launch).
bool inline_build_ok(const lora_pool *pool, const Group &g, const lora_segments *seg, int out_dtype)
{
    static const int enabled = tune_int("LORA_INLINE_BUILD", 1, 0, 1);
    if (!enabled || seg->P <= 0 || seg->P > inline_build_max_rows() ||
        (int64_t)pool->d.n_adapters * pool->d.n_experts > inline_build_max_keys())
        return false;
    if (seg->tile_rows != kDecodeTileRows) return false;
    // the one-launch kernel and the K-split shrink can; the wave-per-tile shrink cannot
    return fused_plan(pool, g, seg, out_dtype, nullptr, nullptr) || !ksplit_of(pool, g.proj0, seg->P).wave_per_tile;
}

// shrink then expand of a group: one launch where that is possible, else two.  `build`: the
// segments of this batch have not been built yet; the shrink does it where it can, else the
// segment builder is launched first.
int do_apply(const lora_pool *pool, int layer, const Group &g, const void *x, int64_t ldx,
             const int32_t *src_row, const lora_segments *seg, int out_dtype, hipStream_t st,
             const SegParams *build = nullptr, void *build_ws = nullptr)
{
    if (build && !inline_build_ok(pool, g, seg, out_dtype)) {
        LORA_HIP(launch_segments(*build, build_ws, st));
        build = nullptr;
    }
    if (fused_plan(pool, g, seg, out_dtype, nullptr, nullptr)) {
        FusedParams fp;
        memset(&fp, 0, sizeof fp);
        fp.s = shrink_params(pool, layer, g, x, ldx, src_row, seg);
        expand_params(pool, layer, g, seg, out_dtype, fp.e);
        fused_plan(pool, g, seg, out_dtype, &fp.s, &fp.e);
        if (build) {
            fp.s.build = 1;
            fp.s.seg = *build;
        }
        LORA_HIP(launch_fused_decode(fp, st));
        return LORA_OK;
    }
    int rc = do_shrink(pool, layer, g, x, ldx, src_row, seg, st, build);
    if (rc != LORA_OK) return rc;
    return do_expand(pool, layer, g, seg, out_dtype, st);
}

Group single(int proj, float *v, void *y, int64_t ldy)
{
    Group g;
    memset(&g, 0, sizeof g);
    g.proj0 = proj;
    g.n = 1;
    g.v[0] = v;
    g.y[0] = y;
    g.ldy[0] = ldy;
    return g;
}

int check_act(const void *ptr, int64_t ld, int width, size_t elem)
{
    if (!ptr) return LORA_ERR_INVALID_ARG;
    if (!aligned(ptr, 16)) return LORA_ERR_MISALIGNED;
    if (ld < width || (ld % 8) != 0) return LORA_ERR_BAD_SHAPE;
    (void)elem;
    return LORA_OK;
}

}  // namespace

extern "C" {

const char *lora_strerror(int status)
{
    switch (status) {
    case LORA_OK: return "ok";
    case LORA_ERR_INVALID_ARG: return "invalid argument";
    case LORA_ERR_BAD_SHAPE: return "bad shape, leading dimension or index";
    case LORA_ERR_UNSUPPORTED_RANK: return "unsupported LoRA rank (supported: 8, 16, 32, 64)";
    case LORA_ERR_BUFFER_TOO_SMALL: return "buffer smaller than its size query";
    case LORA_ERR_NOT_REGISTERED: return "pool not registered or segments not built";
    case LORA_ERR_HIP: return "HIP runtime error";
    case LORA_ERR_MISALIGNED: return "misaligned pointer";
    case LORA_ERR_TOO_LARGE: return "batch or key space too large";
    default: return "unknown status";
    }
}

const char *lora_last_hip_error(void) { return g_hip_error.c_str(); }

size_t lora_pool_bytes(const lora_pool_desc *d)
{
    if (check_desc(d) != LORA_OK) return 0;
    return layout_of(*d).total;
}

int lora_register_pool(const lora_pool_desc *d, void *slab, size_t slab_bytes,
                       const void *const *A_src, const void *const *B_src, void *stream,
                       lora_pool **out)
{
    if (!out) return LORA_ERR_INVALID_ARG;
    *out = nullptr;
    int rc = check_desc(d);
    if (rc != LORA_OK) return rc;
    if (!slab) return LORA_ERR_INVALID_ARG;
    if ((A_src == nullptr) != (B_src == nullptr)) return LORA_ERR_INVALID_ARG;
    if (!aligned(slab, 256)) return LORA_ERR_MISALIGNED;
    const Layout L = layout_of(*d);
    if (slab_bytes < L.total) return LORA_ERR_BUFFER_TOO_SMALL;
    const size_t n_src = (size_t)d->n_adapters * d->n_layers * d->n_experts * d->n_proj;
    if (A_src)
        for (size_t i = 0; i < n_src; ++i) {
            if (!A_src[i] || !B_src[i]) return LORA_ERR_INVALID_ARG;
            if (!aligned(A_src[i], 2) || !aligned(B_src[i], 2)) return LORA_ERR_MISALIGNED;
        }

    lora_pool *p = new (std::nothrow) lora_pool();
    if (!p) return LORA_ERR_INVALID_ARG;
    p->magic = kPoolMagic;
    p->act_policy = LORA_ACT_AUTO;
    p->d = *d;
    p->scale.assign(d->n_adapters, 1.0f);
    if (d->scale) p->scale.assign(d->scale, d->scale + d->n_adapters);
    p->arank.assign(d->n_adapters, d->rank);
    if (d->adapter_rank) p->arank.assign(d->adapter_rank, d->adapter_rank + d->n_adapters);
    p->d.scale = nullptr;
    p->d.adapter_rank = nullptr;
    p->slab = static_cast<char *>(slab);
    p->slab_bytes = slab_bytes;
    p->table_bytes = L.table_bytes;
    p->unit_bytes = L.unit_bytes;
    for (int i = 0; i < d->n_proj; ++i) {
        p->A_off[i] = L.A_off[i];
        p->A_bytes[i] = L.A_bytes[i];
        p->B_off[i] = L.B_off[i];
        p->B_bytes[i] = L.B_bytes[i];
    }
    p->table.resize((size_t)d->n_layers * d->n_adapters * d->n_experts * d->n_proj);
    for (int l = 0; l < d->n_layers; ++l)
        for (int a = 0; a < d->n_adapters; ++a)
            for (int e = 0; e < d->n_experts; ++e)
                for (int j = 0; j < d->n_proj; ++j) {
                    Unit &u = p->table[p->table_index(l, a, e, j)];
                    const size_t base = p->unit_base(l, a, e);
                    u.A = reinterpret_cast<const uint16_t *>(p->slab + base + L.A_off[j]);
                    u.B = reinterpret_cast<const uint16_t *>(p->slab + base + L.B_off[j]);
                    u.scale = p->scale[a];
                    u.rank = p->arank[a];
                    u.pad[0] = u.pad[1] = 0;
                }

    {
        // set-up of this device: the address of the static workspace of lora_moe_apply_static
        void *unused = nullptr;
        rc = static_scratch(&unused);
        if (rc != LORA_OK) {
            p->magic = 0;
            delete p;
            return rc;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipMemcpyAsync(p->slab, p->table.data(), p->table.size() * sizeof(Unit),
                                  hipMemcpyHostToDevice, st);
    if (e == hipSuccess && !A_src)
        e = hipMemsetAsync(p->slab + L.table_bytes, 0, L.total - L.table_bytes, st);
    if (e != hipSuccess) {
        p->magic = 0;
        delete p;
        return hip_fail(e);
    }
    if (A_src) {
        size_t i = 0;
        for (int a = 0; a < d->n_adapters; ++a)
            for (int l = 0; l < d->n_layers; ++l)
                for (int ex = 0; ex < d->n_experts; ++ex)
                    for (int j = 0; j < d->n_proj; ++j, ++i) {
                        rc = lora_pool_load_unit(p, a, l, ex, j, A_src[i], B_src[i], stream);
                        if (rc != LORA_OK) {
                            p->magic = 0;
                            delete p;
                            return rc;
                        }
                    }
    }
    *out = p;
    return LORA_OK;
}

int lora_pool_load_unit(lora_pool *pool, int adapter, int layer, int expert, int proj,
                        const void *A, const void *B, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, layer, expert, proj);
    if (rc != LORA_OK) return rc;
    if (!A || !B) return LORA_ERR_INVALID_ARG;
    if (!aligned(A, 2) || !aligned(B, 2)) return LORA_ERR_MISALIGNED;
    const size_t base = pool->unit_base(layer, adapter, expert);
    hipStream_t st = static_cast<hipStream_t>(stream);
    PackParams pp;
    pp.src = static_cast<const uint16_t *>(A);
    pp.src_stride = 0;
    pp.dst = reinterpret_cast<uint16_t *>(pool->slab + base + pool->A_off[proj]);
    pp.dst_stride = 0;
    pp.n_units = 1;
    pp.h = pool->d.proj[proj].h_in;
    pp.rank = pool->d.rank;
    pp.src_rank = pool->arank[adapter];
    LORA_HIP(launch_pack_A(pp, st));
    pp.src = static_cast<const uint16_t *>(B);
    pp.dst = reinterpret_cast<uint16_t *>(pool->slab + base + pool->B_off[proj]);
    pp.h = pool->d.proj[proj].h_out;
    LORA_HIP(launch_pack_B(pp, st));
    return LORA_OK;
}

int lora_pool_load_adapter_layer(lora_pool *pool, int adapter, int layer, const void *src,
                                 void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, layer, 0, 0);
    if (rc != LORA_OK) return rc;
    if (!src) return LORA_ERR_INVALID_ARG;
    if (!aligned(src, 2)) return LORA_ERR_MISALIGNED;
    const int r = pool->arank[adapter];
    int64_t unit_elems = 0;
    for (int j = 0; j < pool->d.n_proj; ++j)
        unit_elems += ((int64_t)pool->d.proj[j].h_in + pool->d.proj[j].h_out) * r;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t base = pool->unit_base(layer, adapter, 0);
    PackLayerParams ps;
    memset(&ps, 0, sizeof ps);
    ps.n_jobs = 2 * pool->d.n_proj;
    int64_t off = 0;
    for (int j = 0; j < pool->d.n_proj; ++j) {
        PackParams pp;
        pp.src = static_cast<const uint16_t *>(src) + off;
        pp.src_stride = unit_elems;
        pp.dst = reinterpret_cast<uint16_t *>(pool->slab + base + pool->A_off[j]);
        pp.dst_stride = (int64_t)(pool->unit_bytes / 2);
        pp.n_units = pool->d.n_experts;
        pp.h = pool->d.proj[j].h_in;
        pp.rank = pool->d.rank;
        pp.src_rank = r;
        ps.job[2 * j] = pp;
        off += (int64_t)pool->d.proj[j].h_in * r;
        pp.src = static_cast<const uint16_t *>(src) + off;
        pp.dst = reinterpret_cast<uint16_t *>(pool->slab + base + pool->B_off[j]);
        pp.h = pool->d.proj[j].h_out;
        ps.job[2 * j + 1] = pp;
        off += (int64_t)pool->d.proj[j].h_out * r;
    }
    LORA_HIP(launch_pack_layer(ps, st));      // one launch for all projections and experts
    return LORA_OK;
}

int lora_pool_set_adapter(lora_pool *pool, int adapter, int rank, float scale, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, 0, 0, 0);
    if (rc != LORA_OK) return rc;
    if (rank < 1 || rank > pool->d.rank) return LORA_ERR_UNSUPPORTED_RANK;
    if (!(scale == scale)) return LORA_ERR_INVALID_ARG;            // NaN
    const int per_adapter = pool->d.n_experts * pool->d.n_proj;
    LORA_HIP(launch_set_adapter(reinterpret_cast<Unit *>(pool->slab), pool->d.n_layers, pool->d.n_adapters,
                                per_adapter, adapter, rank, scale, static_cast<hipStream_t>(stream)));
    pool->arank[adapter] = rank;
    pool->scale[adapter] = scale;
    for (int l = 0; l < pool->d.n_layers; ++l)
        for (int k = 0; k < per_adapter; ++k) {
            Unit &u = pool->table[pool->table_index(l, adapter, 0, 0) + k];
            u.rank = rank;
            u.scale = scale;
        }
    return LORA_OK;
}

int lora_pool_set_activation_policy(lora_pool *pool, int policy)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    if (policy != LORA_ACT_AUTO && policy != LORA_ACT_RESIDENT && policy != LORA_ACT_STREAMING)
        return LORA_ERR_INVALID_ARG;
    pool->act_policy = policy;
    return LORA_OK;
}

int lora_pool_activation_policy(const lora_pool *pool)
{
    int rc = check_pool(pool);
    return rc != LORA_OK ? rc : pool->act_policy;
}

size_t lora_pool_adapter_layer_bytes(const lora_pool *pool, int adapter)
{
    if (check_pool(pool) != LORA_OK || check_unit(pool, adapter, 0, 0, 0) != LORA_OK) return 0;
    const int r = pool->arank[adapter];
    size_t elems = 0;
    for (int j = 0; j < pool->d.n_proj; ++j)
        elems += ((size_t)pool->d.proj[j].h_in + pool->d.proj[j].h_out) * r;
    return elems * pool->d.n_experts * sizeof(uint16_t);
}

int lora_pool_load_adapter_async(lora_pool *pool, int adapter, const void *host_src, void *staging,
                                 size_t staging_bytes, void *load_stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, 0, 0, 0);
    if (rc != LORA_OK) return rc;
    if (!host_src || !staging) return LORA_ERR_INVALID_ARG;
    if (!aligned(host_src, 2) || !aligned(staging, 16)) return LORA_ERR_MISALIGNED;
    const size_t window = lora_pool_adapter_layer_bytes(pool, adapter);
    if (staging_bytes < window) return LORA_ERR_BUFFER_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(load_stream);
    const int n_layers = pool->d.n_layers;
    if (pool->ready.empty()) pool->ready.assign((size_t)pool->d.n_adapters * n_layers, nullptr);
    for (int l = 0; l < n_layers; ++l) {
        hipEvent_t &ev = pool->ready[(size_t)adapter * n_layers + l];
        if (!ev) LORA_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        // one staging window: the copy of layer l+1 is ordered behind the repack of layer l
        LORA_HIP(hipMemcpyAsync(staging, static_cast<const char *>(host_src) + (size_t)l * window, window,
                                hipMemcpyHostToDevice, st));
        rc = lora_pool_load_adapter_layer(pool, adapter, l, staging, load_stream);
        if (rc != LORA_OK) return rc;
        LORA_HIP(hipEventRecord(ev, st));
    }
    return LORA_OK;
}

int lora_pool_wait_layer(const lora_pool *pool, int adapter, int layer, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, layer, 0, 0);
    if (rc != LORA_OK) return rc;
    if (pool->ready.empty()) return LORA_OK;
    hipEvent_t ev = pool->ready[(size_t)adapter * pool->d.n_layers + layer];
    if (!ev) return LORA_OK;
    LORA_HIP(hipStreamWaitEvent(static_cast<hipStream_t>(stream), ev, 0));
    return LORA_OK;
}

int lora_pool_layer_ready(const lora_pool *pool, int adapter, int layer)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, layer, 0, 0);
    if (rc != LORA_OK) return rc;
    if (pool->ready.empty()) return 1;
    hipEvent_t ev = pool->ready[(size_t)adapter * pool->d.n_layers + layer];
    if (!ev) return 1;
    const hipError_t e = hipEventQuery(ev);
    if (e == hipSuccess) return 1;
    if (e == hipErrorNotReady) {
        (void)hipGetLastError();          // "not ready" is an answer, not an error to leave behind
        return 0;
    }
    LORA_HIP(e);
    return LORA_ERR_HIP;
}

int lora_pool_read_unit(const lora_pool *pool, int adapter, int layer, int expert, int proj,
                        void *A_out, void *B_out, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, layer, expert, proj);
    if (rc != LORA_OK) return rc;
    if (!A_out || !B_out) return LORA_ERR_INVALID_ARG;
    const size_t base = pool->unit_base(layer, adapter, expert);
    hipStream_t st = static_cast<hipStream_t>(stream);
    PackParams pp;
    pp.src = reinterpret_cast<const uint16_t *>(pool->slab + base + pool->A_off[proj]);
    pp.src_stride = 0;
    pp.dst = static_cast<uint16_t *>(A_out);
    pp.dst_stride = 0;
    pp.n_units = 1;
    pp.h = pool->d.proj[proj].h_in;
    pp.rank = pool->d.rank;
    pp.src_rank = pool->d.rank;
    LORA_HIP(launch_unpack_A(pp, st));
    pp.src = reinterpret_cast<const uint16_t *>(pool->slab + base + pool->B_off[proj]);
    pp.dst = static_cast<uint16_t *>(B_out);
    pp.h = pool->d.proj[proj].h_out;
    LORA_HIP(launch_unpack_B(pp, st));
    return LORA_OK;
}

int lora_pool_unit_layout(const lora_pool *pool, int adapter, int layer, int expert, int proj,
                          size_t *A_offset, size_t *A_bytes, size_t *B_offset, size_t *B_bytes,
                          int32_t *rank, float *scale)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_unit(pool, adapter, layer, expert, proj);
    if (rc != LORA_OK) return rc;
    const size_t base = pool->unit_base(layer, adapter, expert);
    if (A_offset) *A_offset = base + pool->A_off[proj];
    if (A_bytes) *A_bytes = pool->A_bytes[proj];
    if (B_offset) *B_offset = base + pool->B_off[proj];
    if (B_bytes) *B_bytes = pool->B_bytes[proj];
    if (rank) *rank = pool->arank[adapter];
    if (scale) *scale = pool->scale[adapter];
    return LORA_OK;
}

const void *lora_pool_device_table(const lora_pool *pool)
{
    if (check_pool(pool) != LORA_OK) return nullptr;
    return pool->slab;
}

int lora_pool_destroy(lora_pool *pool)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    pool->magic = 0;
    for (hipEvent_t e : pool->ready)
        if (e) (void)hipEventDestroy(e);
    delete pool;
    return LORA_OK;
}

size_t lora_segments_ws_bytes(int P)
{
    if (P < 0) return 0;
    // a single workgroup sorts out of LDS; the multi-workgroup builder of long batches keeps
    // its per-chunk counts here
    return std::max<size_t>(256, segments_large_ws_bytes(P));
}

static int key_bits_of(const lora_pool *pool)
{
    const uint32_t n_keys = (uint32_t)pool->d.n_adapters * (uint32_t)pool->d.n_experts;
    int bits = 1;
    while (((n_keys - 1) >> bits) != 0) ++bits;    // bits of the largest key
    return bits;
}

int lora_segments_launches(const lora_pool *pool, int P)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    if (P < 0) return LORA_ERR_INVALID_ARG;
    SegParams sp;
    memset(&sp, 0, sizeof sp);
    sp.P = P;
    sp.key_bits = key_bits_of(pool);
    sp.passes = (sp.key_bits + 7) / 8;
    return segments_large_handles(sp) ? segments_large_launches(sp) : 1;
}

// checks of lora_build_segments; fills the launch parameters and the host fields of `seg`
static int prepare_segments(const lora_pool *pool, const int32_t *adapter_id, const int32_t *expert_id,
                            int P, lora_segments *seg, void *ws, size_t ws_bytes, SegParams &sp)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    if (!seg || P < 0) return LORA_ERR_INVALID_ARG;
    if (!seg->counts || !seg->status) return LORA_ERR_INVALID_ARG;
    if (P > LORA_MAX_ROWS_LONG) return LORA_ERR_TOO_LARGE;
    if (P > 0) {
        if (!adapter_id || !seg->perm || !seg->seg_start || !seg->seg_key || !seg->tiles || !ws)
            return LORA_ERR_INVALID_ARG;
        if (pool->d.n_experts > 1 && !expert_id) return LORA_ERR_INVALID_ARG;
        if (!aligned(ws, 16) || !aligned(seg->tiles, 16)) return LORA_ERR_MISALIGNED;
        if (ws_bytes < lora_segments_ws_bytes(P)) return LORA_ERR_BUFFER_TOO_SMALL;
    }
    memset(&sp, 0, sizeof sp);
    sp.adapter_id = adapter_id;
    sp.expert_id = expert_id;
    sp.P = P;
    sp.n_adapters = pool->d.n_adapters;
    sp.n_experts = pool->d.n_experts;
    sp.tile_rows = pick_tile_rows(pool, P);
    sp.key_bits = key_bits_of(pool);
    sp.passes = (sp.key_bits + 7) / 8;
    sp.perm = seg->perm;
    sp.seg_start = seg->seg_start;
    sp.seg_key = seg->seg_key;
    sp.tiles = seg->tiles;
    sp.counts = seg->counts;
    sp.status = seg->status;
    seg->P = P;
    seg->tile_rows = pick_tile_rows(pool, P);
    seg->n_keys = pool->d.n_adapters * pool->d.n_experts;
    seg->reserved = 0;
    return LORA_OK;
}

int lora_build_segments(const lora_pool *pool, const int32_t *adapter_id, const int32_t *expert_id,
                        int P, lora_segments *seg, void *ws, size_t ws_bytes, void *stream)
{
    SegParams sp;
    int rc = prepare_segments(pool, adapter_id, expert_id, P, seg, ws, ws_bytes, sp);
    if (rc != LORA_OK) return rc;
    LORA_HIP(launch_segments(sp, ws, static_cast<hipStream_t>(stream)));
    return LORA_OK;
}

size_t lora_v_bytes(const lora_pool *pool, int proj, int P)
{
    if (check_pool(pool) != LORA_OK || proj < 0 || proj >= pool->d.n_proj || P < 0) return 0;
    const KSplit ks = ksplit_of(pool, proj, P);
    size_t n = parts_bytes(pool, ks.n_parts, P);
    // long-segment batches: the expand keeps its operand images behind the K parts
    if (pick_tile_rows(pool, P) == kTileRows)
        n += align_up(expand_image_bytes(pool->d.rank, tiles_upper_bound(pool, P, kTileRows)), 256);
    return n;
}

int lora_shrink(const lora_pool *pool, int layer, int proj, const void *x, int64_t ldx,
                const int32_t *src_row, const lora_segments *seg, float *v, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    if (layer < 0 || layer >= pool->d.n_layers || proj < 0 || proj >= pool->d.n_proj)
        return LORA_ERR_BAD_SHAPE;
    if (seg->P == 0) return LORA_OK;
    rc = check_act(x, ldx, pool->d.proj[proj].h_in, 2);
    if (rc != LORA_OK) return rc;
    if (!v) return LORA_ERR_INVALID_ARG;
    if (!aligned(v, 16)) return LORA_ERR_MISALIGNED;
    return do_shrink(pool, layer, single(proj, v, nullptr, 0), x, ldx, src_row, seg,
                     static_cast<hipStream_t>(stream));
}

int lora_expand(const lora_pool *pool, int layer, int proj, float *v,
                const lora_segments *seg, void *y, int64_t ldy, int out_dtype, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    if (layer < 0 || layer >= pool->d.n_layers || proj < 0 || proj >= pool->d.n_proj)
        return LORA_ERR_BAD_SHAPE;
    if (out_dtype != LORA_DTYPE_BF16 && out_dtype != LORA_DTYPE_F32) return LORA_ERR_INVALID_ARG;
    if (seg->P == 0) return LORA_OK;
    rc = check_act(y, ldy, pool->d.proj[proj].h_out, out_dtype == LORA_DTYPE_F32 ? 4 : 2);
    if (rc != LORA_OK) return rc;
    if (!v) return LORA_ERR_INVALID_ARG;
    if (!aligned(v, 16)) return LORA_ERR_MISALIGNED;
    return do_expand(pool, layer, single(proj, v, y, ldy), seg, out_dtype,
                     static_cast<hipStream_t>(stream));
}

int lora_apply(const lora_pool *pool, int layer, int proj, const void *x, int64_t ldx,
               const int32_t *src_row, const lora_segments *seg, void *y, int64_t ldy, int out_dtype,
               float *v, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    if (layer < 0 || layer >= pool->d.n_layers || proj < 0 || proj >= pool->d.n_proj)
        return LORA_ERR_BAD_SHAPE;
    if (out_dtype != LORA_DTYPE_BF16 && out_dtype != LORA_DTYPE_F32) return LORA_ERR_INVALID_ARG;
    if (seg->P == 0) return LORA_OK;
    rc = check_act(x, ldx, pool->d.proj[proj].h_in, 2);
    if (rc != LORA_OK) return rc;
    rc = check_act(y, ldy, pool->d.proj[proj].h_out, out_dtype == LORA_DTYPE_F32 ? 4 : 2);
    if (rc != LORA_OK) return rc;
    if (!v) return LORA_ERR_INVALID_ARG;
    if (!aligned(v, 16)) return LORA_ERR_MISALIGNED;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return do_apply(pool, layer, single(proj, v, y, ldy), x, ldx, src_row, seg, out_dtype, st);
}

size_t lora_group_ws_bytes(const lora_pool *pool, int proj0, int n_proj, int P)
{
    if (check_pool(pool) != LORA_OK || proj0 < 0 || n_proj < 1 || proj0 + n_proj > pool->d.n_proj || P < 0)
        return 0;
    return (size_t)n_proj * lora_v_bytes(pool, proj0, P);
}

// lora_apply_group; `build`: the segments are still to be built (lora_build_apply_group).  A
// call that returns an error has enqueued nothing.
static int apply_group_impl(const lora_pool *pool, int layer, int proj0, int n_proj, const void *x,
                            int64_t ldx, const int32_t *src_row, const lora_segments *seg, void *const *y,
                            const int64_t *ldy, int out_dtype, void *ws, size_t ws_bytes, void *stream,
                            const SegParams *build, void *build_ws)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    const lora_pool_desc &d = pool->d;
    if (n_proj < 1 || n_proj > kMaxFused) return LORA_ERR_INVALID_ARG;
    if (layer < 0 || layer >= d.n_layers || proj0 < 0 || proj0 + n_proj > d.n_proj)
        return LORA_ERR_BAD_SHAPE;
    for (int j = 1; j < n_proj; ++j)
        if (d.proj[proj0 + j].h_in != d.proj[proj0].h_in) return LORA_ERR_BAD_SHAPE;
    if (out_dtype != LORA_DTYPE_BF16 && out_dtype != LORA_DTYPE_F32) return LORA_ERR_INVALID_ARG;
    if (!y || !ldy) return LORA_ERR_INVALID_ARG;
    if (seg->P == 0) {
        if (build) LORA_HIP(launch_segments(*build, build_ws, static_cast<hipStream_t>(stream)));
        return LORA_OK;
    }
    rc = check_act(x, ldx, d.proj[proj0].h_in, 2);
    if (rc != LORA_OK) return rc;
    if (!ws) return LORA_ERR_INVALID_ARG;
    if (!aligned(ws, 16)) return LORA_ERR_MISALIGNED;
    if (ws_bytes < lora_group_ws_bytes(pool, proj0, n_proj, seg->P)) return LORA_ERR_BUFFER_TOO_SMALL;
    Group g;
    memset(&g, 0, sizeof g);
    g.proj0 = proj0;
    g.n = n_proj;
    const size_t vb = lora_v_bytes(pool, proj0, seg->P);
    for (int j = 0; j < n_proj; ++j) {
        rc = check_act(y[j], ldy[j], d.proj[proj0 + j].h_out, out_dtype == LORA_DTYPE_F32 ? 4 : 2);
        if (rc != LORA_OK) return rc;
        g.v[j] = reinterpret_cast<float *>(static_cast<char *>(ws) + j * vb);
        g.y[j] = y[j];
        g.ldy[j] = ldy[j];
    }
    return do_apply(pool, layer, g, x, ldx, src_row, seg, out_dtype, static_cast<hipStream_t>(stream), build,
                    build_ws);
}

int lora_apply_group(const lora_pool *pool, int layer, int proj0, int n_proj, const void *x,
                     int64_t ldx, const int32_t *src_row, const lora_segments *seg, void *const *y,
                     const int64_t *ldy, int out_dtype, void *ws, size_t ws_bytes, void *stream)
{
    return apply_group_impl(pool, layer, proj0, n_proj, x, ldx, src_row, seg, y, ldy, out_dtype, ws, ws_bytes,
                            stream, nullptr, nullptr);
}

int lora_build_apply_group(const lora_pool *pool, int layer, int proj0, int n_proj, const void *x,
                           int64_t ldx, const int32_t *src_row, const int32_t *adapter_id,
                           const int32_t *expert_id, int P, lora_segments *seg, void *seg_ws,
                           size_t seg_ws_bytes, void *const *y, const int64_t *ldy, int out_dtype,
                           void *ws, size_t ws_bytes, void *stream)
{
    SegParams sp;
    int rc = prepare_segments(pool, adapter_id, expert_id, P, seg, seg_ws, seg_ws_bytes, sp);
    if (rc != LORA_OK) return rc;
    return apply_group_impl(pool, layer, proj0, n_proj, x, ldx, src_row, seg, y, ldy, out_dtype, ws, ws_bytes,
                            stream, &sp, seg_ws);
}

int lora_build_apply_launches(const lora_pool *pool, int proj0, int n_proj, int out_dtype, int P)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    if (n_proj < 1 || n_proj > kMaxFused || proj0 < 0 || proj0 + n_proj > pool->d.n_proj || P < 0)
        return LORA_ERR_BAD_SHAPE;
    lora_segments seg;
    memset(&seg, 0, sizeof seg);
    seg.P = P;
    seg.tile_rows = pick_tile_rows(pool, P);
    seg.n_keys = pool->d.n_adapters * pool->d.n_experts;
    Group g;
    memset(&g, 0, sizeof g);
    g.proj0 = proj0;
    g.n = n_proj;
    if (P == 0) return 1;
    const int apply = seg.tile_rows == kDecodeTileRows ? (fused_plan(pool, g, &seg, out_dtype, nullptr, nullptr) ? 1 : 2)
                                                       : (n_proj + 1) / 2 + 2;
    return apply + (inline_build_ok(pool, g, &seg, out_dtype) ? 0 : lora_segments_launches(pool, P));
}

int lora_group_launches(const lora_pool *pool, int proj0, int n_proj, int out_dtype,
                        const lora_segments *seg)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    if (n_proj < 1 || n_proj > kMaxFused || proj0 < 0 || proj0 + n_proj > pool->d.n_proj)
        return LORA_ERR_BAD_SHAPE;
    if (seg->P == 0) return 0;
    Group g;
    memset(&g, 0, sizeof g);
    g.proj0 = proj0;
    g.n = n_proj;
    if (seg->tile_rows == kDecodeTileRows) return fused_plan(pool, g, seg, out_dtype, nullptr, nullptr) ? 1 : 2;
    return (n_proj + 1) / 2 + 2;       // long segments: shrink launches of two projections, images, expand
}

size_t lora_moe_ws_bytes(const lora_pool *pool, int P)
{
    if (check_pool(pool) != LORA_OK || pool->d.n_proj < 3 || P < 0) return 0;
    return std::max(2 * lora_v_bytes(pool, 0, P), lora_v_bytes(pool, 2, P));
}

}  // extern "C"

namespace {

int moe_common_checks(const lora_pool *pool, int layer, int which, const lora_segments *seg,
                      void *ws, size_t ws_bytes)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    if (which != LORA_MOE_UPGATE && which != LORA_MOE_DOWN) return LORA_ERR_INVALID_ARG;
    const lora_pool_desc &d = pool->d;
    if (d.n_proj < 3 || layer < 0 || layer >= d.n_layers) return LORA_ERR_BAD_SHAPE;
    if (d.proj[0].h_in != d.proj[1].h_in || d.proj[0].h_out != d.proj[1].h_out)
        return LORA_ERR_BAD_SHAPE;
    if (seg->P == 0) return LORA_OK;
    if (!ws) return LORA_ERR_INVALID_ARG;
    if (!aligned(ws, 16)) return LORA_ERR_MISALIGNED;
    if (ws_bytes < lora_moe_ws_bytes(pool, seg->P)) return LORA_ERR_BUFFER_TOO_SMALL;
    return LORA_OK;
}

int moe_shrink_checks(const lora_pool *pool, int which, const void *in, int64_t ld_in,
                      const int32_t *token_of_pair)
{
    const lora_pool_desc &d = pool->d;
    int rc = check_act(in, ld_in, d.proj[which == LORA_MOE_UPGATE ? 0 : 2].h_in, 2);
    if (rc != LORA_OK) return rc;
    if (which == LORA_MOE_UPGATE && !token_of_pair) return LORA_ERR_INVALID_ARG;
    return LORA_OK;
}

int moe_expand_checks(const lora_pool *pool, int which, void *y0, void *y1, int64_t ldy)
{
    const lora_pool_desc &d = pool->d;
    int rc = check_act(y0, ldy, d.proj[which == LORA_MOE_UPGATE ? 0 : 2].h_out, 2);
    if (rc != LORA_OK) return rc;
    if (which == LORA_MOE_UPGATE) return check_act(y1, ldy, d.proj[1].h_out, 2);
    return LORA_OK;
}

// UPGATE: projections 0 (gate) and 1 (up) sharing the token rows; DOWN: projection 2
Group moe_group(const lora_pool *pool, int which, const lora_segments *seg, void *ws, void *y0,
                void *y1, int64_t ldy)
{
    Group g;
    memset(&g, 0, sizeof g);
    g.v[0] = static_cast<float *>(ws);
    g.y[0] = y0;
    g.ldy[0] = ldy;
    if (which == LORA_MOE_UPGATE) {
        g.proj0 = 0;
        g.n = 2;
        g.v[1] = reinterpret_cast<float *>(static_cast<char *>(ws) + lora_v_bytes(pool, 0, seg->P));
        g.y[1] = y1;
        g.ldy[1] = ldy;
    } else {
        g.proj0 = 2;
        g.n = 1;
    }
    return g;
}

int moe_shrink_launch(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                      const int32_t *token_of_pair, const lora_segments *seg, void *ws,
                      hipStream_t st)
{
    return do_shrink(pool, layer, moe_group(pool, which, seg, ws, nullptr, nullptr, 0), in, ld_in,
                     which == LORA_MOE_UPGATE ? token_of_pair : nullptr, seg, st);
}

int moe_expand_launch(const lora_pool *pool, int layer, int which, const lora_segments *seg,
                      void *y0, void *y1, int64_t ldy, void *ws, hipStream_t st)
{
    return do_expand(pool, layer, moe_group(pool, which, seg, ws, y0, y1, ldy), seg, LORA_DTYPE_BF16, st);
}

}  // namespace

extern "C" {

int lora_moe_shrink(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                    const int32_t *token_of_pair, const lora_segments *seg, void *ws,
                    size_t ws_bytes, void *stream)
{
    int rc = moe_common_checks(pool, layer, which, seg, ws, ws_bytes);
    if (rc != LORA_OK || seg->P == 0) return rc;
    rc = moe_shrink_checks(pool, which, in, ld_in, token_of_pair);
    if (rc != LORA_OK) return rc;
    return moe_shrink_launch(pool, layer, which, in, ld_in, token_of_pair, seg, ws,
                             static_cast<hipStream_t>(stream));
}

int lora_moe_expand(const lora_pool *pool, int layer, int which, const lora_segments *seg,
                    void *y0, void *y1, int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    int rc = moe_common_checks(pool, layer, which, seg, ws, ws_bytes);
    if (rc != LORA_OK || seg->P == 0) return rc;
    rc = moe_expand_checks(pool, which, y0, y1, ldy);
    if (rc != LORA_OK) return rc;
    return moe_expand_launch(pool, layer, which, seg, y0, y1, ldy, ws,
                             static_cast<hipStream_t>(stream));
}

int lora_moe_apply_static(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                          const int32_t *token_of_pair, const lora_segments *seg, void *y0, void *y1,
                          int64_t ldy, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    if (!seg) return LORA_ERR_INVALID_ARG;
    if (seg->P > 0 && pool->d.n_proj >= 3 && lora_moe_ws_bytes(pool, seg->P) > kStaticScratchBytes)
        return LORA_ERR_TOO_LARGE;
    void *ws = nullptr;
    rc = static_scratch(&ws);            // the device address, never the array's name
    if (rc != LORA_OK) return rc;
    return lora_moe_apply(pool, layer, which, in, ld_in, token_of_pair, seg, y0, y1, ldy, ws,
                          kStaticScratchBytes, stream);
}

static int moe_apply_impl(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                          const int32_t *token_of_pair, const lora_segments *seg, void *y0, void *y1,
                          int64_t ldy, void *ws, size_t ws_bytes, void *stream, const SegParams *build,
                          void *build_ws)
{
    int rc = moe_common_checks(pool, layer, which, seg, ws, ws_bytes);
    if (rc != LORA_OK) return rc;
    if (seg->P == 0) {
        if (build) LORA_HIP(launch_segments(*build, build_ws, static_cast<hipStream_t>(stream)));
        return LORA_OK;
    }
    rc = moe_shrink_checks(pool, which, in, ld_in, token_of_pair);
    if (rc != LORA_OK) return rc;
    rc = moe_expand_checks(pool, which, y0, y1, ldy);
    if (rc != LORA_OK) return rc;
    return do_apply(pool, layer, moe_group(pool, which, seg, ws, y0, y1, ldy), in, ld_in,
                    which == LORA_MOE_UPGATE ? token_of_pair : nullptr, seg, LORA_DTYPE_BF16,
                    static_cast<hipStream_t>(stream), build, build_ws);
}

int lora_moe_apply(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                   const int32_t *token_of_pair, const lora_segments *seg, void *y0, void *y1,
                   int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    return moe_apply_impl(pool, layer, which, in, ld_in, token_of_pair, seg, y0, y1, ldy, ws, ws_bytes, stream,
                          nullptr, nullptr);
}

int lora_moe_build_apply(const lora_pool *pool, int layer, int which, const void *in, int64_t ld_in,
                         const int32_t *token_of_pair, const int32_t *adapter_id,
                         const int32_t *expert_id, int P, lora_segments *seg, void *seg_ws,
                         size_t seg_ws_bytes, void *y0, void *y1, int64_t ldy, void *ws, size_t ws_bytes,
                         void *stream)
{
    SegParams sp;
    int rc = prepare_segments(pool, adapter_id, expert_id, P, seg, seg_ws, seg_ws_bytes, sp);
    if (rc != LORA_OK) return rc;
    return moe_apply_impl(pool, layer, which, in, ld_in, token_of_pair, seg, y0, y1, ldy, ws, ws_bytes, stream,
                          &sp, seg_ws);
}

size_t lora_moe_combine_ws_bytes(const lora_pool *pool, int P)
{
    if (check_pool(pool) != LORA_OK || pool->d.n_proj < 3 || P < 0) return 0;
    const size_t pair_rows = align_up((size_t)std::max(P, 1) * pool->d.proj[2].h_out * sizeof(uint16_t), 256);
    return align_up(lora_moe_ws_bytes(pool, P), 256) + pair_rows;
}

int lora_moe_down_combine(const lora_pool *pool, int layer, const void *hmid, int64_t ld_in,
                          const int32_t *adapter_id, const int32_t *expert_id,
                          const lora_segments *seg, const float *route_w, int top_k, void *y_tok,
                          int64_t ldy, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_pool(pool);
    if (rc != LORA_OK) return rc;
    rc = check_segments(pool, seg);
    if (rc != LORA_OK) return rc;
    const lora_pool_desc &d = pool->d;
    if (d.n_proj < 3 || layer < 0 || layer >= d.n_layers) return LORA_ERR_BAD_SHAPE;
    if (top_k < 1 || top_k > combine_max_top_k()) return LORA_ERR_INVALID_ARG;
    if (seg->P % top_k != 0) return LORA_ERR_BAD_SHAPE;
    if (seg->P == 0) return LORA_OK;
    rc = check_act(hmid, ld_in, d.proj[2].h_in, 2);
    if (rc != LORA_OK) return rc;
    rc = check_act(y_tok, ldy, d.proj[2].h_out, 2);
    if (rc != LORA_OK) return rc;
    if (!adapter_id || !route_w || !ws) return LORA_ERR_INVALID_ARG;
    if (d.n_experts > 1 && !expert_id) return LORA_ERR_INVALID_ARG;
    if (!aligned(ws, 16)) return LORA_ERR_MISALIGNED;
    if (ws_bytes < lora_moe_combine_ws_bytes(pool, seg->P)) return LORA_ERR_BUFFER_TOO_SMALL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int h_out = d.proj[2].h_out;
    uint16_t *pair = reinterpret_cast<uint16_t *>(static_cast<char *>(ws) +
                                                  align_up(lora_moe_ws_bytes(pool, seg->P), 256));
    // 1. shrink of the down projection, as in lora_moe_apply
    rc = moe_shrink_launch(pool, layer, LORA_MOE_DOWN, hmid, ld_in, nullptr, seg, ws, st);
    if (rc != LORA_OK) return rc;
    // 2. the per-pair updates into rows of their own.  Decode batches write them without reading
    // anything; the long-segment expand only knows how to add, so its rows are cleared first.
    Group g = moe_group(pool, LORA_MOE_DOWN, seg, ws, pair, nullptr, h_out);
    if (seg->tile_rows == kDecodeTileRows)
        g.overwrite = 1;
    else
        LORA_HIP(launch_fill_zero(pair, align_up((size_t)seg->P * h_out * sizeof(uint16_t), 16), st));
    rc = do_expand(pool, layer, g, seg, LORA_DTYPE_BF16, st);
    if (rc != LORA_OK) return rc;
    // 3. token rows: y[t] += sum over the token's pairs, ascending, of w * update
    CombineParams cp;
    memset(&cp, 0, sizeof cp);
    cp.pair = pair;
    cp.ld_pair = h_out;
    cp.adapter_id = adapter_id;
    cp.expert_id = d.n_experts > 1 ? expert_id : nullptr;
    cp.route_w = route_w;
    cp.T = seg->P / top_k;
    cp.top_k = top_k;
    cp.n_adapters = d.n_adapters;
    cp.n_experts = d.n_experts;
    cp.h_out = h_out;
    cp.y = static_cast<uint16_t *>(y_tok);
    cp.ldy = ldy;
    LORA_HIP(launch_combine(cp, st));
    return LORA_OK;
}

}  // extern "C"
