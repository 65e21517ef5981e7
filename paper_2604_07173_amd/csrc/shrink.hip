// Shrink for batches with long segments (tiles of up to 32 rows): v = gather(x) * A
// (App. A.2.2 "shrink phase"; Sec. 2.2 x A).
//
// With long segments the traffic is the read of x; A is small, but a wave that multiplies it
// with only 32 rows re-reads it from the L2 four times as fast as x arrives from HBM.  So the
// four waves of a workgroup take four consecutive tiles (up to 128 rows) and share A through
// LDS: work item = (group of four tiles, K part).  Per stage of four K blocks the workgroup
// copies the packed A blocks of the first tile's (adapter, expert) into one of two LDS
// buffers while the previous stage is being multiplied; every wave gathers the x rows of its
// own tile (the next stage's rows are in flight during the current stage's MFMAs) and reads
// its MFMA operands from LDS with 16-byte reads that are contiguous per wave.  The x rows are
// fetched as whole cache lines, four rows x 256 bytes per instruction, and turned into the MFMA
// operand layout (16 rows x 64 bytes per operand) through 4 KiB of LDS per wave: fetching them
// in the operand layout directly costs the address path twice the line look-ups, which a
// load-only probe of the two streams puts at 32 against 27 us for the prefill workload.  A group whose
// tiles do not all belong to one (adapter, expert) (a segment boundary inside the group) takes
// a plain path in which every wave reads its own A from global memory.  Every wave owns its rows for the
// whole K part, so there is no cross-wave reduction; lora_expand adds the K parts in a fixed
// order, so results are bit-identical run to run.
//
// The rank index sits on the M side of v_mfma_f32_16x16x32_bf16 and the rows on the N side, so
// a lane ends up with four consecutive rank entries of one row.  With two fused projections
// (gate and up, or two projections of a group that read the same input) x is loaded once.
// Ranks 16, 32 and 64; rank-8 pools always use the 16-row-tile kernels.
#include "lora_device.h"
#include "lora_internal.h"

namespace lora {

namespace {

constexpr int kLongTiles = 4;        // tiles (waves) per work item
constexpr int kStageKB = 4;          // K blocks per LDS stage

template <int R, int NPROJ>
__global__ __launch_bounds__(256, 2) void shrink_long_kernel(ShrinkParams p,
                                                             const lora_tile *__restrict__ tiles,
                                                             const Unit *__restrict__ units,
                                                             const int32_t *__restrict__ counts)
{
    constexpr int NB = R / 16;                         // 16-wide blocks of the rank index
    constexpr int BLK = NPROJ * NB;                    // 1 KiB operand blocks per K block
    constexpr int STAGE = kStageKB * BLK * 64;         // 16-byte vectors per stage
    constexpr int LOADS = STAGE / 256;                 // per thread and stage
    constexpr int SUB = kTileRows / 16;
    static_assert(STAGE % 256 == 0, "a stage is copied by whole workgroup passes");
    static_assert(kStageKB == 4, "a stage of x is 256 bytes per row: the transposition below is written for that");
    // dynamic LDS: two stages of A, then per wave 4 KiB in which a sub-tile's stage of x is
    // turned from the layout it is fetched in (whole lines per row) into the MFMA operand layout
    extern __shared__ __attribute__((aligned(16))) unsigned char dyn_lds[];
    u32x4 (*lds)[STAGE] = reinterpret_cast<u32x4 (*)[STAGE]>(dyn_lds);
    u32x4 *xt = reinterpret_cast<u32x4 *>(dyn_lds + 2 * STAGE * sizeof(u32x4)) + (threadIdx.x >> 6) * 256;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, i16 = lane & 15;
    const int n_tiles = counts[2];
    const int n_groups = (n_tiles + kLongTiles - 1) / kLongTiles;
    const int n_items = n_groups * p.n_parts;
    const int kblocks = (p.h_in + kKBlock - 1) / kKBlock;
    const u32x4 zero4 = {0u, 0u, 0u, 0u};

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int grp = item / p.n_parts;
        const int part = item - grp * p.n_parts;
        const int key0 = tiles[grp * kLongTiles].key;
        const int tix = __builtin_amdgcn_readfirstlane(grp * kLongTiles + wave);
        const bool live = tix < n_tiles;                      // wave-uniform
        const lora_tile t = tiles[min(tix, n_tiles - 1)];
        // does every tile of the group belong to the first tile's (adapter, expert)?  Uniform
        // over the workgroup: every wave looks at all four records.
        bool same_key = true;
#pragma unroll
        for (int k = 1; k < kLongTiles; ++k)
            same_key = same_key && tiles[min(grp * kLongTiles + k, n_tiles - 1)].key == key0;

        const uint16_t *Ag[NPROJ], *Aw[NPROJ];                // the group's A, this wave's A
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj) {
            Ag[pj] = units[(int64_t)key0 * p.n_proj + p.proj0 + pj].A;
            Aw[pj] = units[(int64_t)t.key * p.n_proj + p.proj0 + pj].A;
        }

        // gathered input rows: lane (i16, g) reads x[row i16 of the sub-tile][8*g ...]; rows
        // beyond the tile re-read its first row and are replaced by zeros
        const uint16_t *xp[SUB];
        bool rv[SUB];
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub) {
            const int r = sub * 16 + i16;
            rv[sub] = live && r < t.n_rows;
            int s = p.perm[t.row0 + min(r, t.n_rows - 1)];
            if (p.src_row) s = p.src_row[s];
            xp[sub] = p.x + (int64_t)s * p.ldx + g * 8;
        }

        // the same rows as they are fetched on the shared-A path: one instruction reads four
        // rows (lane group g) x 256 contiguous bytes (16 lanes x 16 bytes), i.e. whole cache
        // lines, which the address path serves faster than 16 rows x 64 bytes
        const uint16_t *xq[SUB][4];
        bool qv[SUB][4];
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = sub * 16 + j * 4 + g;
                qv[sub][j] = live && r < t.n_rows;
                int s = p.perm[t.row0 + min(r, t.n_rows - 1)];
                if (p.src_row) s = p.src_row[s];
                xq[sub][j] = p.x + (int64_t)s * p.ldx;            // start of the row
            }

        const int kb_begin = part * p.kb_per_part;
        const int kb_end = min(kb_begin + p.kb_per_part, kblocks);
        const int n_stages = (kb_end - kb_begin + kStageKB - 1) / kStageKB;

        f32x4 acc[NPROJ][SUB][NB];
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) acc[pj][sub][nb] = f32x4{0.f, 0.f, 0.f, 0.f};

        // All loads are unconditional: a K block beyond the part re-reads the part's last
        // block and is replaced by zeros (x as well: the padding may hold anything).
        auto load_a = [&](int kb0, u32x4 (&a)[LOADS]) {
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                const int b = 4 * i + wave;                   // operand block of the stage
                const int kbi = b / BLK, rem = b - kbi * BLK;
                const int pj = rem / NB, nb = rem - pj * NB;
                const bool k_ok = kb0 + kbi < kb_end;
                const int kb = k_ok ? kb0 + kbi : kb_end - 1;
                const uint16_t *Ap = NPROJ == 2 && pj == 1 ? Ag[NPROJ - 1] : Ag[0];
                const u32x4 v = ld16<false>(Ap + (((int64_t)kb * NB + nb) * 64 + lane) * 8);
                a[i] = k_ok ? v : zero4;
            }
        };
        auto store_a = [&](const u32x4 (&a)[LOADS], u32x4 *buf) {
#pragma unroll
            for (int i = 0; i < LOADS; ++i) buf[(4 * i + wave) * 64 + lane] = a[i];
        };
        // a stage of x as whole lines: lane (g, i16) of instruction j holds K values
        // kb0 * 32 + 8 * i16 .. + 7 of row 4 j + g of the sub-tile
        auto load_rows = [&](int kb0, u32x4 (&xr)[SUB][4]) {
            const int kb = kb0 + (i16 >> 2);                  // the K block this lane's 16 bytes belong to
            const bool k_ok = kb < kb_end;
            const bool c_ok = k_ok && kb0 * kKBlock + i16 * 8 < p.h_in;
            const int c = c_ok ? kb0 * kKBlock + i16 * 8 : 0;    // beyond the part: the row's first bytes, not used
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const u32x4 v = ld16<true>(xq[sub][j] + c);  // read once: nontemporal
                    xr[sub][j] = (c_ok && qv[sub][j]) ? v : zero4;
                }
        };
        // rows -> MFMA operands through this wave's 4 KiB of LDS.  The 16-byte column of a row
        // is stored at column (col ^ row): the writes of an instruction (one row per 16 lanes)
        // and the reads (16 rows, one column each per 16 lanes) both touch every bank once.
        // LDS operations of one wave execute in order, so no barrier is needed.
        auto to_operands = [&](const u32x4 (&xr)[SUB][4], u32x4 (&xv)[SUB][kStageKB]) {
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int row = j * 4 + g;
                    xt[row * 16 + (i16 ^ row)] = xr[sub][j];
                }
#pragma unroll
                for (int kbi = 0; kbi < kStageKB; ++kbi) xv[sub][kbi] = xt[i16 * 16 + ((kbi * 4 + g) ^ i16)];
            }
        };
        // one stage out of LDS: straight-line code, no global loads inside
        auto compute = [&](const u32x4 *buf, const u32x4 (&xv)[SUB][kStageKB]) {
#pragma unroll
            for (int kbi = 0; kbi < kStageKB; ++kbi)
#pragma unroll
                for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const u32x4 w = buf[((kbi * NPROJ + pj) * NB + nb) * 64 + lane];
#pragma unroll
                        for (int sub = 0; sub < SUB; ++sub)
                            acc[pj][sub][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                as_bf16x8(w), as_bf16x8(xv[sub][kbi]), acc[pj][sub][nb], 0, 0, 0);
                    }
        };

        if (same_key) {
            u32x4 areg[LOADS];
            u32x4 xr[SUB][4];                  // the next stage's x as fetched
            u32x4 xc[SUB][kStageKB];           // the current stage's x as MFMA operands
            load_a(kb_begin, areg);
            load_rows(kb_begin, xr);
            store_a(areg, lds[0]);
            to_operands(xr, xc);
            __syncthreads();
            for (int s = 0; s < n_stages; ++s) {
                const int kb0 = kb_begin + s * kStageKB;
                load_a(kb0 + kStageKB, areg);                 // beyond the part: zeros, never multiplied
                load_rows(kb0 + kStageKB, xr);
                __builtin_amdgcn_sched_barrier(0);            // all of the next stage's loads first
                compute(lds[s & 1], xc);
                store_a(areg, lds[(s + 1) & 1]);
                to_operands(xr, xc);
                __syncthreads();
            }
        } else {
            // a segment boundary inside the group: every wave reads the A of its own tile from
            // global memory, one K block at a time (rare, so kept simple)
            for (int kb = kb_begin; kb < kb_end; ++kb) {
                const bool c_ok = kb * kKBlock + g * 8 < p.h_in;
                u32x4 xv[SUB];
#pragma unroll
                for (int sub = 0; sub < SUB; ++sub) {
                    const u32x4 v = ld16<false>(xp[sub] + (c_ok ? kb * kKBlock : 0));
                    xv[sub] = (c_ok && rv[sub]) ? v : zero4;
                }
#pragma unroll
                for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) {
                        const u32x4 w = ld16<false>(Aw[pj] + (((int64_t)kb * NB + nb) * 64 + lane) * 8);
#pragma unroll
                        for (int sub = 0; sub < SUB; ++sub)
                            acc[pj][sub][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                as_bf16x8(w), as_bf16x8(xv[sub]), acc[pj][sub][nb], 0, 0, 0);
                    }
            }
        }

        // this wave's rows of this part of v: lane (row i16, group g) holds rank entries
        // nb*16 + 4g .. +3 of its row
#pragma unroll
        for (int pj = 0; pj < NPROJ; ++pj)
#pragma unroll
            for (int sub = 0; sub < SUB; ++sub)
                if (rv[sub]) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        st16f(p.v[pj] + ((int64_t)part * p.P + t.row0 + sub * 16 + i16) * R + nb * 16 + g * 4,
                              acc[pj][sub][nb]);
                }
    }
}

template <int R, int NPROJ>
hipError_t launch_rn(const ShrinkParams &p, hipStream_t s)
{
    // two stages of A (kStageKB K blocks of NPROJ * R / 16 operand blocks of 1 KiB) + 4 KiB per wave
    constexpr int kLds = 2 * kStageKB * NPROJ * (R / 16) * 1024 + 4 * 4096;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(shrink_long_kernel<R, NPROJ>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((shrink_long_kernel<R, NPROJ>), dim3(p.grid), dim3(256), kLds, s, p, p.tiles, p.units,
                       p.counts);
    return hipGetLastError();
}

template <int R>
hipError_t launch_r(const ShrinkParams &p, hipStream_t s)
{
    return p.n_fused == 2 ? launch_rn<R, 2>(p, s) : launch_rn<R, 1>(p, s);
}

}  // namespace

int shrink_long_tiles() { return kLongTiles; }

hipError_t launch_shrink(const ShrinkParams &p, hipStream_t s)
{
    if (p.grid <= 0) return hipSuccess;
    switch (p.rank) {
    case 16: return launch_r<16>(p, s);
    case 32: return launch_r<32>(p, s);
    case 64: return launch_r<64>(p, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lora
