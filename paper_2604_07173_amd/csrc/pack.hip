// Repacking of row-major A[h_in][r] / B[r][h_out] into the pool's tiled storage and back.
// One thread moves one 16-byte group (eight values that differ only in their K offset t).
#include <algorithm>

#include "lora_internal.h"
#include "lora_layout.h"

namespace lora {

// direction: 0 = row-major -> packed, 1 = packed -> row-major (padding is dropped)
template <int DIR>
__device__ inline void pack_A_body(const PackParams &p, int64_t gid, int unit)
{
    const int kunit = packA_kunit(p.rank);
    const int k_pad = (p.h + kunit - 1) / kunit * kunit;
    const int64_t groups = (int64_t)(k_pad / 8) * p.rank;       // (c / 8, j)
    if (gid >= groups) return;
    const int j = (int)(gid % p.rank);
    const int c0 = (int)(gid / p.rank) * 8;
    uint16_t *packed = (DIR == 0 ? p.dst : const_cast<uint16_t *>(p.src)) +
                       (int64_t)unit * (DIR == 0 ? p.dst_stride : p.src_stride) +
                       packA_index(c0, j, p.rank);               // t = 0..7 are contiguous
    uint16_t *plain = (DIR == 0 ? const_cast<uint16_t *>(p.src) : p.dst) +
                      (int64_t)unit * (DIR == 0 ? p.src_stride : p.dst_stride);
    for (int t = 0; t < 8; ++t) {
        const int c = c0 + t;
        const bool in = c < p.h && j < p.src_rank;
        if (DIR == 0) packed[t] = in ? plain[(int64_t)c * p.src_rank + j] : (uint16_t)0;
        else if (in) plain[(int64_t)c * p.src_rank + j] = packed[t];
    }
}

template <int DIR>
__global__ __launch_bounds__(256) void pack_A_kernel(PackParams p)
{
    pack_A_body<DIR>(p, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, blockIdx.y);
}

template <int DIR>
__device__ inline void pack_B_body(const PackParams &p, int64_t gid, int unit)
{
    const int chunks = (p.h + 127) / 128;
    const int jg = p.rank / 8;                                 // groups of 8 rank indices
    const int64_t groups = (int64_t)chunks * 128 * jg;         // (d, j/8)
    if (gid >= groups) return;
    const int d = (int)(gid % ((int64_t)chunks * 128));
    const int j0 = (int)(gid / ((int64_t)chunks * 128)) * 8;
    uint16_t *packed = (DIR == 0 ? p.dst : const_cast<uint16_t *>(p.src)) +
                       (int64_t)unit * (DIR == 0 ? p.dst_stride : p.src_stride);
    uint16_t *plain = (DIR == 0 ? const_cast<uint16_t *>(p.src) : p.dst) +
                      (int64_t)unit * (DIR == 0 ? p.src_stride : p.dst_stride);
    for (int t = 0; t < 8; ++t) {
        const int j = j0 + t;
        const bool in = d < p.h && j < p.src_rank;
        uint16_t *q = packed + packB_index(j, d, p.rank);
        if (DIR == 0) *q = in ? plain[(int64_t)j * p.h + d] : (uint16_t)0;
        else if (in) plain[(int64_t)j * p.h + d] = *q;
    }
}

template <int DIR>
__global__ __launch_bounds__(256) void pack_B_kernel(PackParams p)
{
    pack_B_body<DIR>(p, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, blockIdx.y);
}

// every repack of one (adapter, layer): blockIdx.z picks the job (even: an A, odd: a B)
__global__ __launch_bounds__(256) void pack_layer_kernel(PackLayerParams ps)
{
    const int job = blockIdx.z;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (job & 1) pack_B_body<0>(ps.job[job], gid, blockIdx.y);
    else pack_A_body<0>(ps.job[job], gid, blockIdx.y);
}

// scale and rank of one adapter's table entries, all layers: entry (layer, adapter, e, j) sits
// at ((layer * n_adapters + adapter) * per_adapter + (e * n_proj + j))
__global__ __launch_bounds__(256) void set_adapter_kernel(Unit *table, int n_layers, int n_adapters,
                                                          int per_adapter, int adapter, int rank,
                                                          float scale)
{
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)n_layers * per_adapter) return;
    const int layer = (int)(gid / per_adapter), k = (int)(gid % per_adapter);
    Unit *u = table + ((int64_t)layer * n_adapters + adapter) * per_adapter + k;
    u->scale = scale;
    u->rank = rank;
}

hipError_t launch_set_adapter(Unit *table, int n_layers, int n_adapters, int per_adapter, int adapter,
                              int rank, float scale, hipStream_t s)
{
    const int64_t n = (int64_t)n_layers * per_adapter;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(set_adapter_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, table,
                       n_layers, n_adapters, per_adapter, adapter, rank, scale);
    return hipGetLastError();
}

template <typename K>
static hipError_t launch_pack(K kernel, const PackParams &p, int64_t groups, hipStream_t s)
{
    if (p.n_units <= 0 || groups <= 0) return hipSuccess;
    dim3 grid((unsigned)((groups + 255) / 256), (unsigned)p.n_units);
    hipLaunchKernelGGL(kernel, grid, dim3(256), 0, s, p);
    return hipGetLastError();
}

static int64_t groups_A(const PackParams &p)
{
    return (int64_t)kblocks_of(p.h, p.rank) * (kunit_of(p.rank) / 8) * p.rank;
}
static int64_t groups_B(const PackParams &p) { return (int64_t)chunks_of(p.h) * 128 * (p.rank / 8); }

hipError_t launch_pack_layer(const PackLayerParams &ps, hipStream_t s)
{
    int64_t groups = 0;
    for (int j = 0; j < ps.n_jobs; ++j)
        groups = std::max(groups, (j & 1) ? groups_B(ps.job[j]) : groups_A(ps.job[j]));
    if (ps.n_jobs <= 0 || groups <= 0 || ps.job[0].n_units <= 0) return hipSuccess;
    dim3 grid((unsigned)((groups + 255) / 256), (unsigned)ps.job[0].n_units, (unsigned)ps.n_jobs);
    hipLaunchKernelGGL(pack_layer_kernel, grid, dim3(256), 0, s, ps);
    return hipGetLastError();
}

hipError_t launch_pack_A(const PackParams &p, hipStream_t s)
{
    return launch_pack(pack_A_kernel<0>, p, (int64_t)kblocks_of(p.h, p.rank) * (kunit_of(p.rank) / 8) * p.rank, s);
}
hipError_t launch_unpack_A(const PackParams &p, hipStream_t s)
{
    return launch_pack(pack_A_kernel<1>, p, (int64_t)kblocks_of(p.h, p.rank) * (kunit_of(p.rank) / 8) * p.rank, s);
}
hipError_t launch_pack_B(const PackParams &p, hipStream_t s)
{
    return launch_pack(pack_B_kernel<0>, p, (int64_t)chunks_of(p.h) * 128 * (p.rank / 8), s);
}
hipError_t launch_unpack_B(const PackParams &p, hipStream_t s)
{
    return launch_pack(pack_B_kernel<1>, p, (int64_t)chunks_of(p.h) * 128 * (p.rank / 8), s);
}

}  // namespace lora
