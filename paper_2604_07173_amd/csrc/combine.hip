// Routing-weighted combine of the per-pair updates of the down projection into token rows
// (Sec. 4.1: a token activates its top-k experts, pair p = t * k + j; Sec. 3 / Fig. 7b: the
// update is added to the base output):
//   y[t] = bf16( f32(y[t]) + sum over j = 0 .. k-1, ascending, of w[t*k+j] * update[t*k+j] )
// over the pairs that have a valid adapter and expert; a token without any such pair is not
// touched.  The sum runs in a fixed order in fp32, so results are bit-identical run to run.
//
// One workgroup per token; a thread owns eight consecutive output columns at a time (16 bytes
// of a bf16 row, so a wave reads and writes 1 KiB contiguous pieces).  The ids and weights of
// the token's pairs are wave-uniform.
#include <algorithm>

#include "lora_device.h"
#include "lora_internal.h"

namespace lora {

namespace {

constexpr int kMaxTopK = 16;

__global__ __launch_bounds__(256) void combine_kernel(CombineParams p)
{
    const int t = blockIdx.x;
    float w[kMaxTopK];
    unsigned active = 0;
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
        w[j] = 0.f;
        if (j < p.top_k) {
            const int64_t pr = (int64_t)t * p.top_k + j;
            const int a = p.adapter_id[pr];
            const int e = p.expert_id ? p.expert_id[pr] : 0;
            if (a >= 0 && a < p.n_adapters && e >= 0 && e < p.n_experts) {
                active |= 1u << j;
                w[j] = p.route_w[pr];
            }
        }
    }
    if (!active) return;
    const uint16_t *rows = p.pair + (int64_t)t * p.top_k * p.ld_pair;
    uint16_t *yrow = p.y + (int64_t)t * p.ldy;
    for (int c = threadIdx.x * 8; c < p.h_out; c += 256 * 8) {
        const u32x4 yv = ld16<false>(yrow + c);
        float acc[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = 0.f;
#pragma unroll
        for (int j = 0; j < kMaxTopK; ++j) {
            if (j < p.top_k && (active >> j & 1u)) {          // wave-uniform
                const u32x4 d = ld16<true>(rows + (int64_t)j * p.ld_pair + c);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    acc[2 * q] += w[j] * __uint_as_float(d[q] << 16);
                    acc[2 * q + 1] += w[j] * __uint_as_float(d[q] & 0xFFFF0000u);
                }
            }
        }
        u32x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            o[q] = pack_bf16_rne(__uint_as_float(yv[q] << 16) + acc[2 * q],
                                 __uint_as_float(yv[q] & 0xFFFF0000u) + acc[2 * q + 1]);
        st16<false>(yrow + c, o);
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4 *dst, size_t n_vec)
{
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += (size_t)gridDim.x * 256)
        st16<false>(dst + i, z);
}

}  // namespace

int combine_max_top_k() { return kMaxTopK; }

hipError_t launch_combine(const CombineParams &p, hipStream_t s)
{
    if (p.T <= 0) return hipSuccess;
    hipLaunchKernelGGL(combine_kernel, dim3(p.T), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_fill_zero(void *dst, size_t bytes, hipStream_t s)
{
    const size_t n_vec = bytes / 16;
    if (n_vec == 0) return hipSuccess;
    const unsigned grid = (unsigned)std::min<size_t>((n_vec + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(grid), dim3(256), 0, s, static_cast<u32x4 *>(dst), n_vec);
    return hipGetLastError();
}

}  // namespace lora
