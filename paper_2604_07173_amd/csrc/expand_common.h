// Pieces shared by the expand kernels: the packed B tile of one 128-column chunk as MFMA
// operand registers, the hi/lo bf16 operand made from fp32 v, and the MFMA sequence.
//
// rank <= 16 uses v_mfma_f32_16x16x16_bf16 (four K values per lane, 8-byte operands):
//   rank 16: K = the 16 rank entries; hi and lo planes of v are two MFMAs on the same B.
//   rank  8: K = hi of the 8 entries (lane groups 0,1) then lo (groups 2,3); B lane groups
//            2,3 re-read the bytes of groups 0,1; one MFMA.
// rank >= 32 uses v_mfma_f32_16x16x32_bf16 (eight K values per lane, 16-byte operands),
//   rank/32 K steps, hi and lo planes as separate MFMAs on the same B.
#pragma once
#include <type_traits>

#include "lora_device.h"

namespace lora {

typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int R>
struct ExpandTile {
    static constexpr bool K16 = R <= 16;
    static constexpr int KS = R >= 32 ? R / 32 : 1;
    static constexpr int KV = K16 ? 4 : 8;            // K values (v entries) per lane and step
    using vec = typename std::conditional<K16, u32x2, u32x4>::type;

    struct B {
        vec r[8][KS];
    };
    struct A {                 // v operand of one 16-row sub-tile
        vec hi[KS], lo[KS];    // rank 8: hi[0] carries the mixed hi/lo operand, lo unused
    };

    // first rank index of the KV values lane group g holds in K step ks
    __device__ static inline int jbase(int g, int ks)
    {
        if (R >= 32) return ks * 32 + g * 8;
        if (R == 16) return g * 4;
        return (g & 1) * 4;
    }

    template <bool NT>
    __device__ static inline void load_b(const uint16_t *Bp, int chunk, int lane, B &b)
    {
        const int g = lane >> 4, i16 = lane & 15;
        if constexpr (R >= 32) {
#pragma unroll
            for (int blk = 0; blk < 8; ++blk)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int64_t off = (((((int64_t)chunk * 8 + blk) * KS + ks) * 4 + g) * 16 + i16) * 8;
                    b.r[blk][ks] = ld16<NT>(Bp + off);
                }
        } else {
            // one 16-byte load per pair of sub-blocks; rank 8: lane groups 2,3 re-read the
            // bytes of groups 0,1
            constexpr int G = R / 4;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t off = ((((int64_t)chunk * 4 + q) * G + (R == 16 ? g : (g & 1))) * 16 + i16) * 8;
                const u32x4 v = ld16<NT>(Bp + off);
                b.r[2 * q][0] = u32x2{v[0], v[1]};
                b.r[2 * q + 1][0] = u32x2{v[2], v[3]};
            }
        }
    }

    // KV fp32 values (already summed and scaled) -> this lane's part of the operand
    __device__ static inline void make_a(const float (&s)[KV], int g, int ks, A &a)
    {
        unsigned hi[KV / 2], lo[KV / 2];
#pragma unroll
        for (int m = 0; m < KV / 2; ++m) {
            const unsigned h0 = __float_as_uint(s[2 * m]) & 0xFFFF0000u;
            const unsigned h1 = __float_as_uint(s[2 * m + 1]) & 0xFFFF0000u;
            hi[m] = (h0 >> 16) | h1;
            lo[m] = pack_bf16_rne(s[2 * m] - __uint_as_float(h0), s[2 * m + 1] - __uint_as_float(h1));
        }
        vec vh, vl;
#pragma unroll
        for (int m = 0; m < KV / 2; ++m) {
            vh[m] = hi[m];
            vl[m] = lo[m];
        }
        if (R == 8) {
            a.hi[ks] = g < 2 ? vh : vl;
            a.lo[ks] = vl;
        } else {
            a.hi[ks] = vh;
            a.lo[ks] = vl;
        }
    }

    __device__ static inline f32x4 mfma(vec a, vec b, f32x4 c)
    {
        if constexpr (K16)
            return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, a),
                                                             __builtin_bit_cast(s16x4, b), c, 0, 0, 0);
        else
            return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
    }

    // the eight 16x16 blocks of the chunk: acc[blk][i] = row slot 4*g + i, column slot i16
    __device__ static inline void mma(const A &a, const B &b, f32x4 (&acc)[8])
    {
#pragma unroll
        for (int blk = 0; blk < 8; ++blk) {
            f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                c = mfma(a.hi[ks], b.r[blk][ks], c);
                if (R != 8) c = mfma(a.lo[ks], b.r[blk][ks], c);
            }
            acc[blk] = c;
        }
    }
};

}  // namespace lora
