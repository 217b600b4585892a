// Sum over a token's selected experts (Sec. 2.2: the last step of the MoE layer), optionally weighted
// by the router: out[t, n] = bf16( sum_j w[t, j] * Y[t, j, n] ), j ascending, fp32.
// Pure streaming: each lane owns 8 consecutive n of one token (16-byte loads and stores).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace moe {

__device__ __forceinline__ float bf16_lo(uint32_t v) { return __uint_as_float(v << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t v) { return __uint_as_float(v & 0xffff0000u); }

// grid.x covers chunks (8 columns) of all tokens: chunk index c -> token c / (N/8), column 8 * (c % (N/8)).
// KU > 0: k is the compile-time KU and all k loads of a chunk are issued before the first is used.
template <int KU>
__global__ __launch_bounds__(256) void moe_combine_kernel(const u32x4_t* __restrict__ Y, const float* __restrict__ w,
                                                          u32x4_t* __restrict__ out, int T, int k_rt, int N) {
    const int k = KU > 0 ? KU : k_rt;
    const int cpr = N >> 3;  // chunks per row
    const long long total = (long long)T * cpr;
    for (long long c = (long long)blockIdx.x * 256 + threadIdx.x; c < total; c += (long long)gridDim.x * 256) {
        const int t = (int)(c / cpr), col = (int)(c - (long long)t * cpr);
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        const u32x4_t* src = Y + ((size_t)t * k) * cpr + col;
        auto add = [&](const u32x4_t v, float wj) {
            acc[0] += wj * bf16_lo(v.x); acc[1] += wj * bf16_hi(v.x);
            acc[2] += wj * bf16_lo(v.y); acc[3] += wj * bf16_hi(v.y);
            acc[4] += wj * bf16_lo(v.z); acc[5] += wj * bf16_hi(v.z);
            acc[6] += wj * bf16_lo(v.w); acc[7] += wj * bf16_hi(v.w);
        };
        if constexpr (KU > 0) {
            u32x4_t v[KU];
            float wj[KU];
#pragma unroll
            for (int j = 0; j < KU; ++j) {
                v[j] = __builtin_nontemporal_load(src + (size_t)j * cpr);
                wj[j] = w ? w[(size_t)t * KU + j] : 1.f;
            }
#pragma unroll
            for (int j = 0; j < KU; ++j) add(v[j], wj[j]);
        } else {
            for (int j = 0; j < k; ++j) add(src[(size_t)j * cpr], w ? w[(size_t)t * k + j] : 1.f);
        }
        u32x4_t o;
        o.x = pack_bf16(acc[0], acc[1]); o.y = pack_bf16(acc[2], acc[3]);
        o.z = pack_bf16(acc[4], acc[5]); o.w = pack_bf16(acc[6], acc[7]);
        out[(size_t)t * cpr + col] = o;
    }
}

}  // namespace moe
