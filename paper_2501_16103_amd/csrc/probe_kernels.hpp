// Measurement kernels (not part of the method): the sustained MFMA rate of the chip without memory traffic, and
// the inner loop of the 256x256x64 bf16 tile assembled one ingredient at a time.  Built into their own library
// (libmoe_probe.so); the product library does not contain them.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace moe {

// Measurement aid: bf16 MFMAs on register operands and nothing else, two wavefronts per SIMD (512 threads, one
// workgroup per CU).  Per loop trip and wavefront 512 KFLOP: 32 MFMAs of 16x16x32 or 16 of 32x32x16, every
// accumulator independent of the others, 128 accumulator registers either way.
template <int BLOCK, bool RANDOM>
__global__ void __launch_bounds__(512) mfma_probe_kernel(int iters, float* sink) {
    auto bits = [](uint32_t i) {   // two bf16 values of magnitude 2^-3 .. 2, random sign and mantissa
        uint32_t h = i * 2654435761u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; h *= 3266489917u; h ^= h >> 16;
        const uint32_t lo = (h & 0x807fu) | (0x3e00u + ((h >> 16) & 0x0180u));
        const uint32_t hi = ((h >> 8) & 0x807fu) | (0x3e00u + ((h >> 20) & 0x0180u));
        return RANDOM ? (lo | (hi << 16)) : 0x3f803f80u;
    };
    const uint32_t seed = (blockIdx.x * 977u + threadIdx.x) * 64u;
    bf16x8_t fa[4], fb[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const u32x4_t v = {bits(seed + 4 * i), bits(seed + 4 * i + 1), bits(seed + 4 * i + 2), bits(seed + 4 * i + 3)};
        fa[i] = __builtin_bit_cast(bf16x8_t, v);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const u32x4_t v = {bits(seed + 16 + 4 * i), bits(seed + 17 + 4 * i), bits(seed + 18 + 4 * i), bits(seed + 19 + 4 * i)};
        fb[i] = __builtin_bit_cast(bf16x8_t, v);
    }
    float sum = 0.f;
    if constexpr (BLOCK == 16) {
        f32x4_t acc[32];
#pragma unroll
        for (int i = 0; i < 32; ++i) acc[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i * 8 + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa[i], fb[j], acc[i * 8 + j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 32; ++i) sum += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    } else {
        f32x16_t acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i + 2 * h], fb[j + 4 * h], acc[i * 4 + j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += acc[i][j];
    }
    if (sum == 12345.f) sink[0] = sum;   // keeps the loop alive; practically never true
}

// Measurement aid: the inner loop of the 256x256x64 bf16 tile without its arithmetic on addresses -- eight
// wavefronts, each with a 128x64 accumulator block of 16x16x32 MFMAs -- built up one ingredient at a time, so
// that the cost of each shows against the pure-MFMA rate:
//   MODE 1: the LDS fragment reads of a k-step (8 of 16 bytes, 8 transposing ones of 8 bytes), double-buffered
//   MODE 2: + one workgroup barrier per 64-deep k-tile
//   MODE 3: + the k-tile's 64 KB of global->LDS DMA (8 instructions per thread), source resident in cache
//   MODE 4: as 3, but half of the bytes come from lines not touched before (a new 32 KB chunk of `src` per k-tile,
//           shared by two workgroups), about the weight traffic the real kernel draws from HBM
//   MODE 5-8: no MFMAs, the LDS pipe alone: the 16-byte reads, the transposing reads, both, the DMA writes
//   MODE 9: no MFMAs, both kinds of reads AND the DMA writes together (do they share the LDS pipe's time or overlap?)
// `src`: at least 1 MB (MODE 4: 513 MB) of device memory; its first 64 KB fill the LDS region the fragments are
// read from, so bf16 values there make the operands realistic.  Per loop trip (two k-steps) and wavefront 1 MFLOP.
template <int MODE>
__global__ void __launch_bounds__(512) pipeline_probe_kernel(int iters, const char* src, float* sink) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    constexpr int MB = 8, NB = 4;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < 65536 / 16; i += 512) reinterpret_cast<u32x4_t*>(smem)[i] = reinterpret_cast<const u32x4_t*>(src)[i];
    __syncthreads();
    f32x4_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    u32x4_t xq[2][MB];
    u32x2_t wq[2][NB][2];
    // fragments of k-step `it`: conflict-free addresses inside [0, 64 KB), different from step to step
    auto load = [&](int buf, int it) __attribute__((always_inline)) {
        int base = (it & 3) * 16384 + (wave & 1) * 8192;
        asm volatile("" : "+v"(base));
        if (MODE != 6) {
#pragma unroll
            for (int i = 0; i < MB; ++i) xq[buf][i] = *reinterpret_cast<const u32x4_t*>(smem + base + lane * 16 + i * 1024);
        }
        if (MODE != 5) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    wq[buf][j][h] = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (MOE_LDS(s16x4_t)*)(smem + ((base + lane * 8 + (j * 2 + h) * 512) & 65535))));
        }
    };
    auto mma = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const u32x4_t wv = {wq[buf][j][0].x, wq[buf][j][0].y, wq[buf][j][1].x, wq[buf][j][1].y};
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv),
                                                                    __builtin_bit_cast(bf16x8_t, xq[buf][i]), acc[i][j], 0, 0, 0);
            }
    };
    // DMA target: LDS [64 KB, 96 KB), apart from the fragments; sources stay inside `src` by construction:
    // cached part: offsets < 17 * 32 KB + 32 KB <= 1 MB; fresh part: 1 MB + chunk (< 512 MB) + 32 KB
    const uint32_t lds0 = (uint32_t)(uintptr_t)(MOE_LDS(char)*)smem;
    auto dmas = [&](int it, int half) __attribute__((always_inline)) {
        const uint32_t chunk = (((blockIdx.x >> 1) * 4099u + static_cast<uint32_t>(it >> 1)) & 16383u) * 32768u;
        const char* src_w = MODE == 4 ? src + (1u << 20) + chunk : src + 32768 + (blockIdx.x & 15) * 32768;
        const char* src_x = src + (blockIdx.x & 7) * 32768;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            dma16(lane * 16 + wave * 1024 + r * 8192, half ? src_w : src_x, lds0 + 65536 + r * 8192 + wave * 1024);
    };
    if constexpr (MODE >= 5) {
        // no MFMAs: the LDS pipe alone.  5: the 16-byte reads of a k-step, 6: its transposing 8-byte reads,
        // 7: both, 8: the k-tile's DMA writes (cache-resident source)
        for (int it = 0; it < iters; it += 2) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (MODE <= 7 || MODE == 9) load(h, it + h);
                if (MODE == 5 || MODE == 7 || MODE == 9) {
#pragma unroll
                    for (int i = 0; i < MB; ++i) asm volatile("" ::"v"(xq[h][i]));
                }
                if (MODE == 6 || MODE == 7 || MODE == 9) {
#pragma unroll
                    for (int j = 0; j < NB; ++j) asm volatile("" ::"v"(wq[h][j][0]), "v"(wq[h][j][1]));
                }
                if (MODE == 8 || MODE == 9) { dmas(it, h); wait_vmcnt<4>(); }
            }
        }
        if (MODE == 8 || MODE == 9) wait_vmcnt<0>();
        if (iters < 0) sink[0] = 0.f;
        return;
    }
    load(0, 0);
    for (int it = 0; it < iters; it += 2) {
        load(1, it + 1);
        if (MODE >= 3) dmas(it, 0);
        mma(0);
        load(0, it + 2);
        if (MODE >= 3) dmas(it, 1);
        mma(1);
        if (MODE >= 3) wait_vmcnt<8>();      // the previous k-tile's DMA has landed
        if (MODE >= 2) __syncthreads();
    }
    if (MODE >= 3) wait_vmcnt<0>();
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) sum += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    if (sum == 12345.678f) sink[0] = sum;   // keeps the loop alive; practically never true
}

// Measurement aid: the same ingredients as pipeline_probe_kernel, scheduled as two alternating roles instead of one
// interleaved stream (the schedule of the large bf16 tile's k loop).  The two wavefronts of a SIMD take opposite
// roles (decided from the hardware's SIMD id, first come first served); a k-step is two slots separated by
// workgroup barriers, and in every slot one role issues its k-step's MFMAs back to back, all fragments already in
// registers, while the other role does nothing but reload its (single-buffered) fragments for its next k-step.
// Four barriers per 64-deep k-tile instead of one; no wavefront ever waits on an LDS read inside its MFMA run.
//   MODE 10: MFMAs + LDS fragment reads;  11: + the k-tile's 64 KB of DMA, cache-resident source;  12: as 11 with
//   half of the bytes from lines not touched before (the sources of modes 3 and 4 of the probe above)
// DMA instructions: four per wavefront in the slot after the k-tile's third barrier, four in the wavefront's next
// MFMA slot; inside an MFMA slot they follow the first MFMAs, one each.
template <int MODE>
__global__ void __launch_bounds__(512) pipeline_pingpong_kernel(int iters, const char* src, float* sink) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    __shared__ int waves_on_simd[4];
    constexpr int MB = 8, NB = 4;
    constexpr bool DMA = MODE >= 11;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < 65536 / 16; i += 512) reinterpret_cast<u32x4_t*>(smem)[i] = reinterpret_cast<const u32x4_t*>(src)[i];
    if (tid < 4) waves_on_simd[tid] = 0;
    __syncthreads();
    // HW_ID bits 5:4: the SIMD this wavefront runs on
    const int simd = __builtin_amdgcn_s_getreg((1 << 11) | (4 << 6) | 4) & 3;
    int arrival = 0;
    if (lane == 0) arrival = atomicAdd(&waves_on_simd[simd], 1);
    const int role = __builtin_amdgcn_readfirstlane(arrival) & 1;
    __syncthreads();

    f32x4_t acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    u32x4_t xq[MB];
    u32x2_t wq[NB][2];
    auto lgkm0 = []() __attribute__((always_inline)) { __builtin_amdgcn_s_waitcnt(0xc07f); };
    // memory slot: fragments of k-step `it` (addresses as in the probe above)
    auto load = [&](int it) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        int base = (it & 3) * 16384 + (wave & 1) * 8192;
        asm volatile("" : "+v"(base));
#pragma unroll
        for (int i = 0; i < MB; ++i) xq[i] = *reinterpret_cast<const u32x4_t*>(smem + base + lane * 16 + i * 1024);
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                wq[j][h] = __builtin_bit_cast(u32x2_t, __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (MOE_LDS(s16x4_t)*)(smem + ((base + lane * 8 + (j * 2 + h) * 512) & 65535))));
    };
    const uint32_t lds0 = (uint32_t)(uintptr_t)(MOE_LDS(char)*)smem;
    // d-th of a wavefront's 8 DMA instructions of a k-tile (0-3 token half, 4-7 weight half; targets and sources as
    // in the probe above)
    auto dma_one = [&](int it, int d) __attribute__((always_inline)) {
        const uint32_t chunk = (((blockIdx.x >> 1) * 4099u + static_cast<uint32_t>(it >> 1)) & 16383u) * 32768u;
        const char* src_w = MODE == 12 ? src + (1u << 20) + chunk : src + 32768 + (blockIdx.x & 15) * 32768;
        const char* src_x = src + (blockIdx.x & 7) * 32768;
        const int r = d & 3;
        dma16(lane * 16 + wave * 1024 + r * 8192, (d & 4) ? src_w : src_x, lds0 + 65536 + r * 8192 + wave * 1024);
    };
    // compute slot: the k-step's 32 MFMAs, DMA instructions d0 .. d0 + nd - 1 behind the first nd of them
    auto mma = [&](int it, int d0, int nd) __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int i = 0; i < MB; ++i) {
                const u32x4_t wv = {wq[j][0].x, wq[j][0].y, wq[j][1].x, wq[j][1].y};
                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wv),
                                                                    __builtin_bit_cast(bf16x8_t, xq[i]), acc[i][j], 0, 0, 0);
                if (DMA && j * MB + i < nd) { dma_one(it, d0 + j * MB + i); __builtin_amdgcn_sched_barrier(0); }
            }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto bar = []() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };
    // Both roles pass the same four barriers per trip.  The wait on the DMA ring sits before the third one in both
    // (all but the newest half of a k-tile's instructions have landed: the token half of the tile before).
    if (role == 0) {
        load(0);
        lgkm0();
        for (int it = 0; it < iters; it += 2) {
            mma(it, 4, 4);
            bar();
            load(it + 1);
            lgkm0();
            bar();
            mma(it, 0, 0);
            if (DMA) wait_vmcnt<4>();
            bar();
            load(it + 2);
            if (DMA) {
#pragma unroll
                for (int d = 0; d < 4; ++d) dma_one(it, d);
            }
            lgkm0();
            bar();
        }
    } else {
        for (int it = 0; it < iters; it += 2) {
            load(it);
            lgkm0();
            bar();
            mma(it, 4, 4);
            bar();
            load(it + 1);
            lgkm0();
            if (DMA) wait_vmcnt<4>();
            bar();
            mma(it, 0, 4);
            bar();
        }
    }
    if (DMA) wait_vmcnt<0>();
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) sum += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
    if (sum == 12345.678f) sink[0] = sum;   // keeps the loop alive; practically never true
}

// Measurement aid: where the hardware puts the eight wavefronts of a 512-thread workgroup that has a CU to itself
// (the large tiles' launch shape).  out[8 * workgroup + w] = SIMD (0..3) that wavefront w runs on.  The alternating
// schedule of the large bf16 tiles gives wavefronts w and w + 4 opposite roles because they share a SIMD; if a
// device placed them otherwise the results would be the same and only the schedule's benefit would be lost.
__global__ void __launch_bounds__(512) wave_placement_kernel(int* out) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int simd = __builtin_amdgcn_s_getreg((1 << 11) | (4 << 6) | 4) & 3;   // HW_ID bits 5:4
    if ((threadIdx.x & 63) == 0) out[blockIdx.x * 8 + (threadIdx.x >> 6)] = simd;
    if (simd > 3) smem[threadIdx.x] = 1;   // never true: keeps the LDS allocation, which is what gives the workgroup its own CU
}

}  // namespace moe
