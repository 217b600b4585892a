// C-ABI entry points of libmoe_probe: the measurement kernels, kept out of the product library.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/moe_probe.h"
#include "probe_kernels.hpp"

namespace {

constexpr int kOk = 0, kInvalid = -1, kHip = -4;
std::mutex g_attr_lock;

// The large-LDS attribute of a kernel is set once per device (bit d of *done: device d, d < 64).
int ensure_lds_attr(const void* fn, int lds, unsigned long long* done) {
    std::lock_guard<std::mutex> hold(g_attr_lock);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return kHip;
    const unsigned long long bit = dev >= 0 && dev < 64 ? 1ull << dev : 0;
    if (bit && (*done & bit)) return kOk;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess) return kHip;
    *done |= bit;
    return kOk;
}

}  // namespace

extern "C" {

int moe_probe_mfma(int block, int random_operands, int iters, void* sink, void* stream) {
    if ((block != 16 && block != 32) || iters < 1 || !sink) return kInvalid;
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* out = static_cast<float*>(sink);
    if (block == 16) {
        if (random_operands) moe::mfma_probe_kernel<16, true><<<256, 512, 0, s>>>(iters, out);
        else moe::mfma_probe_kernel<16, false><<<256, 512, 0, s>>>(iters, out);
    } else {
        if (random_operands) moe::mfma_probe_kernel<32, true><<<256, 512, 0, s>>>(iters, out);
        else moe::mfma_probe_kernel<32, false><<<256, 512, 0, s>>>(iters, out);
    }
    return hipGetLastError() == hipSuccess ? kOk : kHip;
}

int moe_probe_pipeline(int mode, int iters, const void* src, size_t src_bytes, void* sink, void* stream) {
    const size_t need = (mode == 4 || mode == 12) ? (size_t(513) << 20) : (size_t(1) << 20);
    if (mode < 1 || mode > 12 || iters < 2 || (iters & 1) || !src || !sink || src_bytes < need ||
        (reinterpret_cast<uintptr_t>(src) & 15))
        return kInvalid;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const char* in = static_cast<const char*>(src);
    float* out = static_cast<float*>(sink);
    constexpr int lds = 96 * 1024;   // one workgroup per CU, as for the tile it imitates
    static unsigned long long done[12] = {0};
    auto go = [&](auto kernel, unsigned long long* d) {
        if (ensure_lds_attr(reinterpret_cast<const void*>(kernel), lds, d) != kOk) return int(kHip);
        kernel<<<256, 512, lds, s>>>(iters, in, out);
        return hipGetLastError() == hipSuccess ? int(kOk) : int(kHip);
    };
    switch (mode) {
        case 1: return go(&moe::pipeline_probe_kernel<1>, &done[0]);
        case 2: return go(&moe::pipeline_probe_kernel<2>, &done[1]);
        case 3: return go(&moe::pipeline_probe_kernel<3>, &done[2]);
        case 4: return go(&moe::pipeline_probe_kernel<4>, &done[3]);
        case 5: return go(&moe::pipeline_probe_kernel<5>, &done[4]);
        case 6: return go(&moe::pipeline_probe_kernel<6>, &done[5]);
        case 7: return go(&moe::pipeline_probe_kernel<7>, &done[6]);
        case 8: return go(&moe::pipeline_probe_kernel<8>, &done[7]);
        case 9: return go(&moe::pipeline_probe_kernel<9>, &done[8]);
        case 10: return go(&moe::pipeline_pingpong_kernel<10>, &done[9]);
        case 11: return go(&moe::pipeline_pingpong_kernel<11>, &done[10]);
        default: return go(&moe::pipeline_pingpong_kernel<12>, &done[11]);
    }
}

int moe_probe_wave_placement(int workgroups, int32_t* out, void* stream) {
    if (workgroups < 1 || workgroups > 65536 || !out) return kInvalid;
    constexpr int lds = 150 * 1024;   // one workgroup per CU
    static unsigned long long done = 0;
    if (ensure_lds_attr(reinterpret_cast<const void*>(&moe::wave_placement_kernel), lds, &done) != kOk) return kHip;
    moe::wave_placement_kernel<<<workgroups, 512, lds, static_cast<hipStream_t>(stream)>>>(out);
    return hipGetLastError() == hipSuccess ? kOk : kHip;
}

}  // extern "C"
