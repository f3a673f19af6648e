// FPROP convolution for gfx950 (MI355X): the registry of tile variants and their launch, plus the
// register-only matrix-core loop.  The kernel itself is the template in conv_tile.h (the design
// notes are at its top); conv_variants_*.hip instantiate it.
#include <hip/hip_runtime.h>

#include <atomic>
#include <vector>

#include "gfx950_util.h"
#include "mdnn_internal.h"

namespace mdnn {

namespace {

// ---- register-only FP32 MFMA loop: the sustained matrix rate with no memory traffic
__global__ void __launch_bounds__(256) mfma_probe_kernel(float* sink, int iters)
{
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int v = 0; v < 16; ++v) { c0[v] = 0.f; c1[v] = 0.f; c2[v] = 0.f; c3[v] = 0.f; }
    const float a = 1.0f + (threadIdx.x & 3) * 0.25f;
    const float b = 1.0f / (float)(1 + (threadIdx.x & 7));
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

constexpr int kMaxEntries = 64;

const std::vector<VariantEntry>& entries()
{
    static const std::vector<VariantEntry> all = [] {
        std::vector<VariantEntry> v;
        const VariantEntry* (*const groups[])(int*) = {conv_variants_a, conv_variants_b, conv_variants_c, conv_variants_d,
                                                       conv_variants_e, conv_variants_f, conv_variants_g,
                                                       conv_variants_h, conv_variants_i};
        for (auto g : groups) {
            int n = 0;
            const VariantEntry* e = g(&n);
            for (int i = 0; i < n && (int)v.size() < kMaxEntries; ++i) v.push_back(e[i]);
        }
        return v;
    }();
    return all;
}

}  // namespace

int variant_count() { return (int)entries().size(); }
const VariantInfo& variant_info(int i) { return entries()[i].info; }
uint32_t variant_lds_bytes(int i, int tab_cap)
{
    return entries()[i].ring_bytes + (uint32_t)tab_cap * 8u;
}

int launch_variant(int i, const ConvParams& p, void* stream)
{
    const VariantEntry& e = entries()[i];
    const uint32_t lds = variant_lds_bytes(i, p.tab_cap);
    hipError_t err = hipSuccess;
    if (lds > 48u * 1024u) {
        // once per kernel, device and size class: a launch should only enqueue (a caller may be
        // capturing the stream into a graph)
        static std::atomic<uint64_t> raised[kMaxEntries];
        int dev = 0;
        err = hipGetDevice(&dev);
        if (err != hipSuccess) return (int)err;
        const uint64_t bit = 1ull << (dev & 63);
        if (!(raised[i].load(std::memory_order_acquire) & bit)) {
            err = hipFuncSetAttribute(reinterpret_cast<const void*>(e.fn),
                                      hipFuncAttributeMaxDynamicSharedMemorySize,
                                      (int)variant_lds_bytes(i, e.info.max_tab));
            if (err != hipSuccess) return (int)err;
            raised[i].fetch_or(bit, std::memory_order_release);
        }
    }
    const dim3 grid((unsigned)(p.front.wgs + 8 * p.tiles_per_xcd + p.back.wgs)), block((unsigned)e.info.threads);
    hipLaunchKernelGGL(e.fn, grid, block, lds, static_cast<hipStream_t>(stream), p);
    err = hipGetLastError();
    return (int)err;
}

int launch_mfma_probe(float* sink, int blocks, int waves_per_block, int iters, void* stream)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3((unsigned)(64 * waves_per_block)),
                       0, static_cast<hipStream_t>(stream), sink, iters);
    return (int)hipGetLastError();
}

}  // namespace mdnn
