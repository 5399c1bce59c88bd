// Attainable rates of this device, measured with kernels that do nothing else: a streaming copy
// (HBM read + write) and back-to-back MFMA chains on registers (no memory traffic).  They put
// the published peaks that the roofline fractions are quoted against next to what the part
// sustains at its running clocks.
#include <vector>

#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// n4 is a multiple of 4 * gridDim.x * blockDim.x: four independent 16-byte loads per trip
__global__ __launch_bounds__(kBlock) void copy_kernel(const float4* __restrict__ in,
                                                      float4* __restrict__ out, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += 4 * stride) {
        const float4 a = in[i], b = in[i + stride], c = in[i + 2 * stride], d = in[i + 3 * stride];
        out[i] = a;
        out[i + stride] = b;
        out[i + 2 * stride] = c;
        out[i + 3 * stride] = d;
    }
}

__global__ __launch_bounds__(kBlock) void read_kernel(const float4* __restrict__ in,
                                                      float* __restrict__ out, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    float s = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += 4 * stride) {
        const float4 a = in[i], b = in[i + stride], c = in[i + 2 * stride], d = in[i + 3 * stride];
        s += (a.x + a.y + a.z + a.w) + (b.x + b.y + b.z + b.w) + (c.x + c.y + c.z + c.w) +
             (d.x + d.y + d.z + d.w);
    }
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Random 128-byte gathers: every group of 8 lanes reads one pseudo-random line of the buffer
// (16 bytes per lane), four independent loads in flight per lane, nothing else.  line_mask + 1
// lines (a power of two) are addressed.
__global__ __launch_bounds__(kBlock) void gather_kernel(const uint4* __restrict__ buf,
                                                        uint32_t line_mask, int iters,
                                                        uint4* __restrict__ out)
{
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t grp = t >> 3, lj = t & 7;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (int it = 0; it < iters; it += 4) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            uint32_t x = (grp * (uint32_t)iters + (uint32_t)(it + u)) * 0x9E3779B1u;
            x ^= x >> 15;
            x *= 0x85EBCA77u;
            x ^= x >> 13;
            v[u] = buf[(size_t)(x & line_mask) * 8 + lj];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            acc.x ^= v[u].x;
            acc.y ^= v[u].y;
            acc.z ^= v[u].z;
            acc.w ^= v[u].w;
        }
    }
    out[t] = acc;
}

constexpr int kChains = 4;  // independent accumulators per wavefront

__global__ __launch_bounds__(kBlock) void mfma_f32_loop_kernel(float* out, int iters, float seed)
{
    floatx16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
    const float a = seed + (float)(threadIdx.x & 3), b = seed * 0.5f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c)
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[c][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

__global__ __launch_bounds__(kBlock) void mfma_bf16_loop_kernel(float* out, int iters, float seed)
{
    floatx16 acc[kChains];
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(seed + (float)((threadIdx.x + e) & 3));
        b[e] = (__bf16)(seed * 0.5f);
    }
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int c = 0; c < kChains; ++c)
            acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < kChains; ++c)
#pragma unroll
        for (int v = 0; v < 16; ++v) s += acc[c][v];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

struct Events {
    hipEvent_t a = nullptr, b = nullptr;
    ~Events()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

struct DevBuf {
    void* p = nullptr;
    ~DevBuf()
    {
        if (p) (void)hipFree(p);
    }
};

}  // namespace
}  // namespace mixgcn

using namespace mixgcn;

extern "C" int mixgcn_measure_peaks(double* read_gbs, double* copy_gbs, double* gather_l2_gbs,
                                    double* gather_hbm_gbs, double* mfma_f32_tflops,
                                    double* mfma_bf16_tflops, void* stream)
{
    if (!read_gbs || !copy_gbs || !gather_l2_gbs || !gather_hbm_gbs || !mfma_f32_tflops ||
        !mfma_bf16_tflops)
        return fail(MIXGCN_EINVAL, "measure_peaks: null output");
    hipStream_t s = (hipStream_t)stream;
    int dev = 0, n_cu = 0;
    MIXGCN_HIP_TRY(hipGetDevice(&dev));
    MIXGCN_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    Events ev;
    MIXGCN_HIP_TRY(hipEventCreate(&ev.a));
    MIXGCN_HIP_TRY(hipEventCreate(&ev.b));
    float ms = 0.f;

    // streaming copy of 4 GiB (read 4 GiB + write 4 GiB), third of three runs
    const int64_t bytes = 4ll << 30, n4 = bytes / 16;
    DevBuf src, dst;
    MIXGCN_HIP_TRY(hipMalloc(&src.p, (size_t)bytes));
    MIXGCN_HIP_TRY(hipMalloc(&dst.p, (size_t)bytes));
    const unsigned copy_grid = 8192;  // 4 * 8192 * 256 float4 = 128 MiB per trip of the loop
    hipLaunchKernelGGL(copy_kernel, dim3(copy_grid), dim3(kBlock), 0, s, (const float4*)dst.p,
                       (float4*)src.p, n4);  // first touch of both buffers
    for (int rep = 0; rep < 3; ++rep) {
        MIXGCN_HIP_TRY(hipEventRecord(ev.a, s));
        hipLaunchKernelGGL(copy_kernel, dim3(copy_grid), dim3(kBlock), 0, s, (const float4*)src.p,
                           (float4*)dst.p, n4);
        MIXGCN_HIP_TRY(hipEventRecord(ev.b, s));
        MIXGCN_HIP_TRY(hipEventSynchronize(ev.b));
        MIXGCN_HIP_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
    }
    *copy_gbs = 2.0 * (double)bytes / ((double)ms * 1e-3) / 1e9;
    DevBuf sums;
    MIXGCN_HIP_TRY(hipMalloc(&sums.p, (size_t)copy_grid * kBlock * sizeof(float)));
    for (int rep = 0; rep < 3; ++rep) {
        MIXGCN_HIP_TRY(hipEventRecord(ev.a, s));
        hipLaunchKernelGGL(read_kernel, dim3(copy_grid), dim3(kBlock), 0, s, (const float4*)src.p,
                           (float*)sums.p, n4);
        MIXGCN_HIP_TRY(hipEventRecord(ev.b, s));
        MIXGCN_HIP_TRY(hipEventSynchronize(ev.b));
        MIXGCN_HIP_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
    }
    *read_gbs = (double)bytes / ((double)ms * 1e-3) / 1e9;

    // random 128-byte lines: from 2 MiB (every L2 holds it: the L2 -> L1 fill rate) and from
    // the whole 4 GiB buffer (every line comes from HBM)
    {
        const unsigned ggrid = (unsigned)n_cu * 32;  // 8 workgroups per SIMD row, 4 x 8 waves
        const int giters = 256;
        const double gbytes = (double)ggrid * kBlock * giters * 16.0;
        const uint32_t masks[2] = {(2u << 20) / 128 - 1, (uint32_t)(bytes / 128 - 1)};
        double* outs[2] = {gather_l2_gbs, gather_hbm_gbs};
        DevBuf gout;
        MIXGCN_HIP_TRY(hipMalloc(&gout.p, (size_t)ggrid * kBlock * sizeof(uint4)));
        for (int k = 0; k < 2; ++k) {
            for (int rep = 0; rep < 3; ++rep) {
                MIXGCN_HIP_TRY(hipEventRecord(ev.a, s));
                hipLaunchKernelGGL(gather_kernel, dim3(ggrid), dim3(kBlock), 0, s,
                                   (const uint4*)src.p, masks[k], giters, (uint4*)gout.p);
                MIXGCN_HIP_TRY(hipEventRecord(ev.b, s));
                MIXGCN_HIP_TRY(hipEventSynchronize(ev.b));
                MIXGCN_HIP_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
            }
            *outs[k] = gbytes / ((double)ms * 1e-3) / 1e9;
        }
    }

    // MFMA chains: 2 workgroups of 4 wavefronts per CU, kChains accumulators each
    const unsigned grid = (unsigned)n_cu * 2;
    const int iters = 20000;
    float* out = (float*)dst.p;
    const double waves = (double)grid * (kBlock / kWave);
    for (int rep = 0; rep < 2; ++rep) {
        MIXGCN_HIP_TRY(hipEventRecord(ev.a, s));
        hipLaunchKernelGGL(mfma_f32_loop_kernel, dim3(grid), dim3(kBlock), 0, s, out, iters, 1.0f);
        MIXGCN_HIP_TRY(hipEventRecord(ev.b, s));
        MIXGCN_HIP_TRY(hipEventSynchronize(ev.b));
        MIXGCN_HIP_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
    }
    *mfma_f32_tflops = waves * iters * kChains * (2.0 * 32 * 32 * 2) / ((double)ms * 1e-3) / 1e12;
    for (int rep = 0; rep < 2; ++rep) {
        MIXGCN_HIP_TRY(hipEventRecord(ev.a, s));
        hipLaunchKernelGGL(mfma_bf16_loop_kernel, dim3(grid), dim3(kBlock), 0, s, out, iters, 1.0f);
        MIXGCN_HIP_TRY(hipEventRecord(ev.b, s));
        MIXGCN_HIP_TRY(hipEventSynchronize(ev.b));
        MIXGCN_HIP_TRY(hipEventElapsedTime(&ms, ev.a, ev.b));
    }
    *mfma_bf16_tflops = waves * iters * kChains * (2.0 * 32 * 32 * 16) / ((double)ms * 1e-3) / 1e12;
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}
