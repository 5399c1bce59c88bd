// Loss glue (paper Algorithm 2, loss line): mean softmax cross-entropy over all nodes and its
// gradient (softmax - onehot) / n.  One wavefront per node row; block partial sums of the loss
// are combined in a fixed order by a second kernel, so the result is deterministic.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kRowsPerBlock = 256;

__device__ inline float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ inline float ld_elem(const float* p) { return *p; }
__device__ inline float ld_elem(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
__device__ inline void st_elem(float* p, float x) { *p = x; }
__device__ inline void st_elem(uint16_t* p, float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + ((u >> 16) & 1u);
    *p = (uint16_t)(u >> 16);
}

// T: storage type of logits and dlogits (fp32, or bf16 widened to fp32 for the arithmetic).
template <typename T>
__global__ __launch_bounds__(kBlock) void xent_rows_kernel(const T* logits, int64_t ldl,
                                                           const int32_t* __restrict__ labels,
                                                           int64_t n, int c, T* dlogits,
                                                           int64_t ldd, double* __restrict__ part)
{
    __shared__ double wsum[kBlock / kWave];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t r_begin = (int64_t)blockIdx.x * kRowsPerBlock;
    const int64_t r_end = (r_begin + kRowsPerBlock) < n ? (r_begin + kRowsPerBlock) : n;
    const float inv_n = 1.0f / (float)n;
    double acc = 0.0;
    for (int64_t r = r_begin + w; r < r_end; r += kBlock / kWave) {
        const T* x = logits + r * ldl;
        float mx = -INFINITY;
        for (int j = lane; j < c; j += kWave) mx = fmaxf(mx, ld_elem(x + j));
        mx = wave_max(mx);
        float se = 0.f;
        for (int j = lane; j < c; j += kWave) se += expf(ld_elem(x + j) - mx);
        se = wave_sum(se);
        const float lse = mx + logf(se);
        const int y = labels[r];
        const float xy = ld_elem(x + y);
        for (int j = lane; j < c; j += kWave) {
            const float p = expf(ld_elem(x + j) - lse);
            st_elem(dlogits + r * ldd + j, (p - (j == y ? 1.f : 0.f)) * inv_n);
        }
        acc += (double)(lse - xy);
    }
    if (lane == 0) wsum[w] = acc;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ __launch_bounds__(kBlock) void xent_final_kernel(const double* __restrict__ part,
                                                            int64_t n_parts, int64_t n,
                                                            double* __restrict__ loss)
{
    __shared__ double sh[kBlock];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < n_parts; i += kBlock) s += part[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = kBlock / 2; o > 0; o >>= 1) {
        if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = sh[0] / (double)n;
}

}  // namespace

int launch_softmax_xent(int dtype, const void* logits, int64_t ldl, const int32_t* labels,
                        int64_t n, int32_t c, void* dlogits, int64_t ldd, double* loss,
                        hipStream_t s)
{
    const int64_t n_parts = ceil_div(n, kRowsPerBlock);
    void* scratch = nullptr;
    MIXGCN_TRY(get_scratch(1, (size_t)n_parts * sizeof(double), &scratch));
    if (dtype == MIXGCN_F32)
        hipLaunchKernelGGL(xent_rows_kernel<float>, dim3((unsigned)n_parts), dim3(kBlock), 0, s,
                           (const float*)logits, ldl, labels, n, c, (float*)dlogits, ldd,
                           (double*)scratch);
    else
        hipLaunchKernelGGL(xent_rows_kernel<uint16_t>, dim3((unsigned)n_parts), dim3(kBlock), 0, s,
                           (const uint16_t*)logits, ldl, labels, n, c, (uint16_t*)dlogits, ldd,
                           (double*)scratch);
    hipLaunchKernelGGL(xent_final_kernel, dim3(1), dim3(kBlock), 0, s, (const double*)scratch,
                       n_parts, n, loss);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace mixgcn
