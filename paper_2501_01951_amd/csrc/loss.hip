// Loss glue (paper Algorithm 2, loss line): mean softmax cross-entropy over all nodes and its
// gradient (softmax - onehot) / n.  A group of lanes per node row; block partial sums of the loss
// are combined in a fixed order by a second kernel, so the result is deterministic.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kRowsPerBlock = 256;

// reductions over the G lanes that share a node row (G a power of two, groups are lane aligned)
template <int G>
__device__ inline float group_max(float v)
{
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
template <int G>
__device__ inline float group_sum(float v)
{
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ inline float ld_elem(const float* p) { return *p; }
__device__ inline float ld_elem(const uint16_t* p) { return __uint_as_float((uint32_t)*p << 16); }
__device__ inline void ld_pair(const float* p, float& a, float& b)
{
    const float2 v = *reinterpret_cast<const float2*>(p);
    a = v.x;
    b = v.y;
}
__device__ inline void ld_pair(const uint16_t* p, float& a, float& b)
{
    const uint32_t u = *reinterpret_cast<const uint32_t*>(p);
    a = __uint_as_float(u << 16);
    b = __uint_as_float(u & 0xFFFF0000u);
}
__device__ inline void st_elem(float* p, float x) { *p = x; }
__device__ inline void st_elem(uint16_t* p, float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + ((u >> 16) & 1u);
    *p = (uint16_t)(u >> 16);
}

__device__ inline void st_pair(float* p, float a, float b)
{
    *reinterpret_cast<float2*>(p) = make_float2(a, b);
}
__device__ inline void st_pair(uint16_t* p, float a, float b)
{
    uint16_t lo, hi;
    st_elem(&lo, a);
    st_elem(&hi, b);
    *reinterpret_cast<uint32_t*>(p) = (uint32_t)lo | ((uint32_t)hi << 16);
}

// T: storage type of logits and dlogits (fp32, or bf16 widened to fp32 for the arithmetic).
// G lanes work on one node row, two neighboring classes each (G = the power of two that covers
// half the class count, at most 64), so a wavefront handles 64 / G rows at a time; more than 128
// classes are walked in a loop.
template <typename T, int G, bool PAIR>
__global__ __launch_bounds__(kBlock) void xent_rows_kernel(const T* logits, int64_t ldl,
                                                           const int32_t* __restrict__ labels,
                                                           int64_t n, int c, T* dlogits,
                                                           int64_t ldd, double* __restrict__ part)
{
    constexpr int RPW = kWave / G;  // rows per wavefront and trip
    __shared__ double wsum[kBlock / kWave];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int gl = lane % G, gi = lane / G;
    const int64_t r_begin = (int64_t)blockIdx.x * kRowsPerBlock;
    const int64_t r_end = (r_begin + kRowsPerBlock) < n ? (r_begin + kRowsPerBlock) : n;
    const float inv_n = 1.0f / (float)n;
    double acc = 0.0;
    for (int64_t r0 = r_begin + (int64_t)w * RPW; r0 < r_end; r0 += (kBlock / kWave) * RPW) {
        const int64_t r = r0 + gi;
        const bool live = r < r_end;
        const int64_t rr = live ? r : r_end - 1;  // idle groups redo the last row, write nothing
        const T* x = logits + rr * ldl;
        if (!PAIR && c <= G) {
            // one class per lane: the row is read once and stays in registers
            const bool has = gl < c;
            const float v = has ? ld_elem(x + gl) : -INFINITY;
            const float mx = group_max<G>(v);
            const float se = group_sum<G>(has ? expf(v - mx) : 0.f);
            const float lse = mx + logf(se);
            const int y = labels[rr];
            const float xy = __shfl(v, gi * G + y, kWave);
            if (live) {
                if (has) st_elem(dlogits + r * ldd + gl, (expf(v - lse) - (gl == y ? 1.f : 0.f)) * inv_n);
                if (gl == 0) acc += (double)(lse - xy);
            }
            continue;
        }
        if (PAIR && c <= 2 * G) {
            // two neighboring classes per lane (rows and pitches of whole pairs: the caller
            // checks): the row is read once, one 4- or 8-byte load per lane, and stays in
            // registers
            const int e0 = 2 * gl;
            const bool has0 = e0 < c, has1 = e0 + 1 < c;
            float v0, v1;
            ld_pair(x + (has0 ? e0 : 0), v0, v1);  // the pitch covers an odd row's last pair
            if (!has0) v0 = -INFINITY;
            if (!has1) v1 = -INFINITY;
            const float mx = group_max<G>(fmaxf(v0, v1));
            const float se = group_sum<G>((has0 ? expf(v0 - mx) : 0.f) + (has1 ? expf(v1 - mx) : 0.f));
            const float lse = mx + logf(se);
            const int y = labels[rr];
            const float xy = __shfl((y & 1) ? v1 : v0, gi * G + (y >> 1), kWave);
            if (live) {
                const float p0 = (expf(v0 - lse) - (e0 == y ? 1.f : 0.f)) * inv_n;
                const float p1 = (expf(v1 - lse) - (e0 + 1 == y ? 1.f : 0.f)) * inv_n;
                if (has1) st_pair(dlogits + r * ldd + e0, p0, p1);
                else if (has0) st_elem(dlogits + r * ldd + e0, p0);
                if (gl == 0) acc += (double)(lse - xy);
            }
            continue;
        }
        float mx = -INFINITY;
        for (int j = gl; j < c; j += G) mx = fmaxf(mx, ld_elem(x + j));
        mx = group_max<G>(mx);
        float se = 0.f;
        for (int j = gl; j < c; j += G) se += expf(ld_elem(x + j) - mx);
        se = group_sum<G>(se);
        const float lse = mx + logf(se);
        const int y = labels[rr];
        const float xy = ld_elem(x + y);
        if (live) {
            for (int j = gl; j < c; j += G) {
                const float p = expf(ld_elem(x + j) - lse);
                st_elem(dlogits + r * ldd + j, (p - (j == y ? 1.f : 0.f)) * inv_n);
            }
            if (gl == 0) acc += (double)(lse - xy);
        }
    }
    // the row leaders of a wavefront, in a fixed order
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, kWave);
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
    // two classes per lane need rows that start and end on whole pairs
    const size_t es = dtype == MIXGCN_F32 ? 4 : 2;
    const bool pair = ldl % 2 == 0 && ldd % 2 == 0 && (uintptr_t)logits % (2 * es) == 0 &&
                      (uintptr_t)dlogits % (2 * es) == 0;
#define MIXGCN_XENT(T, G, PAIR)                                                                  \
    hipLaunchKernelGGL((xent_rows_kernel<T, G, PAIR>), dim3((unsigned)n_parts), dim3(kBlock), 0, s, \
                       (const T*)logits, ldl, labels, n, c, (T*)dlogits, ldd, (double*)scratch)
#define MIXGCN_XENT_G(T)                                                                         \
    do {                                                                                         \
        const int cover = pair ? (c + 1) / 2 : c; /* lanes a row needs */                        \
        if (cover <= 4) { if (pair) MIXGCN_XENT(T, 4, true); else MIXGCN_XENT(T, 4, false); }    \
        else if (cover <= 8) { if (pair) MIXGCN_XENT(T, 8, true); else MIXGCN_XENT(T, 8, false); } \
        else if (cover <= 16) { if (pair) MIXGCN_XENT(T, 16, true); else MIXGCN_XENT(T, 16, false); } \
        else if (cover <= 32) { if (pair) MIXGCN_XENT(T, 32, true); else MIXGCN_XENT(T, 32, false); } \
        else { if (pair) MIXGCN_XENT(T, 64, true); else MIXGCN_XENT(T, 64, false); }             \
    } while (0)
    if (dtype == MIXGCN_F32) MIXGCN_XENT_G(float);
    else MIXGCN_XENT_G(uint16_t);
#undef MIXGCN_XENT_G
#undef MIXGCN_XENT
    hipLaunchKernelGGL(xent_final_kernel, dim3(1), dim3(kBlock), 0, s, (const double*)scratch,
                       n_parts, n, loss);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace mixgcn
