// Stable least-significant-digit radix sort of 64-bit keys, 8 bits per pass.
// Per pass: (1) per-tile digit histogram, (2) exclusive scan of the digit-major histogram,
// (3) scatter with a stable rank computed per wave by ballot matching.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kRadixBits = 8;
constexpr int kRadix = 1 << kRadixBits;
constexpr int kSortItems = 16;                    // keys per thread
constexpr int kSortTile = kBlock * kSortItems;    // 4096 keys per block
constexpr int kWaveKeys = kWave * kSortItems;     // 1024 consecutive keys per wave

__global__ __launch_bounds__(kBlock) void radix_hist_kernel(const uint64_t* __restrict__ keys,
                                                            uint32_t* __restrict__ hist,
                                                            int64_t n, int shift, int64_t n_tiles)
{
    __shared__ uint32_t h[kRadix];
    h[threadIdx.x] = 0;
    __syncthreads();
    const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
    for (int j = 0; j < kSortItems; ++j) {
        const int64_t i = base + (int64_t)j * kBlock + threadIdx.x;
        if (i < n) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & (kRadix - 1)], 1u);
    }
    __syncthreads();
    hist[(int64_t)threadIdx.x * n_tiles + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kBlock) void radix_scatter_kernel(const uint64_t* __restrict__ keys,
                                                               uint64_t* __restrict__ out,
                                                               const uint64_t* __restrict__ offs,
                                                               int64_t n, int shift, int64_t n_tiles)
{
    __shared__ uint32_t whist[kBlock / kWave][kRadix];
    __shared__ uint64_t gbase[kRadix];
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < kBlock / kWave; ++i) whist[i][threadIdx.x] = 0;
    __syncthreads();

    // wave w owns the contiguous keys [base, base + 1024) and walks them 64 at a time
    const int64_t base = (int64_t)blockIdx.x * kSortTile + (int64_t)w * kWaveKeys;
    uint64_t key[kSortItems];
    uint32_t rank[kSortItems];
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t i = base + (int64_t)r * kWave + lane;
        const bool valid = i < n;
        key[r] = valid ? keys[i] : 0ull;
        const uint32_t d = (uint32_t)(key[r] >> shift) & (kRadix - 1);
        uint64_t m = __ballot(valid);
#pragma unroll
        for (int b = 0; b < kRadixBits; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t bal = __ballot(bit);
            m &= bit ? bal : ~bal;
        }
        // m: valid lanes of this round with my digit (includes me when valid)
        const int leader = m ? (__ffsll((unsigned long long)m) - 1) : 0;
        uint32_t prior = 0;
        if (valid && lane == leader) prior = atomicAdd(&whist[w][d], (uint32_t)__popcll(m));
        prior = __shfl(prior, leader, kWave);
        rank[r] = prior + (uint32_t)__popcll(m & lt_mask);
    }
    __syncthreads();
    {
        // thread t = digit t: turn per-wave counts into exclusive wave offsets
        const int d = threadIdx.x;
        uint32_t run = 0;
#pragma unroll
        for (int i = 0; i < kBlock / kWave; ++i) {
            const uint32_t c = whist[i][d];
            whist[i][d] = run;
            run += c;
        }
        gbase[d] = offs[(int64_t)d * n_tiles + blockIdx.x];
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kSortItems; ++r) {
        const int64_t i = base + (int64_t)r * kWave + lane;
        if (i < n) {
            const uint32_t d = (uint32_t)(key[r] >> shift) & (kRadix - 1);
            out[gbase[d] + whist[w][d] + rank[r]] = key[r];
        }
    }
}

}  // namespace

size_t sort_tmp_bytes(int64_t n)
{
    const int64_t n_tiles = ceil_div(n > 0 ? n : 1, kSortTile);
    const int64_t h = n_tiles * kRadix;
    // histogram (u32) + offsets (u64) + scan scratch
    return (size_t)h * 4 + 256 + (size_t)h * 8 + 256 + scan_tmp_bytes(h) + 256;
}

int radix_sort_u64(uint64_t* keys, uint64_t* alt, int64_t n, int n_bits, uint64_t** sorted,
                   void* tmp, hipStream_t s)
{
    *sorted = keys;
    if (n <= 1 || n_bits <= 0) return MIXGCN_OK;
    const int64_t n_tiles = ceil_div(n, kSortTile);
    const int64_t h = n_tiles * kRadix;
    char* p = (char*)tmp;
    uint32_t* hist = (uint32_t*)p;
    p += ((size_t)h * 4 + 255) / 256 * 256;
    uint64_t* offs = (uint64_t*)p;
    p += ((size_t)h * 8 + 255) / 256 * 256;
    void* scan_tmp = p;
    uint64_t* src = keys;
    uint64_t* dst = alt;
    for (int shift = 0; shift < n_bits; shift += kRadixBits) {
        hipLaunchKernelGGL(radix_hist_kernel, dim3((unsigned)n_tiles), dim3(kBlock), 0, s, src,
                           hist, n, shift, n_tiles);
        MIXGCN_TRY(exclusive_scan_u32_to_u64(hist, offs, h, nullptr, scan_tmp, s));
        hipLaunchKernelGGL(radix_scatter_kernel, dim3((unsigned)n_tiles), dim3(kBlock), 0, s, src,
                           dst, offs, n, shift, n_tiles);
        uint64_t* t = src;
        src = dst;
        dst = t;
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    *sorted = src;
    return MIXGCN_OK;
}

}  // namespace mixgcn
