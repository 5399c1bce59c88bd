// Device-wide exclusive prefix sum (uint32 or uint64 counts -> uint64 offsets), three phases:
// tile sums, recursive scan of the tile sums, per-tile scan with the tile offset added.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kScanItems = 8;
constexpr int kScanTile = kBlock * kScanItems;  // 2048

template <typename TIn>
__global__ __launch_bounds__(kBlock) void scan_tile_sums_kernel(const TIn* __restrict__ in,
                                                                uint64_t* __restrict__ sums,
                                                                int64_t n)
{
    __shared__ uint64_t lds[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint64_t s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j)
        if (base + j < n) s += (uint64_t)in[base + j];
    uint64_t total;
    block_exclusive_scan_u64(s, &total, lds);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// out may alias in (uint64 case): every thread reads its items before any thread writes.
template <typename TIn>
__global__ __launch_bounds__(kBlock) void scan_tile_apply_kernel(const TIn* in, uint64_t* out,
                                                                 const uint64_t* tile_off,
                                                                 uint64_t* total_out, int64_t n)
{
    __shared__ uint64_t lds[4];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint64_t v[kScanItems];
    uint64_t s = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = (base + j < n) ? (uint64_t)in[base + j] : 0;
        s += v[j];
    }
    uint64_t total;
    uint64_t run = block_exclusive_scan_u64(s, &total, lds) + (tile_off ? tile_off[blockIdx.x] : 0);
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (base + j < n) out[base + j] = run;
        run += v[j];
    }
    if (total_out && blockIdx.x == 0 && threadIdx.x == 0 && !tile_off) *total_out = total;
}

template <typename TIn>
int scan_rec(const TIn* in, uint64_t* out, int64_t n, uint64_t* total, uint64_t* tmp, hipStream_t s)
{
    const int64_t nb = ceil_div(n, kScanTile);
    if (nb <= 1) {
        hipLaunchKernelGGL((scan_tile_apply_kernel<TIn>), dim3(1), dim3(kBlock), 0, s, in, out,
                           (const uint64_t*)nullptr, total, n);
        return MIXGCN_OK;
    }
    uint64_t* sums = tmp;  // nb entries, then the next level's scratch
    hipLaunchKernelGGL((scan_tile_sums_kernel<TIn>), dim3((unsigned)nb), dim3(kBlock), 0, s, in,
                       sums, n);
    MIXGCN_TRY(scan_rec<uint64_t>(sums, sums, nb, total, tmp + nb, s));
    hipLaunchKernelGGL((scan_tile_apply_kernel<TIn>), dim3((unsigned)nb), dim3(kBlock), 0, s, in,
                       out, (const uint64_t*)sums, (uint64_t*)nullptr, n);
    return MIXGCN_OK;
}

}  // namespace

size_t scan_tmp_bytes(int64_t n)
{
    size_t words = 16;
    while (n > kScanTile) {
        n = ceil_div(n, kScanTile);
        words += (size_t)n;
    }
    return words * sizeof(uint64_t);
}

int exclusive_scan_u32_to_u64(const uint32_t* in, uint64_t* out, int64_t n, uint64_t* total,
                              void* tmp, hipStream_t s)
{
    if (n <= 0) {
        if (total) MIXGCN_HIP_TRY(hipMemsetAsync(total, 0, sizeof(uint64_t), s));
        return MIXGCN_OK;
    }
    MIXGCN_TRY(scan_rec<uint32_t>(in, out, n, total, (uint64_t*)tmp, s));
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace mixgcn
