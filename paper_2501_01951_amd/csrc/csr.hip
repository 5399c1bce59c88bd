// CSR construction of A_tilde = A + I from an edge list (paper Sec. 2.1) and the symmetric
// normalisation A_hat = D^-1/2 A_tilde D^-1/2.  Integer work: key emission, radix sort,
// duplicate removal by a tiled compaction, row pointers, per-group start rows.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kCompactItems = 8;
constexpr int kCompactTile = kBlock * kCompactItems;

// key = row << bits | col; self edges become the diagonal key when the diagonal is added anyway
// (the duplicate is removed later), otherwise the drop marker 1 << 2*bits, which sorts last.
__global__ __launch_bounds__(kBlock) void emit_keys_kernel(
    const uint32_t* __restrict__ src, const uint32_t* __restrict__ dst, uint64_t n_edges,
    uint32_t n, int bits, int symmetrize, int self_loops, int transposed,
    uint64_t* __restrict__ keys, uint32_t* __restrict__ err)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    const uint64_t drop = 1ull << (2 * bits);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_edges; i += stride) {
        uint64_t u = src[i], v = dst[i];
        uint64_t k1, k2;
        if (u >= n || v >= n) {
            atomicOr(err, 1u);
            k1 = k2 = drop;
        } else if (u == v) {
            k1 = k2 = self_loops ? ((u << bits) | u) : drop;
        } else {
            if (transposed) { uint64_t t = u; u = v; v = t; }
            k1 = (u << bits) | v;
            k2 = (v << bits) | u;
        }
        keys[i] = k1;
        if (symmetrize) keys[n_edges + i] = k2;
    }
    if (self_loops) {
        const uint64_t base = (symmetrize ? 2 : 1) * n_edges;
        for (uint64_t u = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; u < n; u += stride)
            keys[base + u] = (u << bits) | u;
    }
}

__device__ inline bool is_first_of_run(const uint64_t* keys, int64_t i, uint64_t drop)
{
    const uint64_t k = keys[i];
    return k < drop && (i == 0 || keys[i - 1] != k);
}

__global__ __launch_bounds__(kBlock) void unique_count_kernel(const uint64_t* __restrict__ keys,
                                                              int64_t n_keys, uint64_t drop,
                                                              uint32_t* __restrict__ tile_cnt)
{
    __shared__ uint64_t lds[4];
    const int64_t base = (int64_t)blockIdx.x * kCompactTile + (int64_t)threadIdx.x * kCompactItems;
    uint64_t c = 0;
#pragma unroll
    for (int j = 0; j < kCompactItems; ++j)
        if (base + j < n_keys && is_first_of_run(keys, base + j, drop)) ++c;
    uint64_t total;
    block_exclusive_scan_u64(c, &total, lds);
    if (threadIdx.x == 0) tile_cnt[blockIdx.x] = (uint32_t)total;
}

__global__ __launch_bounds__(kBlock) void fill_i64_kernel(int64_t* p, int64_t n, int64_t v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// Writes col/cv for every distinct key and rowptr[q] = (index of the first entry with row >= q)
// for every q up to the last non-empty row; later rows keep the preset value nnz.
__global__ __launch_bounds__(kBlock) void unique_fill_kernel(
    const uint64_t* __restrict__ keys, int64_t n_keys, uint64_t drop, int bits,
    const uint64_t* __restrict__ tile_off, uint32_t* __restrict__ col,
    uint2* __restrict__ cv, int64_t* __restrict__ rowptr)
{
    __shared__ uint64_t lds[4];
    const int64_t base = (int64_t)blockIdx.x * kCompactTile + (int64_t)threadIdx.x * kCompactItems;
    bool f[kCompactItems];
    uint64_t c = 0;
#pragma unroll
    for (int j = 0; j < kCompactItems; ++j) {
        f[j] = (base + j < n_keys) && is_first_of_run(keys, base + j, drop);
        c += f[j] ? 1 : 0;
    }
    uint64_t total;
    uint64_t pos = block_exclusive_scan_u64(c, &total, lds) + tile_off[blockIdx.x];
    const uint64_t cmask = (1ull << bits) - 1;
#pragma unroll
    for (int j = 0; j < kCompactItems; ++j) {
        if (!f[j]) continue;
        const int64_t i = base + j;
        const uint64_t k = keys[i];
        const uint32_t c32 = (uint32_t)(k & cmask);
        col[pos] = c32;
        cv[pos] = make_uint2(c32, 0u);
        const int64_t row = (int64_t)(k >> bits);
        const int64_t prev = (i == 0) ? -1 : (int64_t)(keys[i - 1] >> bits);
        for (int64_t q = prev + 1; q <= row; ++q) rowptr[q] = (int64_t)pos;
        ++pos;
    }
}

// Marks the last stored entry of every non-empty row in cv and reports empty rows.
__global__ __launch_bounds__(kBlock) void mark_row_ends_kernel(const int64_t* __restrict__ rowptr,
                                                               uint32_t n, uint2* cv,
                                                               uint32_t* __restrict__ any_empty)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n) return;
    const int64_t a = rowptr[r], b = rowptr[r + 1];
    if (b > a) cv[b - 1].x |= kEntryEndBit;
    else atomicOr(any_empty, 1u);
}

// grp_row[g] = the row that holds stored entry g * kGroupNnz (last row with rowptr <= that).
__global__ __launch_bounds__(kBlock) void group_rows_kernel(const int64_t* __restrict__ rowptr,
                                                            uint32_t n, int64_t nnz,
                                                            int64_t n_groups,
                                                            uint32_t* __restrict__ grp_row)
{
    const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g > n_groups) return;
    const int64_t e = g * kGroupNnz;
    if (e >= nnz) {
        grp_row[g] = n ? n - 1 : 0;
        return;
    }
    // upper_bound(rowptr[0..n], e) - 1
    int64_t lo = 0, hi = (int64_t)n + 1;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (rowptr[mid] <= e) lo = mid + 1;
        else hi = mid;
    }
    grp_row[g] = (uint32_t)(lo - 1);
}

// Row sums of the binary matrix and the scaling vector of the mode: D^-1/2 (symmetric), D^-1
// (mean), unused (sum).
__global__ __launch_bounds__(kBlock) void degree_kernel(const int64_t* __restrict__ rowptr,
                                                        uint32_t n, int mode,
                                                        uint32_t* __restrict__ deg,
                                                        float* __restrict__ dinv)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n) return;
    const uint32_t d = (uint32_t)(rowptr[r + 1] - rowptr[r]);
    deg[r] = d;
    if (mode == MIXGCN_NORM_MEAN) dinv[r] = d ? (float)(1.0 / (double)d) : 0.0f;
    else dinv[r] = d ? (float)(1.0 / sqrt((double)d)) : 0.0f;
}

// One thread per stored entry (r, c) of the CSR at hand, its row found by binary search in
// rowptr.  `swapped`: the CSR holds the transpose of the aggregation matrix, so its entry
// (r, c) carries the value of entry (c, r).
//   symmetric: dinv[r] * dinv[c] - a single fp32 multiply, so val(u,v) == val(v,u) bit for bit;
//   mean:      dinv[row of the aggregation matrix] = 1 / deg;
//   sum:       1, and 1 + eps on the diagonal.
__global__ __launch_bounds__(kBlock) void values_kernel(const int64_t* __restrict__ rowptr,
                                                        const uint32_t* __restrict__ col,
                                                        const float* __restrict__ dinv,
                                                        uint32_t n, int64_t nnz, int mode,
                                                        float eps, int swapped,
                                                        float* __restrict__ val,
                                                        uint2* __restrict__ cv)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= nnz) return;
    int64_t lo = 0, hi = (int64_t)n + 1;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (rowptr[mid] <= e) lo = mid + 1;
        else hi = mid;
    }
    const int64_t row = lo - 1;
    const uint32_t c = col[e];
    float v;
    if (mode == MIXGCN_NORM_MEAN) v = swapped ? dinv[c] : dinv[row];
    else if (mode == MIXGCN_NORM_SUM) v = ((int64_t)c == row) ? 1.0f + eps : 1.0f;
    else v = dinv[row] * dinv[c];
    val[e] = v;
    cv[e].y = __float_as_uint(v);
}

// cv_t = cv with the value words left for values_kernel to fill (same columns and row marks)
__global__ __launch_bounds__(kBlock) void copy_entries_kernel(const uint2* __restrict__ in,
                                                              uint2* __restrict__ out, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) out[i] = in[i];
}

template <typename T>
int dmalloc(T** p, size_t count)
{
    *p = nullptr;
    if (count == 0) count = 1;
    MIXGCN_HIP_TRY(hipMalloc((void**)p, count * sizeof(T)));
    return MIXGCN_OK;
}

struct TmpBufs {
    uint64_t* keys = nullptr;
    uint64_t* alt = nullptr;
    void* tmp = nullptr;
    uint32_t* flags = nullptr;
    ~TmpBufs()
    {
        if (keys) (void)hipFree(keys);
        if (alt) (void)hipFree(alt);
        if (tmp) (void)hipFree(tmp);
        if (flags) (void)hipFree(flags);
    }
};

}  // namespace

void csr_free(Csr* c)
{
    if (c->rowptr) (void)hipFree(c->rowptr);
    if (c->col) (void)hipFree(c->col);
    if (c->cv) (void)hipFree(c->cv);
    if (c->val) (void)hipFree(c->val);
    if (c->cv_t) (void)hipFree(c->cv_t);
    if (c->val_t) (void)hipFree(c->val_t);
    if (c->grp_row) (void)hipFree(c->grp_row);
    *c = Csr();
}

int csr_from_edges(const uint32_t* d_src, const uint32_t* d_dst, uint64_t n_edges, uint32_t n,
                   bool symmetrize, bool self_loops, bool transposed, Csr* out, hipStream_t s)
{
    int bits = 1;
    while ((1ull << bits) < (uint64_t)n) ++bits;
    const uint64_t drop = 1ull << (2 * bits);
    const int sort_bits = 2 * bits + (self_loops ? 0 : 1);  // the drop marker needs one more bit
    const int64_t n_keys = (int64_t)((symmetrize ? 2 : 1) * n_edges + (self_loops ? n : 0));

    TmpBufs t;
    MIXGCN_TRY(dmalloc(&t.keys, (size_t)n_keys));
    MIXGCN_TRY(dmalloc(&t.alt, (size_t)n_keys));
    const int64_t n_ctiles = ceil_div(n_keys > 0 ? n_keys : 1, kCompactTile);
    size_t tmp_bytes = sort_tmp_bytes(n_keys);
    const size_t compact_bytes =
        ((size_t)n_ctiles * 4 + 255) / 256 * 256 + ((size_t)n_ctiles * 8 + 255) / 256 * 256 +
        scan_tmp_bytes(n_ctiles) + 256;
    if (compact_bytes > tmp_bytes) tmp_bytes = compact_bytes;
    MIXGCN_HIP_TRY(hipMalloc(&t.tmp, tmp_bytes));
    MIXGCN_TRY(dmalloc(&t.flags, 4));  // [0] bad endpoint, [1] empty rows, [2..3] total (u64)
    MIXGCN_HIP_TRY(hipMemsetAsync(t.flags, 0, 16, s));

    if (n_keys > 0) {
        const uint64_t work = n_edges > n ? n_edges : n;
        unsigned grid = (unsigned)((work + kBlock - 1) / kBlock);
        if (grid > 65536u) grid = 65536u;
        if (grid == 0) grid = 1;
        hipLaunchKernelGGL(emit_keys_kernel, dim3(grid), dim3(kBlock), 0, s, d_src, d_dst, n_edges,
                           n, bits, symmetrize ? 1 : 0, self_loops ? 1 : 0, transposed ? 1 : 0,
                           t.keys, t.flags);
    }
    uint64_t* sorted = t.keys;
    MIXGCN_TRY(radix_sort_u64(t.keys, t.alt, n_keys, sort_bits, &sorted, t.tmp, s));

    // distinct keys per tile -> tile offsets and nnz
    char* p = (char*)t.tmp;
    uint32_t* tile_cnt = (uint32_t*)p;
    p += ((size_t)n_ctiles * 4 + 255) / 256 * 256;
    uint64_t* tile_off = (uint64_t*)p;
    p += ((size_t)n_ctiles * 8 + 255) / 256 * 256;
    void* scan_tmp = p;
    uint64_t* d_total = (uint64_t*)(t.flags + 2);
    if (n_keys > 0) {
        hipLaunchKernelGGL(unique_count_kernel, dim3((unsigned)n_ctiles), dim3(kBlock), 0, s,
                           sorted, n_keys, drop, tile_cnt);
        MIXGCN_TRY(exclusive_scan_u32_to_u64(tile_cnt, tile_off, n_ctiles, d_total, scan_tmp, s));
    }
    uint32_t h_flags[4];
    MIXGCN_HIP_TRY(hipMemcpyAsync(h_flags, t.flags, 16, hipMemcpyDeviceToHost, s));
    MIXGCN_HIP_TRY(hipStreamSynchronize(s));
    if (h_flags[0]) return fail(MIXGCN_EINVAL, "edge endpoint >= n_nodes");
    const uint64_t nnz64 = (uint64_t)h_flags[2] | ((uint64_t)h_flags[3] << 32);
    const int64_t nnz = (int64_t)nnz64;

    Csr c;
    c.nnz = nnz;
    c.n_groups = ceil_div(nnz, kGroupNnz);
    c.nnz_padded = (c.n_groups + 1) * kGroupNnz + kEntryPad;
    int rc = MIXGCN_OK;
    do {
        if ((rc = dmalloc(&c.rowptr, (size_t)n + 1)) != MIXGCN_OK) break;
        if ((rc = dmalloc(&c.col, (size_t)nnz)) != MIXGCN_OK) break;
        if ((rc = dmalloc(&c.cv, (size_t)c.nnz_padded)) != MIXGCN_OK) break;
        if ((rc = dmalloc(&c.grp_row, (size_t)c.n_groups + 1)) != MIXGCN_OK) break;
        if (hipMemsetAsync(c.cv, 0, (size_t)c.nnz_padded * 8, s) != hipSuccess) {
            rc = fail(MIXGCN_EHIP, "hipMemsetAsync(cv)");
            break;
        }
        hipLaunchKernelGGL(fill_i64_kernel, dim3((unsigned)ceil_div((int64_t)n + 1, kBlock)),
                           dim3(kBlock), 0, s, c.rowptr, (int64_t)n + 1, nnz);
        if (n_keys > 0)
            hipLaunchKernelGGL(unique_fill_kernel, dim3((unsigned)n_ctiles), dim3(kBlock), 0, s,
                               sorted, n_keys, drop, bits, tile_off, c.col, c.cv, c.rowptr);
        if (n > 0)
            hipLaunchKernelGGL(mark_row_ends_kernel, dim3((unsigned)ceil_div(n, kBlock)),
                               dim3(kBlock), 0, s, c.rowptr, n, c.cv, t.flags + 1);
        hipLaunchKernelGGL(group_rows_kernel, dim3((unsigned)ceil_div(c.n_groups + 1, kBlock)),
                           dim3(kBlock), 0, s, c.rowptr, n, nnz, c.n_groups, c.grp_row);
        c.h_rowptr.resize((size_t)n + 1);
        if (hipMemcpyAsync(c.h_rowptr.data(), c.rowptr, ((size_t)n + 1) * 8, hipMemcpyDeviceToHost,
                           s) != hipSuccess ||
            hipMemcpyAsync(h_flags, t.flags, 16, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess || hipGetLastError() != hipSuccess) {
            rc = fail(MIXGCN_EHIP, "CSR fill failed");
            break;
        }
        c.has_empty_rows = h_flags[1] != 0;
    } while (0);
    if (rc != MIXGCN_OK) {
        csr_free(&c);
        return rc;
    }
    *out = std::move(c);
    return MIXGCN_OK;
}

int normalize_graph(mixgcn_graph* g, int mode, float eps, hipStream_t s)
{
    const uint32_t n = g->n;
    if (!g->deg) MIXGCN_TRY(dmalloc(&g->deg, n));
    if (!g->dinv) MIXGCN_TRY(dmalloc(&g->dinv, n));
    if (n > 0)
        hipLaunchKernelGGL(degree_kernel, dim3((unsigned)ceil_div(n, kBlock)), dim3(kBlock), 0, s,
                           g->fwd.rowptr, n, mode, g->deg, g->dinv);
    Csr* mats[2] = {&g->fwd, g->has_transpose ? &g->tr : nullptr};
    for (Csr* c : mats) {
        if (!c) continue;
        if (!c->val) MIXGCN_TRY(dmalloc(&c->val, (size_t)c->nnz));
        if (c->nnz > 0)
            hipLaunchKernelGGL(values_kernel, dim3((unsigned)ceil_div(c->nnz, kBlock)),
                               dim3(kBlock), 0, s, c->rowptr, c->col, g->dinv, n, c->nnz, mode, eps,
                               c == &g->tr ? 1 : 0, c->val, c->cv);
    }
    // A symmetrised graph stores one pattern for the matrix and its transpose.  The mean
    // weights are not symmetric, so the transpose gets value arrays of its own on that pattern.
    Csr& f = g->fwd;
    if (mode == MIXGCN_NORM_MEAN && (g->flags & MIXGCN_SYMMETRIZE)) {
        if (!f.val_t) MIXGCN_TRY(dmalloc(&f.val_t, (size_t)f.nnz));
        if (!f.cv_t) MIXGCN_TRY(dmalloc(&f.cv_t, (size_t)f.nnz_padded));
        hipLaunchKernelGGL(copy_entries_kernel, dim3((unsigned)ceil_div(f.nnz_padded, kBlock)),
                           dim3(kBlock), 0, s, f.cv, f.cv_t, f.nnz_padded);
        if (f.nnz > 0)
            hipLaunchKernelGGL(values_kernel, dim3((unsigned)ceil_div(f.nnz, kBlock)), dim3(kBlock), 0,
                               s, f.rowptr, f.col, g->dinv, n, f.nnz, mode, eps, 1, f.val_t, f.cv_t);
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    g->normalized = true;
    g->norm_mode = mode;
    return MIXGCN_OK;
}

}  // namespace mixgcn
