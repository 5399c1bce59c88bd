// Node reordering (paper Sec. 3.2.2): reverse Cuthill-McKee positions of a graph's nodes, the
// graph bandwidth b = max |p_u - p_v| under a processing sequence, the batch count of
// Proposition 3.5, and the kernels that apply a sequence (relabel an edge list, permute rows).
//
// Cuthill-McKee is written level by level so that every step is a parallel pass.  The serial
// rule - visit in queue order; the unvisited neighbors of the visited node join the queue in
// increasing (degree, id) - puts the nodes of one breadth-first level in the order of
// (queue index of the earliest visited neighbor, degree, id).  So per level: every frontier
// node offers its queue index to its unvisited neighbors with an atomic minimum, the first
// offer also appends the neighbor to the next level's list, and that list is sorted by
// (winning index, rank of the node in the global (degree, id) order).  Components start from
// the unvisited node of smallest (degree, id); runs of single-node components are appended in
// one pass.  The host reads one counter per level, so the time grows with the number of levels.
#include <vector>

#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr uint32_t kNone = 0xFFFFFFFFu;

struct DevMem {
    std::vector<void*> ptrs;
    ~DevMem()
    {
        for (void* p : ptrs) (void)hipFree(p);
    }
    template <typename T>
    int alloc(T** out, size_t count)
    {
        *out = nullptr;
        void* p = nullptr;
        MIXGCN_HIP_TRY(hipMalloc(&p, (count ? count : 1) * sizeof(T)));
        ptrs.push_back(p);
        *out = (T*)p;
        return MIXGCN_OK;
    }
};

__global__ __launch_bounds__(kBlock) void degree_keys_kernel(const int64_t* __restrict__ rowptr,
                                                             uint32_t n, uint64_t* __restrict__ keys)
{
    const uint32_t v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= n) return;
    keys[v] = ((uint64_t)(rowptr[v + 1] - rowptr[v]) << 32) | v;
}

// bydeg[i] = i-th node in (degree, id) order; degrank = its inverse; single[v] = the row of v
// holds no node but v itself
__global__ __launch_bounds__(kBlock) void rank_kernel(const uint64_t* __restrict__ sorted,
                                                      const int64_t* __restrict__ rowptr,
                                                      const uint32_t* __restrict__ col, uint32_t n,
                                                      uint32_t* __restrict__ bydeg,
                                                      uint32_t* __restrict__ degrank,
                                                      uint32_t* __restrict__ single,
                                                      uint32_t* __restrict__ cm_idx,
                                                      uint32_t* __restrict__ parent)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t v = (uint32_t)sorted[i];
    bydeg[i] = v;
    degrank[v] = i;
    const int64_t a = rowptr[v], b = rowptr[v + 1];
    single[v] = (b == a || (b == a + 1 && col[a] == v)) ? 1u : 0u;
    cm_idx[i] = kNone;
    parent[i] = kNone;
}

// result = smallest position i >= cursor in bydeg whose node is unvisited and not single
__global__ __launch_bounds__(kBlock) void next_root_kernel(const uint32_t* __restrict__ bydeg,
                                                           const uint32_t* __restrict__ cm_idx,
                                                           const uint32_t* __restrict__ single,
                                                           uint32_t cursor, uint32_t n,
                                                           uint32_t* __restrict__ result)
{
    const uint32_t stride = gridDim.x * blockDim.x;
    uint32_t best = kNone;
    for (uint32_t i = cursor + blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint32_t v = bydeg[i];
        if (cm_idx[v] == kNone && !single[v]) {
            best = i;
            break;  // positions grow along this thread's walk
        }
    }
    if (best != kNone) atomicMin(result, best);
}

// flags[i] = node bydeg[cursor + i] is unvisited (it is then a single-node component)
__global__ __launch_bounds__(kBlock) void single_flags_kernel(const uint32_t* __restrict__ bydeg,
                                                              const uint32_t* __restrict__ cm_idx,
                                                              uint32_t cursor, uint32_t count,
                                                              uint32_t* __restrict__ flags)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    flags[i] = cm_idx[bydeg[cursor + i]] == kNone ? 1u : 0u;
}

__global__ __launch_bounds__(kBlock) void single_append_kernel(
    const uint32_t* __restrict__ bydeg, const uint32_t* __restrict__ flags,
    const uint64_t* __restrict__ offs, uint32_t cursor, uint32_t count, uint32_t base,
    uint32_t* __restrict__ cm_idx, uint32_t* __restrict__ order)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count || !flags[i]) return;
    const uint32_t v = bydeg[cursor + i];
    const uint32_t at = base + (uint32_t)offs[i];
    cm_idx[v] = at;
    order[at] = v;
}

__global__ void start_component_kernel(const uint32_t* __restrict__ bydeg, uint32_t pos_in_bydeg,
                                       uint32_t base, uint32_t* __restrict__ cm_idx,
                                       uint32_t* __restrict__ order)
{
    const uint32_t v = bydeg[pos_in_bydeg];
    cm_idx[v] = base;
    order[base] = v;
}

// One wavefront per frontier node order[f_begin + i]: offers its queue index to every unvisited
// neighbor; the first offer a node receives also puts it on the next level's list.
__global__ __launch_bounds__(kBlock) void expand_kernel(
    const int64_t* __restrict__ rowptr, const uint32_t* __restrict__ col,
    const uint32_t* __restrict__ order, uint32_t f_begin, uint32_t f_count,
    const uint32_t* __restrict__ cm_idx, uint32_t* __restrict__ parent,
    uint32_t* __restrict__ next_list, uint32_t* __restrict__ next_count)
{
    const uint32_t i = blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    if (i >= f_count) return;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t qi = f_begin + i;
    const uint32_t u = order[qi];
    for (int64_t e = rowptr[u] + lane; e < rowptr[u + 1]; e += kWave) {
        const uint32_t w = col[e];
        if (cm_idx[w] != kNone) continue;
        const uint32_t old = atomicMin(&parent[w], qi);
        if (old == kNone) next_list[atomicAdd(next_count, 1u)] = w;
    }
}

__global__ __launch_bounds__(kBlock) void level_keys_kernel(const uint32_t* __restrict__ next_list,
                                                            uint32_t m,
                                                            const uint32_t* __restrict__ parent,
                                                            const uint32_t* __restrict__ degrank,
                                                            uint64_t* __restrict__ keys)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= m) return;
    const uint32_t w = next_list[i];
    keys[i] = ((uint64_t)parent[w] << 32) | degrank[w];
}

__global__ __launch_bounds__(kBlock) void level_assign_kernel(const uint64_t* __restrict__ sorted,
                                                              uint32_t m,
                                                              const uint32_t* __restrict__ bydeg,
                                                              uint32_t base,
                                                              uint32_t* __restrict__ cm_idx,
                                                              uint32_t* __restrict__ order)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= m) return;
    const uint32_t w = bydeg[(uint32_t)sorted[i]];
    cm_idx[w] = base + i;
    order[base + i] = w;
}

__global__ __launch_bounds__(kBlock) void reverse_kernel(const uint32_t* __restrict__ order,
                                                         uint32_t n, uint32_t* __restrict__ pos)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) pos[order[i]] = n - 1 - i;
}

// One wavefront per row: max over its entries of |p_row - p_col|
__global__ __launch_bounds__(kBlock) void bandwidth_kernel(const int64_t* __restrict__ rowptr,
                                                           const uint32_t* __restrict__ col,
                                                           const uint32_t* __restrict__ pos,
                                                           uint32_t n, uint32_t* __restrict__ result)
{
    const uint32_t u = blockIdx.x * (kBlock / kWave) + (threadIdx.x >> 6);
    if (u >= n) return;
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t pu = pos ? pos[u] : u;
    uint32_t best = 0;
    for (int64_t e = rowptr[u] + lane; e < rowptr[u + 1]; e += kWave) {
        const uint32_t pv = pos ? pos[col[e]] : col[e];
        const uint32_t d = pu > pv ? pu - pv : pv - pu;
        best = d > best ? d : best;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t other = (uint32_t)__shfl_xor((int)best, o, kWave);
        best = other > best ? other : best;
    }
    if (lane == 0 && best > 0) atomicMax(result, best);
}

__global__ __launch_bounds__(kBlock) void relabel_kernel(const uint32_t* __restrict__ src,
                                                         const uint32_t* __restrict__ dst,
                                                         uint64_t n_edges,
                                                         const uint32_t* __restrict__ pos,
                                                         uint32_t n, uint32_t* __restrict__ src_out,
                                                         uint32_t* __restrict__ dst_out,
                                                         uint32_t* __restrict__ bad)
{
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_edges) return;
    const uint32_t a = src[i], b = dst[i];
    if (a >= n || b >= n) {
        atomicOr(bad, 1u);
        return;
    }
    src_out[i] = pos[a];
    dst_out[i] = pos[b];
}

// Y[pos[v], :] = X[v, :], 16 bytes per lane
__global__ __launch_bounds__(kBlock) void permute_rows_kernel(const uint4* __restrict__ X,
                                                              int64_t ldx16, uint4* __restrict__ Y,
                                                              int64_t ldy16, int64_t n, int vecs,
                                                              const uint32_t* __restrict__ pos)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * vecs) return;
    const int64_t v = i / vecs;
    const int c = (int)(i % vecs);
    Y[(int64_t)pos[v] * ldy16 + c] = X[v * ldx16 + c];
}

inline unsigned blocks_for(uint64_t items) { return (unsigned)ceil_div((int64_t)items, kBlock); }

int read_u32(const uint32_t* d, uint32_t* h, hipStream_t s)
{
    MIXGCN_HIP_TRY(hipMemcpyAsync(h, d, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
    MIXGCN_HIP_TRY(hipStreamSynchronize(s));
    return MIXGCN_OK;
}

int bits_for(uint64_t max_value)
{
    int b = 1;
    while (b < 64 && (max_value >> b) != 0) ++b;
    return b;
}

}  // namespace
}  // namespace mixgcn

using namespace mixgcn;

extern "C" {

int mixgcn_reorder_rcm(const mixgcn_graph* g, uint32_t* pos, void* stream)
{
    if (!g || !pos) return fail(MIXGCN_EINVAL, "reorder_rcm: null argument");
    hipStream_t s = (hipStream_t)stream;
    const uint32_t n = g->n;
    if (n == 0) return MIXGCN_OK;
    const Csr& m = g->fwd;
    DevMem mem;
    uint64_t *keys, *alt, *offs;
    uint32_t *bydeg, *degrank, *single, *cm_idx, *parent, *order, *next_list, *flags, *counters;
    void* tmp;
    MIXGCN_TRY(mem.alloc(&keys, n));
    MIXGCN_TRY(mem.alloc(&alt, n));
    MIXGCN_TRY(mem.alloc(&offs, n));
    MIXGCN_TRY(mem.alloc(&bydeg, n));
    MIXGCN_TRY(mem.alloc(&degrank, n));
    MIXGCN_TRY(mem.alloc(&single, n));
    MIXGCN_TRY(mem.alloc(&cm_idx, n));
    MIXGCN_TRY(mem.alloc(&parent, n));
    MIXGCN_TRY(mem.alloc(&order, n));
    MIXGCN_TRY(mem.alloc(&next_list, n));
    MIXGCN_TRY(mem.alloc(&flags, n));
    MIXGCN_TRY(mem.alloc(&counters, 2));  // [0] next-level count, [1] next root position
    const size_t tmp_bytes = sort_tmp_bytes(n) > scan_tmp_bytes(n) ? sort_tmp_bytes(n) : scan_tmp_bytes(n);
    {
        char* t;
        MIXGCN_TRY(mem.alloc(&t, tmp_bytes));
        tmp = t;
    }

    // global (degree, id) order
    hipLaunchKernelGGL(degree_keys_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s, m.rowptr, n, keys);
    uint64_t* sorted = nullptr;
    const uint64_t max_deg_key = ((uint64_t)(m.nnz > 0 ? m.nnz : 1) << 32) | 0xFFFFFFFFull;
    MIXGCN_TRY(radix_sort_u64(keys, alt, n, bits_for(max_deg_key), &sorted, tmp, s));
    hipLaunchKernelGGL(rank_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s, sorted, m.rowptr, m.col,
                       n, bydeg, degrank, single, cm_idx, parent);

    uint32_t count = 0;   // nodes placed so far
    uint32_t cursor = 0;  // position in bydeg from which the next root is searched
    while (count < n) {
        // next root that has neighbors; every unvisited node before it is a single-node component
        const uint32_t none = kNone;
        MIXGCN_HIP_TRY(hipMemcpyAsync(counters + 1, &none, 4, hipMemcpyHostToDevice, s));
        hipLaunchKernelGGL(next_root_kernel, dim3(1024), dim3(kBlock), 0, s, bydeg, cm_idx, single,
                           cursor, n, counters + 1);
        uint32_t root_at = kNone;
        MIXGCN_TRY(read_u32(counters + 1, &root_at, s));
        const uint32_t run_end = root_at == kNone ? n : root_at;
        if (run_end > cursor) {
            const uint32_t cnt = run_end - cursor;
            hipLaunchKernelGGL(single_flags_kernel, dim3(blocks_for(cnt)), dim3(kBlock), 0, s, bydeg,
                               cm_idx, cursor, cnt, flags);
            uint64_t* total = keys;  // free at this point
            MIXGCN_TRY(exclusive_scan_u32_to_u64(flags, offs, cnt, total, tmp, s));
            hipLaunchKernelGGL(single_append_kernel, dim3(blocks_for(cnt)), dim3(kBlock), 0, s, bydeg,
                               flags, offs, cursor, cnt, count, cm_idx, order);
            uint64_t added = 0;
            MIXGCN_HIP_TRY(hipMemcpyAsync(&added, total, 8, hipMemcpyDeviceToHost, s));
            MIXGCN_HIP_TRY(hipStreamSynchronize(s));
            count += (uint32_t)added;
        }
        if (root_at == kNone) break;
        cursor = root_at + 1;

        // breadth-first levels of the component of bydeg[root_at]
        hipLaunchKernelGGL(start_component_kernel, dim3(1), dim3(1), 0, s, bydeg, root_at, count,
                           cm_idx, order);
        uint32_t f_begin = count, f_count = 1;
        count += 1;
        while (f_count > 0) {
            MIXGCN_HIP_TRY(hipMemsetAsync(counters, 0, 4, s));
            hipLaunchKernelGGL(expand_kernel, dim3((unsigned)ceil_div(f_count, kBlock / kWave)),
                               dim3(kBlock), 0, s, m.rowptr, m.col, order, f_begin, f_count, cm_idx,
                               parent, next_list, counters);
            uint32_t mcount = 0;
            MIXGCN_TRY(read_u32(counters, &mcount, s));
            if (mcount == 0) break;
            hipLaunchKernelGGL(level_keys_kernel, dim3(blocks_for(mcount)), dim3(kBlock), 0, s,
                               next_list, mcount, parent, degrank, keys);
            const uint64_t max_key = ((uint64_t)(count - 1) << 32) | (uint64_t)(n - 1);
            // the low word only needs the bits of n - 1, the high word those of count - 1, but
            // the sort works on a contiguous bit range: [0, 32 + bits(count - 1))
            MIXGCN_TRY(radix_sort_u64(keys, alt, mcount, bits_for(max_key), &sorted, tmp, s));
            hipLaunchKernelGGL(level_assign_kernel, dim3(blocks_for(mcount)), dim3(kBlock), 0, s,
                               sorted, mcount, bydeg, count, cm_idx, order);
            f_begin = count;
            f_count = mcount;
            count += mcount;
        }
    }
    hipLaunchKernelGGL(reverse_kernel, dim3(blocks_for(n)), dim3(kBlock), 0, s, order, n, pos);
    MIXGCN_HIP_TRY(hipGetLastError());
    MIXGCN_HIP_TRY(hipStreamSynchronize(s));  // the work arrays are freed on return
    return MIXGCN_OK;
}

int mixgcn_bandwidth(const mixgcn_graph* g, const uint32_t* pos, int64_t* bandwidth, void* stream)
{
    if (!g || !bandwidth) return fail(MIXGCN_EINVAL, "bandwidth: null argument");
    hipStream_t s = (hipStream_t)stream;
    *bandwidth = 0;
    if (g->n == 0) return MIXGCN_OK;
    void* scratch = nullptr;
    MIXGCN_TRY(get_scratch(3, 256, &scratch));
    uint32_t* result = (uint32_t*)scratch;
    MIXGCN_HIP_TRY(hipMemsetAsync(result, 0, 4, s));
    hipLaunchKernelGGL(bandwidth_kernel, dim3((unsigned)ceil_div((int64_t)g->n, kBlock / kWave)),
                       dim3(kBlock), 0, s, g->fwd.rowptr, g->fwd.col, pos, g->n, result);
    uint32_t h = 0;
    MIXGCN_TRY(read_u32(result, &h, s));
    *bandwidth = (int64_t)h;
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

int64_t mixgcn_pipeline_stages(int64_t n_nodes, int64_t bandwidth)
{
    if (n_nodes <= 0 || bandwidth < 0 || bandwidth >= n_nodes) return 0;
    return (2 * n_nodes + (n_nodes - bandwidth) - 1) / (n_nodes - bandwidth);
}

int mixgcn_relabel_edges(const uint32_t* src, const uint32_t* dst, uint64_t n_edges,
                         const uint32_t* pos, uint32_t n_nodes, uint32_t* src_out,
                         uint32_t* dst_out, void* stream)
{
    if (n_edges == 0) return MIXGCN_OK;
    if (!src || !dst || !pos || !src_out || !dst_out)
        return fail(MIXGCN_EINVAL, "relabel_edges: null argument");
    hipStream_t s = (hipStream_t)stream;
    void* scratch = nullptr;
    MIXGCN_TRY(get_scratch(3, 256, &scratch));
    uint32_t* bad = (uint32_t*)scratch;
    MIXGCN_HIP_TRY(hipMemsetAsync(bad, 0, 4, s));
    hipLaunchKernelGGL(relabel_kernel, dim3(blocks_for(n_edges)), dim3(kBlock), 0, s, src, dst,
                       n_edges, pos, n_nodes, src_out, dst_out, bad);
    uint32_t h = 0;
    MIXGCN_TRY(read_u32(bad, &h, s));
    if (h) return fail(MIXGCN_EINVAL, "relabel_edges: an endpoint is >= n_nodes");
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

int mixgcn_permute_rows(int dtype, const void* X, int64_t ldx, void* Y, int64_t ldy, int64_t n_rows,
                        int32_t n_cols, const uint32_t* pos, void* stream)
{
    if (dtype != MIXGCN_F32 && dtype != MIXGCN_BF16) return fail(MIXGCN_EINVAL, "permute_rows: dtype");
    if (n_rows < 0 || n_cols <= 0) return fail(MIXGCN_EINVAL, "permute_rows: sizes");
    if (!X || !Y || !pos) return fail(MIXGCN_EINVAL, "permute_rows: null argument");
    const int es = dtype == MIXGCN_F32 ? 4 : 2;
    if (((uintptr_t)X | (uintptr_t)Y) % 16 != 0 || (ldx * es) % 16 != 0 || (ldy * es) % 16 != 0 ||
        ldx < n_cols || ldy < n_cols)
        return fail(MIXGCN_EINVAL, "permute_rows: matrices must be 16-byte aligned with ld >= columns");
    if (n_rows == 0) return MIXGCN_OK;
    const int vecs = (n_cols * es + 15) / 16;  // the last vector may reach into the row padding
    hipLaunchKernelGGL(permute_rows_kernel, dim3(blocks_for((uint64_t)n_rows * vecs)), dim3(kBlock), 0,
                       (hipStream_t)stream, (const uint4*)X, ldx * es / 16, (uint4*)Y, ldy * es / 16,
                       n_rows, vecs, pos);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // extern "C"
