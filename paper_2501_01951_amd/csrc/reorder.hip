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
// one pass.  Wide levels run as grid-wide kernels with one counter read back per level; levels
// whose frontier is small (at most kNarrowFrontier nodes with kNarrowEdges stored entries) are
// walked by ONE workgroup that stays on the device from level to level, and from component to
// component, until it meets a level too wide for it - a banded graph with tens of thousands of
// levels costs a few microseconds per level instead of a launch and a host round trip.
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

// ---- narrow levels: one resident workgroup --------------------------------------------------
constexpr int kNarrowFrontier = 1024;  // frontier nodes the workgroup takes on
constexpr int kNarrowEdges = 4096;     // stored entries of such a frontier (bounds the next level)

// Progress shared between the host loop and the resident workgroup.
struct RcmState {
    uint32_t count;    // nodes placed so far
    uint32_t cursor;   // position in bydeg from which the next root is searched
    uint32_t f_begin;  // the current frontier is order[f_begin, f_begin + f_count)
    uint32_t f_count;  // 0: no component is open
    uint32_t done;     // every node is placed
    uint32_t levels;   // levels walked on the device (statistics)
};

__device__ inline uint32_t load_coherent(const uint32_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void store_coherent(uint32_t* p, uint32_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Exclusive prefix sum of one value per thread over the 256 threads of the block; *total gets
// the block sum.  lds: 4 words.  Two barriers.
__device__ inline uint32_t block_scan_u32(uint32_t v, uint32_t* total, uint32_t* lds)
{
    const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const uint32_t t = (uint32_t)__shfl_up((int)inc, o, kWave);
        if (lane >= o) inc += t;
    }
    if (lane == kWave - 1) lds[w] = inc;
    __syncthreads();
    uint32_t woff = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < kBlock / kWave; ++i) {
        const uint32_t x = lds[i];
        if (i < w) woff += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return woff + inc - v;
}

// Walks breadth-first levels, and the search for the next component's root (with the runs of
// single-node components before it), for as long as the frontier stays narrow.  Same rule and
// same keys as the grid-wide kernels below, so the sequence does not depend on which path a
// level takes.  Invariant used here: a placed node has parent != kNone (roots and single-node
// components carry their own queue index), so one atomic minimum per stored entry both tests
// "unvisited" and makes the offer - a placed node's parent is smaller than any current queue
// index and stays as it is.  Launched with one workgroup; leaves when every node is placed or
// the next level is too wide (st->f_count then names that frontier).
__global__ __launch_bounds__(kBlock) void narrow_levels_kernel(
    const int64_t* __restrict__ rowptr, const uint32_t* __restrict__ col,
    const uint32_t* __restrict__ bydeg, const uint32_t* __restrict__ degrank,
    const uint32_t* __restrict__ single, uint32_t* __restrict__ cm_idx,
    uint32_t* __restrict__ parent, uint32_t* __restrict__ order, uint32_t n, RcmState* st)
{
    __shared__ uint64_t keys[kNarrowEdges];
    __shared__ uint32_t vals[kNarrowEdges];
    __shared__ uint32_t nextl[kNarrowEdges];
    __shared__ uint32_t f_node[kNarrowFrontier];
    __shared__ uint32_t f_pre[kNarrowFrontier + 1];  // entries before frontier node i
    __shared__ int64_t f_row[kNarrowFrontier];       // rowptr of frontier node i
    __shared__ uint32_t s_scan[4];
    __shared__ uint32_t s_cnt, s_min;
    const uint32_t tid = threadIdx.x;
    uint32_t count = st->count, cursor = st->cursor, f_begin = st->f_begin, f_count = st->f_count;
    uint32_t levels = 0, done = 0;
    bool have = false;  // f_node holds the current frontier
    for (;;) {
        if (f_count == 0) {
            // next root: the unvisited node of smallest (degree, id) that has neighbors; every
            // unvisited node passed on the way is a single-node component and is placed in order
            bool found = false;
            while (!found) {
                if (cursor >= n || count >= n) {
                    done = 1;
                    break;
                }
                if (tid == 0) s_min = kBlock;
                __syncthreads();
                const uint32_t i = cursor + tid;
                uint32_t v = 0;
                bool fresh = false;
                if (i < n) {
                    v = bydeg[i];
                    fresh = load_coherent(&cm_idx[v]) == kNone;
                }
                const bool is_root = fresh && !single[v];
                if (is_root) atomicMin(&s_min, tid);
                __syncthreads();
                const uint32_t r = s_min;
                const uint32_t flag = (fresh && !is_root && tid < r) ? 1u : 0u;
                uint32_t total = 0;
                const uint32_t off = block_scan_u32(flag, &total, s_scan);
                if (flag) {
                    store_coherent(&cm_idx[v], count + off);
                    store_coherent(&parent[v], count + off);
                    order[count + off] = v;
                }
                count += total;
                if (r < (uint32_t)kBlock) {
                    if (tid == r) {
                        store_coherent(&cm_idx[v], count);
                        store_coherent(&parent[v], count);
                        order[count] = v;
                        f_node[0] = v;
                    }
                    f_begin = count;
                    f_count = 1;
                    count += 1;
                    cursor += r + 1;
                    have = true;
                    found = true;
                } else {
                    cursor += kBlock;
                }
                __syncthreads();
            }
            if (done) break;
        }
        if (f_count > (uint32_t)kNarrowFrontier) break;
        if (!have) {
            for (uint32_t i = tid; i < f_count; i += kBlock) f_node[i] = order[f_begin + i];
            __syncthreads();
        }
        // stored entries of the frontier, and where each node's entries start among them
        uint32_t run = 0;  // entries of the frontier nodes before this thread's first one
        {
            constexpr int PER = kNarrowFrontier / kBlock;
            uint32_t d[PER], mine = 0;
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const uint32_t i = tid * PER + q;
                d[q] = 0;
                if (i < f_count) {
                    const uint32_t u = f_node[i];
                    const int64_t a = rowptr[u], b = rowptr[u + 1];
                    f_row[i] = a;
                    // a degree beyond the cap is enough to know that the level is too wide
                    d[q] = (b - a) > (int64_t)kNarrowEdges ? (uint32_t)kNarrowEdges + 1u : (uint32_t)(b - a);
                }
                mine += d[q];
            }
            uint32_t total = 0;
            run = block_scan_u32(mine, &total, s_scan);
            if (total > (uint32_t)kNarrowEdges) {
                have = false;
                break;  // too many entries for one workgroup: the grid-wide kernels take the level
            }
#pragma unroll
            for (int q = 0; q < PER; ++q) {
                const uint32_t i = tid * PER + q;
                if (i < f_count) f_pre[i] = run;
                run += d[q];
            }
            if (tid == 0) {
                f_pre[f_count] = total;
                s_cnt = 0;
            }
            __syncthreads();
            // every stored entry offers its row's queue index to its column
            for (uint32_t t = tid; t < total; t += kBlock) {
                uint32_t lo = 0, hi = f_count;  // node i with f_pre[i] <= t < f_pre[i + 1]
                while (hi - lo > 1) {
                    const uint32_t mid = (lo + hi) >> 1;
                    if (f_pre[mid] <= t) lo = mid;
                    else hi = mid;
                }
                const uint32_t w = col[f_row[lo] + (int64_t)(t - f_pre[lo])];
                const uint32_t old = atomicMin(&parent[w], f_begin + lo);
                if (old == kNone) nextl[atomicAdd(&s_cnt, 1u)] = w;
            }
            __syncthreads();
        }
        ++levels;
        const uint32_t m = s_cnt;
        if (m == 0) {  // the component is complete
            f_count = 0;
            have = false;
            __syncthreads();
            continue;
        }
        // order the next level by (smallest queue index that offered, rank in (degree, id))
        if (m <= (uint32_t)kBlock) {
            uint64_t key = 0;
            uint32_t w = 0;
            if (tid < m) {
                w = nextl[tid];
                key = ((uint64_t)load_coherent(&parent[w]) << 32) | degrank[w];
                keys[tid] = key;
            }
            __syncthreads();
            if (tid < m) {
                uint32_t rank = 0;
                for (uint32_t j = 0; j < m; ++j) rank += keys[j] < key ? 1u : 0u;
                vals[rank] = w;
            }
            __syncthreads();
        } else {
            uint32_t P = 512;
            while (P < m) P <<= 1;
            for (uint32_t i = tid; i < P; i += kBlock) {
                uint64_t key = ~0ull;
                uint32_t w = 0;
                if (i < m) {
                    w = nextl[i];
                    key = ((uint64_t)load_coherent(&parent[w]) << 32) | degrank[w];
                }
                keys[i] = key;
                vals[i] = w;
            }
            __syncthreads();
            for (uint32_t k = 2; k <= P; k <<= 1)
                for (uint32_t j = k >> 1; j > 0; j >>= 1) {
                    for (uint32_t t = tid; t < P / 2; t += kBlock) {
                        const uint32_t a = (t / j) * 2 * j + (t % j), b = a + j;
                        const bool up = (a & k) == 0;
                        const uint64_t ka = keys[a], kb = keys[b];
                        if ((ka > kb) == up) {
                            keys[a] = kb;
                            keys[b] = ka;
                            const uint32_t va = vals[a];
                            vals[a] = vals[b];
                            vals[b] = va;
                        }
                    }
                    __syncthreads();
                }
        }
        for (uint32_t i = tid; i < m; i += kBlock) {
            const uint32_t w = vals[i];
            store_coherent(&cm_idx[w], count + i);
            order[count + i] = w;
            if (i < (uint32_t)kNarrowFrontier) f_node[i] = w;
        }
        f_begin = count;
        f_count = m;
        count += m;
        have = m <= (uint32_t)kNarrowFrontier;
        __syncthreads();
    }
    __threadfence();
    if (tid == 0) {
        st->count = count;
        st->cursor = cursor;
        st->f_begin = f_begin;
        st->f_count = f_count;
        st->done = done;
        st->levels += levels;
    }
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
    uint64_t *keys, *alt;
    uint32_t *bydeg, *degrank, *single, *cm_idx, *parent, *order, *next_list, *counters;
    void* tmp;
    MIXGCN_TRY(mem.alloc(&keys, n));
    MIXGCN_TRY(mem.alloc(&alt, n));
    MIXGCN_TRY(mem.alloc(&bydeg, n));
    MIXGCN_TRY(mem.alloc(&degrank, n));
    MIXGCN_TRY(mem.alloc(&single, n));
    MIXGCN_TRY(mem.alloc(&cm_idx, n));
    MIXGCN_TRY(mem.alloc(&parent, n));
    MIXGCN_TRY(mem.alloc(&order, n));
    MIXGCN_TRY(mem.alloc(&next_list, n));
    MIXGCN_TRY(mem.alloc(&counters, 2));  // [0] next-level count
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

    // The resident workgroup walks narrow levels and finds roots until it meets a level too
    // wide for it; the host then runs that one level with the grid-wide kernels and hands back.
    RcmState* d_state;
    MIXGCN_TRY(mem.alloc(&d_state, 1));
    RcmState st = {};
    MIXGCN_HIP_TRY(hipMemcpyAsync(d_state, &st, sizeof(st), hipMemcpyHostToDevice, s));
    for (;;) {
        hipLaunchKernelGGL(narrow_levels_kernel, dim3(1), dim3(kBlock), 0, s, m.rowptr, m.col, bydeg,
                           degrank, single, cm_idx, parent, order, n, d_state);
        MIXGCN_HIP_TRY(hipMemcpyAsync(&st, d_state, sizeof(st), hipMemcpyDeviceToHost, s));
        MIXGCN_HIP_TRY(hipStreamSynchronize(s));
        if (st.done) break;
        if (st.f_count == 0 || st.count >= n + 1)
            return fail(MIXGCN_EHIP, "reorder_rcm: the level walk stopped without a frontier");
        // wide levels, until the frontier is narrow again or the component ends
        uint32_t count = st.count, f_begin = st.f_begin, f_count = st.f_count;
        bool first = true;  // the level the workgroup refused is run here whatever its node count
        while (f_count > 0 && (first || f_count > (uint32_t)kNarrowFrontier)) {
            first = false;
            MIXGCN_HIP_TRY(hipMemsetAsync(counters, 0, 4, s));
            hipLaunchKernelGGL(expand_kernel, dim3((unsigned)ceil_div(f_count, kBlock / kWave)),
                               dim3(kBlock), 0, s, m.rowptr, m.col, order, f_begin, f_count, cm_idx,
                               parent, next_list, counters);
            uint32_t mcount = 0;
            MIXGCN_TRY(read_u32(counters, &mcount, s));
            if (mcount == 0) {
                f_count = 0;
                break;
            }
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
        st.count = count;
        st.f_begin = f_begin;
        st.f_count = f_count;
        MIXGCN_HIP_TRY(hipMemcpyAsync(d_state, &st, sizeof(st), hipMemcpyHostToDevice, s));
    }
    if (st.count != n) return fail(MIXGCN_EHIP, "reorder_rcm: not every node was placed");
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
