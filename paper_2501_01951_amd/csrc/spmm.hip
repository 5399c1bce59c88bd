// Neighbor aggregation  Z[r, c0:c1) = sum_e val[e] * H[col[e], c0:c1)  (paper Algorithm 2,
// aggregation phase) as a gather kernel balanced by stored entries rather than by rows.
//
// Work split.  The stored entries of the CSR are cut into consecutive windows of kGroupNnz
// entries.  A "lane group" of G lanes (G * VEC = padded slice width; a 64-wide wavefront holds
// 64 / G groups) walks one window front to back: every lane keeps VEC accumulators of one
// output row, each entry costs one 16-byte load per lane from the neighbor's feature row
// (a full row per group, coalesced), and the end-of-row mark stored in bit 31 of the column
// index tells the group when to write the row out.  Hubs of a power-law graph are therefore
// spread over many groups and low-degree rows share a group; every group does the same amount
// of gather work whatever the degree distribution.
//
// Rows that cross a window boundary are finished by a second, tiny kernel: a group stores the
// piece that completes a row begun in an earlier window in its "head" slot and the piece of a
// row it cannot complete in its "tail" slot; the fix-up kernel adds the pieces of each such row
// in window order.  The result is deterministic (no atomics).
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kL = kGroupNnz;
constexpr uint32_t kEndBit = 0x80000000u;

// 16-byte feature load: 4 fp32 or 8 bf16 (widened to fp32)
template <int DT>
struct Feat;

template <>
struct Feat<MIXGCN_F32> {
    static constexpr int VEC = 4;
    using Raw = float4;
    __device__ static inline void widen(const Raw& r, float* o)
    {
        o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w;
    }
    __device__ static inline void store(void* base, int64_t elem_off, const float* a)
    {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(base) + elem_off) =
            make_float4(a[0], a[1], a[2], a[3]);
    }
    __device__ static inline const Raw* ptr(const void* base, int64_t elem_off)
    {
        return reinterpret_cast<const Raw*>(reinterpret_cast<const float*>(base) + elem_off);
    }
};

__device__ inline uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

template <>
struct Feat<MIXGCN_BF16> {
    static constexpr int VEC = 8;
    using Raw = uint4;
    __device__ static inline void widen(const Raw& r, float* o)
    {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            o[2 * i] = __uint_as_float(w[i] << 16);
            o[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static inline void store(void* base, int64_t elem_off, const float* a)
    {
        uint4 r;
        r.x = f32_to_bf16_rne(a[0]) | (f32_to_bf16_rne(a[1]) << 16);
        r.y = f32_to_bf16_rne(a[2]) | (f32_to_bf16_rne(a[3]) << 16);
        r.z = f32_to_bf16_rne(a[4]) | (f32_to_bf16_rne(a[5]) << 16);
        r.w = f32_to_bf16_rne(a[6]) | (f32_to_bf16_rne(a[7]) << 16);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(base) + elem_off) = r;
    }
    __device__ static inline const Raw* ptr(const void* base, int64_t elem_off)
    {
        return reinterpret_cast<const Raw*>(reinterpret_cast<const uint16_t*>(base) + elem_off);
    }
};

__device__ inline uint32_t comp(const uint4& v, int i)
{
    return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}
__device__ inline float comp(const float4& v, int i)
{
    return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

// State of one lane group while it walks its window.
template <int VEC>
struct GroupState {
    float acc[VEC];
    int64_t r;      // row being accumulated
    bool head;      // the next completed piece belongs to a row begun in an earlier window
    bool pending;   // acc holds entries of a row whose end has not been seen
};

// Eight consecutive entries [e, e + 8) of one staged chunk: broadcast index and value from the
// lanes that staged them, issue the eight feature loads back to back, then accumulate and
// write rows out at the end-of-row marks.  All loads are in bounds by construction (padding
// entries carry column 0 and value 0), so only the accumulation is predicated when CHECK is on.
template <int G, int DT, bool HAS_EMPTY, bool CHECK>
__device__ inline void walk8(const uint4& cc, const float4& vv, int j, int64_t e, int64_t es,
                             int64_t ee, const void* __restrict__ H, int64_t ldh,
                             int64_t coff_load, void* __restrict__ Z, int64_t ldz, int64_t coff,
                             bool active, float* my_part, const int64_t* __restrict__ rowptr,
                             int64_t row_end, GroupState<Feat<DT>::VEC>& st)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    uint32_t c[8];
    float a[8];
    typename F::Raw h[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        c[u] = __shfl(comp(cc, u & 3), j + (u >> 2), G);
        a[u] = __shfl(comp(vv, u & 3), j + (u >> 2), G);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) h[u] = *F::ptr(H, (int64_t)(c[u] & ~kEndBit) * ldh + coff_load);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        if (CHECK && !(e + u >= es && e + u < ee)) continue;
        float x[VEC];
        F::widen(h[u], x);
#pragma unroll
        for (int i = 0; i < VEC; ++i) st.acc[i] = fmaf(a[u], x[i], st.acc[i]);
        st.pending = true;
        if (c[u] & kEndBit) {
            if (active) {
                if (st.head) {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) my_part[i] = st.acc[i];
                } else {
                    F::store(Z, st.r * ldz + coff, st.acc);
                }
            }
            st.head = false;
            st.pending = false;
#pragma unroll
            for (int i = 0; i < VEC; ++i) st.acc[i] = 0.f;
            ++st.r;
            if (HAS_EMPTY) {
                while (st.r + 1 < row_end && rowptr[st.r + 1] <= e + u + 1) ++st.r;
            }
        }
    }
}

// Partial-sum slots: [group in call][head = 0 / tail = 1][G * VEC] fp32.
template <int G, int DT, bool HAS_EMPTY>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(
    const int64_t* __restrict__ rowptr, const uint32_t* __restrict__ colf,
    const float* __restrict__ val, const uint32_t* __restrict__ grp_row,
    const void* __restrict__ H, int64_t ldh, void* __restrict__ Z, int64_t ldz, int c0, int width,
    int64_t row_begin, int64_t row_end, int64_t e_begin, int64_t e_end, int64_t k_first,
    int64_t n_groups_call, float* __restrict__ partials)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    constexpr int GPB = kBlock / G;        // groups per block
    constexpr int CHUNK = 4 * G;           // entries staged per index load
    constexpr int PW = G * VEC;            // padded slice width
    const int lg = threadIdx.x % G;        // lane within group
    const int64_t gk = (int64_t)blockIdx.x * GPB + threadIdx.x / G;
    if (gk >= n_groups_call) return;
    const int64_t k = k_first + gk;
    const int64_t gs = k * kL;
    const int64_t es = gs > e_begin ? gs : e_begin;
    const int64_t ee = (gs + kL) < e_end ? (gs + kL) : e_end;
    if (es >= ee) return;

    GroupState<VEC> st;
    st.r = (gs < e_begin) ? row_begin : (int64_t)grp_row[k];
    if (HAS_EMPTY) {
        while (st.r + 1 < row_end && rowptr[st.r + 1] <= es) ++st.r;
    }
    st.head = es > rowptr[st.r];
    st.pending = false;
#pragma unroll
    for (int i = 0; i < VEC; ++i) st.acc[i] = 0.f;
    const bool active = lg * VEC < width;
    const int64_t coff = (int64_t)c0 + (int64_t)lg * VEC;
    const int64_t coff_load = active ? coff : (int64_t)c0;  // idle lanes re-read column c0
    float* my_part = partials + (size_t)gk * 2 * PW + (size_t)lg * VEC;

    for (int ch = 0; ch < kL / CHUNK; ++ch) {
        const int64_t cb = gs + (int64_t)ch * CHUNK;
        if (cb >= ee) break;
        if (cb + CHUNK <= es) continue;
        // colf / val are padded to a whole number of windows, so these loads stay in bounds
        const uint4 cc = *reinterpret_cast<const uint4*>(colf + cb + 4 * lg);
        const float4 vv = *reinterpret_cast<const float4*>(val + cb + 4 * lg);
        if ((cb >= es) && (cb + CHUNK <= ee)) {
#pragma unroll 1
            for (int j = 0; j < G; j += 2)
                walk8<G, DT, HAS_EMPTY, false>(cc, vv, j, cb + 4 * j, es, ee, H, ldh, coff_load, Z,
                                               ldz, coff, active, my_part, rowptr, row_end, st);
        } else {
#pragma unroll 1
            for (int j = 0; j < G; j += 2)
                walk8<G, DT, HAS_EMPTY, true>(cc, vv, j, cb + 4 * j, es, ee, H, ldh, coff_load, Z,
                                              ldz, coff, active, my_part, rowptr, row_end, st);
        }
    }
    if (st.pending && active) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) my_part[PW + i] = st.acc[i];
    }
}

// One lane group per window boundary; the group whose boundary is the first one crossed by a
// row adds that row's pieces in window order and writes the row.
template <int G, int DT>
__global__ __launch_bounds__(kBlock) void aggregate_fixup_kernel(
    const int64_t* __restrict__ rowptr, const uint32_t* __restrict__ grp_row,
    void* __restrict__ Z, int64_t ldz, int c0, int width, int64_t e_begin, int64_t e_end,
    int64_t k_first, int64_t n_groups_call, const float* __restrict__ partials)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    constexpr int GPB = kBlock / G;
    constexpr int PW = G * VEC;
    const int lg = threadIdx.x % G;
    const int64_t gk = (int64_t)blockIdx.x * GPB + threadIdx.x / G + 1;
    if (gk >= n_groups_call) return;
    const int64_t b = (k_first + gk) * kL;  // boundary between windows gk-1 and gk
    if (b <= e_begin || b >= e_end) return;
    const int64_t r = grp_row[k_first + gk];
    const int64_t rs = rowptr[r];
    if (rs >= b) return;                  // a row starts exactly here: nothing crosses
    if ((rs / kL + 1) * kL != b) return;  // not the first boundary this row crosses
    if (lg * VEC >= width) return;
    const int64_t re = rowptr[r + 1];
    float acc[VEC];
    const float* p = partials + (size_t)(gk - 1) * 2 * PW + PW + (size_t)lg * VEC;  // tail
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = p[i];
    int64_t kk = gk;
    while ((k_first + kk + 1) * kL < re) {  // windows that lie wholly inside the row
        p = partials + (size_t)kk * 2 * PW + PW + (size_t)lg * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += p[i];
        ++kk;
    }
    p = partials + (size_t)kk * 2 * PW + (size_t)lg * VEC;  // head of the window where it ends
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] += p[i];
    F::store(Z, r * ldz + (int64_t)c0 + (int64_t)lg * VEC, acc);
}

template <int DT>
__global__ __launch_bounds__(kBlock) void zero_rows_kernel(void* Z, int64_t ldz, int c0, int width,
                                                           int64_t row_begin, int64_t row_end)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rows = row_end - row_begin;
    if (i >= rows * width) return;
    const int64_t r = row_begin + i / width;
    const int c = c0 + (int)(i % width);
    if (DT == MIXGCN_F32) reinterpret_cast<float*>(Z)[r * ldz + c] = 0.f;
    else reinterpret_cast<uint16_t*>(Z)[r * ldz + c] = 0;
}

template <int G, int DT>
int launch_one(const Csr& m, const void* H, int64_t ldh, void* Z, int64_t ldz, int c0, int width,
               int64_t r0, int64_t r1, int64_t e0, int64_t e1, float* partials, hipStream_t s)
{
    constexpr int GPB = kBlock / G;
    const int64_t k_first = e0 / kL;
    const int64_t n_groups = ceil_div(e1, kL) - k_first;
    const unsigned grid = (unsigned)ceil_div(n_groups, GPB);
    if (m.has_empty_rows)
        hipLaunchKernelGGL((aggregate_kernel<G, DT, true>), dim3(grid), dim3(kBlock), 0, s,
                           m.rowptr, m.colf, m.val, m.grp_row, H, ldh, Z, ldz, c0, width, r0, r1,
                           e0, e1, k_first, n_groups, partials);
    else
        hipLaunchKernelGGL((aggregate_kernel<G, DT, false>), dim3(grid), dim3(kBlock), 0, s,
                           m.rowptr, m.colf, m.val, m.grp_row, H, ldh, Z, ldz, c0, width, r0, r1,
                           e0, e1, k_first, n_groups, partials);
    if (n_groups > 1) {
        const unsigned fgrid = (unsigned)ceil_div(n_groups - 1, GPB);
        hipLaunchKernelGGL((aggregate_fixup_kernel<G, DT>), dim3(fgrid), dim3(kBlock), 0, s,
                           m.rowptr, m.grp_row, Z, ldz, c0, width, e0, e1, k_first, n_groups,
                           partials);
    }
    return MIXGCN_OK;
}

template <int DT>
int launch_dt(const mixgcn_graph* g, const Csr& m, const void* H, int64_t ldh, void* Z,
              int64_t ldz, int32_t c0, int32_t c1, int64_t r0, int64_t r1, hipStream_t s)
{
    constexpr int VEC = Feat<DT>::VEC;
    constexpr int kMaxTile = 64 * VEC;  // widest slice one pass can hold
    if (m.has_empty_rows) {
        const int64_t cells = (r1 - r0) * (int64_t)(c1 - c0);
        hipLaunchKernelGGL((zero_rows_kernel<DT>), dim3((unsigned)ceil_div(cells, kBlock)),
                           dim3(kBlock), 0, s, Z, ldz, c0, c1 - c0, r0, r1);
    }
    const int64_t e0 = m.h_rowptr[(size_t)r0], e1 = m.h_rowptr[(size_t)r1];
    if (e1 <= e0) return MIXGCN_OK;
    const int64_t n_groups = ceil_div(e1, kL) - e0 / kL;
    // scratch for the row pieces: sized for the widest pass of this call
    const int wmax = (c1 - c0) < kMaxTile ? (c1 - c0) : kMaxTile;
    int gmax = 4;
    while (gmax * VEC < wmax) gmax *= 2;
    const size_t need = (size_t)n_groups * 2 * gmax * VEC * sizeof(float);
    if (need > g->partials_bytes) {
        // growing the scratch waits for earlier work that may still read the old one
        MIXGCN_HIP_TRY(hipDeviceSynchronize());
        if (g->partials) (void)hipFree(g->partials);
        g->partials = nullptr;
        g->partials_bytes = 0;
        const size_t want = need + need / 4;
        MIXGCN_HIP_TRY(hipMalloc((void**)&g->partials, want));
        g->partials_bytes = want;
    }
    for (int32_t cb = c0; cb < c1; cb += kMaxTile) {
        const int w = (c1 - cb) < kMaxTile ? (c1 - cb) : kMaxTile;
        int G = 4;
        while (G * VEC < w) G *= 2;
        switch (G) {
        case 4: MIXGCN_TRY((launch_one<4, DT>(m, H, ldh, Z, ldz, cb, w, r0, r1, e0, e1, g->partials, s))); break;
        case 8: MIXGCN_TRY((launch_one<8, DT>(m, H, ldh, Z, ldz, cb, w, r0, r1, e0, e1, g->partials, s))); break;
        case 16: MIXGCN_TRY((launch_one<16, DT>(m, H, ldh, Z, ldz, cb, w, r0, r1, e0, e1, g->partials, s))); break;
        case 32: MIXGCN_TRY((launch_one<32, DT>(m, H, ldh, Z, ldz, cb, w, r0, r1, e0, e1, g->partials, s))); break;
        default: MIXGCN_TRY((launch_one<64, DT>(m, H, ldh, Z, ldz, cb, w, r0, r1, e0, e1, g->partials, s))); break;
        }
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace

int launch_aggregate(const mixgcn_graph* g, const Csr& m, int dtype, const void* H, int64_t ldh,
                     void* Z, int64_t ldz, int32_t c0, int32_t c1, int64_t r0, int64_t r1,
                     hipStream_t s)
{
    if (dtype == MIXGCN_F32) return launch_dt<MIXGCN_F32>(g, m, H, ldh, Z, ldz, c0, c1, r0, r1, s);
    return launch_dt<MIXGCN_BF16>(g, m, H, ldh, Z, ldz, c0, c1, r0, r1, s);
}

}  // namespace mixgcn
