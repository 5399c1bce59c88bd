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
#include <cstdlib>

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

// The walk is a rolling software pipeline over batches of U entries: while the feature rows of
// batch b are consumed one by one, the load for the same slot of batch b + 1 is issued as soon
// as the slot's data has been copied out, so a lane group keeps U row loads in flight all the
// time.  Index and value of an entry are staged 4 per lane with one 16-byte load per chunk of
// 4 G entries (the next chunk is fetched one chunk ahead) and broadcast inside the group with
// lane shuffles.  All loads are in bounds by construction (padding entries carry column 0 and
// value 0); with CHECK only the accumulation is predicated on the entry lying in [es, ee).
template <int G, int DT, int U, bool HAS_EMPTY, bool CHECK>
__device__ inline void roll(uint32_t (&c)[U], float (&a)[U], typename Feat<DT>::Raw (&h)[U],
                            const uint4& ncc, const float4& nvv, int nj, bool issue, int64_t e,
                            int64_t es, int64_t ee, const void* __restrict__ H, int64_t ldh,
                            int64_t coff_load, void* __restrict__ Z, int64_t ldz, int64_t coff,
                            bool active, float* my_part, int part_stride,
                            const int64_t* __restrict__ rowptr, int64_t row_end,
                            GroupState<Feat<DT>::VEC>& st)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float x[VEC];
        F::widen(h[u], x);
        const uint32_t cu = c[u];
        const float au = a[u];
        if (issue) {
            c[u] = __shfl(comp(ncc, u & 3), nj + (u >> 2), G);
            a[u] = __shfl(comp(nvv, u & 3), nj + (u >> 2), G);
            h[u] = *F::ptr(H, (int64_t)(c[u] & ~kEndBit) * ldh + coff_load);
        }
        if (CHECK && !(e + u >= es && e + u < ee)) continue;
#pragma unroll
        for (int i = 0; i < VEC; ++i) st.acc[i] = fmaf(au, x[i], st.acc[i]);
        st.pending = true;
        if (cu & kEndBit) {
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

// Partial-sum slots: [window in call][head = 0 / tail = 1][part_stride] fp32, indexed by the
// column offset within the pass.
template <int G, int DT, int U, bool HAS_EMPTY>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(
    const int64_t* __restrict__ rowptr, const uint32_t* __restrict__ colf,
    const float* __restrict__ val, const uint32_t* __restrict__ grp_row,
    const void* __restrict__ H, int64_t ldh, void* __restrict__ Z, int64_t ldz, int c0, int width,
    int64_t row_begin, int64_t row_end, int64_t e_begin, int64_t e_end, int64_t k_first,
    int64_t n_groups_call, float* __restrict__ partials, int n_slices, int part_stride)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    constexpr int GPB = kBlock / G;        // groups per block
    constexpr int CHUNK = 4 * G;           // entries staged per index load
    constexpr int BPC = CHUNK / U;         // batches per chunk
    constexpr int PW = G * VEC;            // columns of one slice
    static_assert(CHUNK % U == 0 && U % 4 == 0, "batch must tile the staged chunk");
    const int lg = threadIdx.x % G;        // lane within group
    // Consecutive workgroups are dealt round-robin to the 8 XCDs, so taking the column slice
    // from the low bits of the block index pins every slice to a fixed subset of the XCDs:
    // each L2 then caches only its own 1/n_slices of the hot feature rows.
    const int slice = (int)(blockIdx.x % (unsigned)n_slices);
    const int64_t gk = (int64_t)(blockIdx.x / (unsigned)n_slices) * GPB + threadIdx.x / G;
    if (gk >= n_groups_call) return;
    c0 += slice * PW;
    width -= slice * PW;
    if (width > PW) width = PW;
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
    float* my_part = partials + (size_t)gk * 2 * part_stride + (size_t)slice * PW + (size_t)lg * VEC;

    // chunks of this window that overlap [es, ee)
    const int ch_begin = (int)((es - gs) / CHUNK);
    const int ch_end = (int)((ee - gs + CHUNK - 1) / CHUNK);
    // colf / val are padded to a whole number of windows, so staging loads stay in bounds
    uint4 cc = *reinterpret_cast<const uint4*>(colf + gs + (int64_t)ch_begin * CHUNK + 4 * lg);
    float4 vv = *reinterpret_cast<const float4*>(val + gs + (int64_t)ch_begin * CHUNK + 4 * lg);
    uint32_t c[U];
    float a[U];
    typename F::Raw h[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {  // prologue: first batch of the first chunk
        c[u] = __shfl(comp(cc, u & 3), u >> 2, G);
        a[u] = __shfl(comp(vv, u & 3), u >> 2, G);
        h[u] = *F::ptr(H, (int64_t)(c[u] & ~kEndBit) * ldh + coff_load);
    }
    for (int ch = ch_begin; ch < ch_end; ++ch) {
        const bool more = ch + 1 < ch_end;
        uint4 ccn = cc;
        float4 vvn = vv;
        if (more) {
            ccn = *reinterpret_cast<const uint4*>(colf + gs + (int64_t)(ch + 1) * CHUNK + 4 * lg);
            vvn = *reinterpret_cast<const float4*>(val + gs + (int64_t)(ch + 1) * CHUNK + 4 * lg);
        }
        const int64_t cb = gs + (int64_t)ch * CHUNK;
        const bool full = (cb >= es) && (cb + CHUNK <= ee);
#pragma unroll 1
        for (int jb = 0; jb < BPC; ++jb) {
            const bool last = jb == BPC - 1;
            const uint4 ncc = last ? ccn : cc;
            const float4 nvv = last ? vvn : vv;
            const int nj = last ? 0 : (jb + 1) * (U / 4);
            const bool issue = !last || more;
            const int64_t e = cb + (int64_t)jb * U;
            if (full)
                roll<G, DT, U, HAS_EMPTY, false>(c, a, h, ncc, nvv, nj, issue, e, es, ee, H, ldh,
                                                 coff_load, Z, ldz, coff, active, my_part,
                                                 part_stride, rowptr, row_end, st);
            else
                roll<G, DT, U, HAS_EMPTY, true>(c, a, h, ncc, nvv, nj, issue, e, es, ee, H, ldh,
                                                coff_load, Z, ldz, coff, active, my_part,
                                                part_stride, rowptr, row_end, st);
        }
        cc = ccn;
        vv = vvn;
    }
    if (st.pending && active) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) my_part[part_stride + i] = st.acc[i];
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

// Row loads a lane group keeps in flight (8 or 16); MIXGCN_AGG_BATCH overrides for experiments.
int batch_entries()
{
    static const int v = [] {
        const char* e = getenv("MIXGCN_AGG_BATCH");
        const int x = e ? atoi(e) : 8;
        return x == 16 ? 16 : 8;
    }();
    return v;
}

template <int G, int DT>
int launch_main(const Csr& m, const void* H, int64_t ldh, void* Z, int64_t ldz, int c0, int width,
                int64_t r0, int64_t r1, int64_t e0, int64_t e1, float* partials, int part_stride,
                hipStream_t s, Timer* timer)
{
    constexpr int GPB = kBlock / G;
    constexpr int PW = G * Feat<DT>::VEC;
    // timed by the width class of the whole pass (lanes that would span it), not of a slice
    const int gf = part_stride / Feat<DT>::VEC;
    const int kind = gf == 4 ? kTimeAggG4 : gf == 8 ? kTimeAggG8 : gf == 16 ? kTimeAggG16
                     : gf == 32 ? kTimeAggG32 : kTimeAggG64;
    const int n_slices = (int)ceil_div(width, PW);
    const int64_t k_first = e0 / kL;
    const int64_t n_groups = ceil_div(e1, kL) - k_first;
    const int64_t grid64 = ceil_div(n_groups, GPB) * n_slices;
    if (grid64 > 0x7FFFFFFF) return fail(MIXGCN_EINVAL, "aggregate: grid too large");
    const unsigned grid = (unsigned)grid64;
    if (timer) MIXGCN_TRY(timer->begin(kind, s));
#define MIXGCN_AGG_LAUNCH(UU, EMPTY)                                                              \
    hipLaunchKernelGGL((aggregate_kernel<G, DT, UU, EMPTY>), dim3(grid), dim3(kBlock), 0, s,       \
                       m.rowptr, m.colf, m.val, m.grp_row, H, ldh, Z, ldz, c0, width, r0, r1, e0,  \
                       e1, k_first, n_groups, partials, n_slices, part_stride)
    if (batch_entries() == 16) {
        if (m.has_empty_rows) MIXGCN_AGG_LAUNCH(16, true);
        else MIXGCN_AGG_LAUNCH(16, false);
    } else {
        if (m.has_empty_rows) MIXGCN_AGG_LAUNCH(8, true);
        else MIXGCN_AGG_LAUNCH(8, false);
    }
#undef MIXGCN_AGG_LAUNCH
    if (timer) MIXGCN_TRY(timer->end(s));
    return MIXGCN_OK;
}

template <int GF, int DT>
int launch_fixup(const Csr& m, void* Z, int64_t ldz, int c0, int width, int64_t e0, int64_t e1,
                 const float* partials, hipStream_t s)
{
    constexpr int GPB = kBlock / GF;
    const int64_t k_first = e0 / kL;
    const int64_t n_groups = ceil_div(e1, kL) - k_first;
    if (n_groups > 1) {
        const unsigned fgrid = (unsigned)ceil_div(n_groups - 1, GPB);
        hipLaunchKernelGGL((aggregate_fixup_kernel<GF, DT>), dim3(fgrid), dim3(kBlock), 0, s,
                           m.rowptr, m.grp_row, Z, ldz, c0, width, e0, e1, k_first, n_groups,
                           partials);
    }
    return MIXGCN_OK;
}

// Lanes per group of the main kernel (columns per slice = lanes * 4 fp32 or * 8 bf16).
// 8 lanes = 128 bytes of every gathered row = one cache line.  MIXGCN_AGG_GROUP overrides it
// (4, 8, 16, 32 or 64) for experiments.
int slice_group_lanes()
{
    static const int v = [] {
        const char* e = getenv("MIXGCN_AGG_GROUP");
        const int x = e ? atoi(e) : 16;
        return (x == 4 || x == 8 || x == 16 || x == 32 || x == 64) ? x : 16;
    }();
    return v;
}

template <int DT>
int launch_dt(const mixgcn_graph* g, const Csr& m, const void* H, int64_t ldh, void* Z,
              int64_t ldz, int32_t c0, int32_t c1, int64_t r0, int64_t r1, hipStream_t s,
              Timer* timer)
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
        int GF = 4;  // lanes that span the whole pass: fix-up group and partial-slot stride
        while (GF * VEC < w) GF *= 2;
        int G = slice_group_lanes();
        if (G > GF) G = GF;
        const int ps = GF * VEC;
        float* P = g->partials;
#define MIXGCN_AGG_MAIN(GG) \
    MIXGCN_TRY((launch_main<GG, DT>(m, H, ldh, Z, ldz, cb, w, r0, r1, e0, e1, P, ps, s, timer)))
#define MIXGCN_AGG_FIX(GG) MIXGCN_TRY((launch_fixup<GG, DT>(m, Z, ldz, cb, w, e0, e1, P, s)))
        switch (G) {
        case 4: MIXGCN_AGG_MAIN(4); break;
        case 8: MIXGCN_AGG_MAIN(8); break;
        case 16: MIXGCN_AGG_MAIN(16); break;
        case 32: MIXGCN_AGG_MAIN(32); break;
        default: MIXGCN_AGG_MAIN(64); break;
        }
        switch (GF) {
        case 4: MIXGCN_AGG_FIX(4); break;
        case 8: MIXGCN_AGG_FIX(8); break;
        case 16: MIXGCN_AGG_FIX(16); break;
        case 32: MIXGCN_AGG_FIX(32); break;
        default: MIXGCN_AGG_FIX(64); break;
        }
#undef MIXGCN_AGG_MAIN
#undef MIXGCN_AGG_FIX
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace

int launch_aggregate(const mixgcn_graph* g, const Csr& m, int dtype, const void* H, int64_t ldh,
                     void* Z, int64_t ldz, int32_t c0, int32_t c1, int64_t r0, int64_t r1,
                     hipStream_t s, Timer* timer)
{
    if (dtype == MIXGCN_F32)
        return launch_dt<MIXGCN_F32>(g, m, H, ldh, Z, ldz, c0, c1, r0, r1, s, timer);
    return launch_dt<MIXGCN_BF16>(g, m, H, ldh, Z, ldz, c0, c1, r0, r1, s, timer);
}

}  // namespace mixgcn
