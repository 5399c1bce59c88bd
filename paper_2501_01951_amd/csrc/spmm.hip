// Neighbor aggregation  Z[r, c0:c1) = sum_e val[e] * H[col[e], c0:c1)  (paper Algorithm 2,
// aggregation phase; with the transpose CSR its adjoint for the backward pass) as a gather
// kernel balanced by stored entries rather than by rows.
//
// Work split.  A pass handles up to 256 fp32 (512 bf16) columns and is cut into column slices
// of LPR lanes x 16 bytes.  One wavefront walks one *span* of consecutive stored entries for one
// slice: its 64 lanes form 64 / LPR sub-groups, sub-group s takes entry s of every batch of
// 64 / LPR entries, so one 16-byte load per lane fetches the slice of 64 / LPR neighbor rows.
// Every wavefront does the same amount of gather work (256 such loads) whatever the degree
// distribution: a hub is spread over many spans, a run of short rows shares one.  Control flow
// is uniform across the wavefront: the end-of-row marks (bit 31 of an entry's column word) of a
// batch are collected with one ballot, and only when a row ends inside the batch the sub-group
// sums are combined with lane shuffles and the row is written.
//
// Rows that cross a span boundary are finished by a second, tiny kernel: a wavefront stores the
// piece that completes a row begun in an earlier span in its "head" slot and the piece of a row
// it cannot complete in its "tail" slot; the fix-up kernel adds the pieces of each such row in
// span order.  No atomics: the result is deterministic.
//
// XCD mapping.  The slice index is taken from the low bits of the workgroup index.  Workgroups
// are dealt round-robin to the 8 XCDs, so every slice is pinned to a fixed subset of the XCDs
// and each private L2 caches only its own part of the hot feature rows.
#include <mutex>

#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

constexpr int kBatchesPerSpan = 256;  // gather instructions per wavefront (fewer on small inputs)
constexpr int kDepth = 4;             // gather instructions a wavefront keeps in flight

// 16-byte feature vector: 4 fp32 or 8 bf16 (widened to fp32)
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
    __device__ static inline void store_one(void* base, int64_t elem_off, float a)
    {
        reinterpret_cast<float*>(base)[elem_off] = a;
    }
    __device__ static inline const Raw* ptr(const void* base, int64_t elem_off)
    {
        return reinterpret_cast<const Raw*>(reinterpret_cast<const float*>(base) + elem_off);
    }
};

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
    // two fp32 -> two bf16, round to nearest even, by the conversion instruction of this part
    // (rounding in software made a row's end a third of the vector work of this kernel at bf16)
    __device__ static inline uint32_t pack2(float lo, float hi)
    {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        const floatx2 v = {lo, hi};
        const bf16x2 h = __builtin_convertvector(v, bf16x2);
        uint32_t u;
        __builtin_memcpy(&u, &h, 4);
        return u;
    }
    __device__ static inline void store(void* base, int64_t elem_off, const float* a)
    {
        uint4 r;
        r.x = pack2(a[0], a[1]);
        r.y = pack2(a[2], a[3]);
        r.z = pack2(a[4], a[5]);
        r.w = pack2(a[6], a[7]);
        *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(base) + elem_off) = r;
    }
    __device__ static inline void store_one(void* base, int64_t elem_off, float a)
    {
        reinterpret_cast<uint16_t*>(base)[elem_off] = (uint16_t)pack2(a, 0.f);
    }
    __device__ static inline const Raw* ptr(const void* base, int64_t elem_off)
    {
        return reinterpret_cast<const Raw*>(reinterpret_cast<const uint16_t*>(base) + elem_off);
    }
};

// Writes a lane's VEC columns [c, c + VEC) of one output row: the whole 16-byte group when it
// lies inside the call's column range [c_lo, c_hi), else only the elements that do, one by one
// (a range need not start or end on a group; what lies outside it is never written).
template <int DT>
__device__ inline void store_in_range(void* Z, int64_t row_off, int64_t c, const float* t, int c_lo,
                                      int c_hi)
{
    using F = Feat<DT>;
    if (c >= c_lo && c + F::VEC <= c_hi) {
        F::store(Z, row_off + c, t);
    } else {
#pragma unroll
        for (int i = 0; i < F::VEC; ++i)
            if (c + i >= c_lo && c + i < c_hi) F::store_one(Z, row_off + c + i, t[i]);
    }
}

// A value that is the same in every lane, moved to scalar registers.
__device__ inline int uniform32(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline int64_t uniform64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Sum over the 64 / LPR sub-groups of a wavefront (lanes that hold the same columns).
template <int LPR, int VEC>
__device__ inline void reduce_subgroups(float* v)
{
#pragma unroll
    for (int d = LPR; d < kWave; d <<= 1)
#pragma unroll
        for (int i = 0; i < VEC; ++i) v[i] += __shfl_xor(v[i], d, kWave);
}

// Output mask of the S-SpMM (paper Eq. 4), a bitmap: column c of row r is bit c % 32 of word
// mask[r * ldm + c / 32].  A lane's VEC consecutive columns start at a multiple of VEC, so
// their bits lie in one word.
template <int VEC>
__device__ inline void apply_mask(float* t, const uint32_t* __restrict__ mask, int64_t ldm,
                                  int64_t r, int64_t c)
{
    const uint32_t bits = mask[r * ldm + (c >> 5)] >> (c & 31);
#pragma unroll
    for (int i = 0; i < VEC; ++i) t[i] = ((bits >> i) & 1u) ? t[i] : 0.f;
}

// Epilogue flags carried in the kernels' `relu` argument (MIXGCN_EPI_* of the ABI).
constexpr int kEpiRelu = 1;        // Z = max(., 0)
constexpr int kEpiAccumulate = 2;  // Z = Z + (.): the finished row sum is added to what Z holds

template <int DT>
__device__ inline void add_stored(float* t, const void* Z, int64_t elem_off)
{
    using F = Feat<DT>;
    float o[F::VEC];
    F::widen(*F::ptr(Z, elem_off), o);
#pragma unroll
    for (int i = 0; i < F::VEC; ++i) t[i] += o[i];
}

// Partial-sum slots: [span in call][head = 0 / tail = 1][part_stride] fp32, indexed by the
// column offset within the pass.
// GF = lanes that would span the whole pass (its width class: 4 GF fp32 or 8 GF bf16 columns);
// it fixes the stride of the partial-sum slots and names the instantiation in profiles.
// OFF32: every byte offset into H fits 32 bits and every column index 24 bits, so a gather
// address is a scalar base plus one 24-bit multiply-add per lane.
template <int LPR, int GF, int DT, bool HAS_EMPTY, bool OFF32>
__global__ __launch_bounds__(kBlock) void aggregate_kernel(
    const int64_t* __restrict__ rowptr, const uint2* __restrict__ cv,
    const uint32_t* __restrict__ grp_row, const void* __restrict__ H, int64_t ldh,
    void* __restrict__ Z, int64_t ldz, int c0, int width, int64_t row_begin, int64_t row_end,
    int64_t e_begin, int64_t e_end, int64_t span_first, int64_t n_spans,
    float* __restrict__ partials, int n_slices, int relu, const uint32_t* __restrict__ mask,
    int64_t ldm, int span_batches, int c_lo, int c_hi)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    constexpr int part_stride = GF * VEC;
    constexpr int EPB = kWave / LPR;                  // entries per batch (= sub-groups)
    const int64_t SPAN = (int64_t)span_batches * EPB; // a multiple of kGroupNnz
    constexpr int PW = LPR * VEC;                     // columns of one slice
    constexpr int D = (kDepth * EPB <= kWave) ? kDepth : (kWave / EPB);  // slots per round
    constexpr uint64_t kLane0Mask = LPR == 64 ? 1ull
                                  : LPR == 32 ? 0x0000000100000001ull
                                  : LPR == 16 ? 0x0001000100010001ull
                                  : LPR == 8  ? 0x0101010101010101ull
                                              : 0x1111111111111111ull;
    const int lane = threadIdx.x & (kWave - 1);
    const int sub = lane / LPR;   // entry of the batch this lane works on
    const int lj = lane % LPR;    // position inside the slice
    const int slice = (int)(blockIdx.x % (unsigned)n_slices);
    const int64_t sk = uniform64((int64_t)(blockIdx.x / (unsigned)n_slices) * (kBlock / kWave) +
                                 (threadIdx.x >> 6));
    if (sk >= n_spans) return;
    c0 += slice * PW;
    width -= slice * PW;
    if (width > PW) width = PW;
    const int64_t gs = (span_first + sk) * SPAN;
    const int64_t es = gs > e_begin ? gs : e_begin;
    const int64_t ee = (gs + SPAN) < e_end ? (gs + SPAN) : e_end;
    if (es >= ee) return;

    // row that holds the first entry of the span (uniform)
    int64_t r = (gs < e_begin) ? row_begin : (int64_t)grp_row[gs / kGroupNnz];
    r = uniform64(r);
    if (HAS_EMPTY) {
        while (r + 1 < row_end && rowptr[r + 1] <= es) ++r;
    }
    bool head = es > rowptr[r];  // the first completed piece belongs to a row begun earlier
    bool pending = false;        // acc holds entries of a row whose end has not been seen
    const bool active = lj * VEC < width;
    const int64_t coff = (int64_t)c0 + (int64_t)lj * VEC;
    const int64_t coff_load = active ? coff : (int64_t)c0;  // idle lanes re-read column c0
    float* const part = partials + (size_t)sk * 2 * part_stride + (size_t)slice * PW + (size_t)lj * VEC;

    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.f;

    // batches of this span that overlap [es, ee), and those that lie wholly inside it; all
    // per-batch bookkeeping is done on 32-bit positions relative to the span start
    const int es_rel = (int)(es - gs), ee_rel = (int)(ee - gs);
    const int b0 = es_rel / EPB;
    const int b1 = (ee_rel + EPB - 1) / EPB;
    const int b_in0 = (es_rel + EPB - 1) / EPB;  // first batch with no entry before es
    const int b_in1 = ee_rel / EPB;              // first batch with an entry at or after ee

    // Rolling pipeline over rounds of D batches; slot u of a round holds batch b + u.  The
    // entries {column word, value} of a whole round are fetched with ONE coalesced 8-byte load
    // per lane (lane l takes entry l of the round) two rounds ahead and handed to the lanes that
    // need them with shuffles; the feature rows are gathered one round ahead.  Two rounds are
    // written out per loop trip with the entry registers swapping roles, so no value that is
    // still in flight is ever copied (a copy would make the wavefront wait for the load).  cv is
    // padded past nnz (zero entries: column 0, value 0, no mark), so nothing here needs a bounds
    // check.
    constexpr int RE = D * EPB;  // entries per round (<= 64)
    static_assert(RE <= kWave, "a round's entries must fit one load per lane");
    const uint2* const rcv = cv + gs + (lane < RE ? lane : 0);  // entry `lane` of round 0 of span
    // byte address of this lane's 16 bytes in feature row 0; a row pitch always fits 32 bits, so
    // the address of a gathered row is one 32 x 32 + 64-bit multiply-add
    constexpr int ES = (int)sizeof(typename F::Raw) / VEC;  // bytes per stored element
    const char* const hbase = reinterpret_cast<const char*>(F::ptr(H, coff_load));
    const uint32_t pitch = (uint32_t)(ldh * ES);
    const uint32_t lane_off = (uint32_t)(coff_load * ES);
    uint32_t c[D];
    float a[D];
    typename F::Raw h[D];
    uint2 ea, eb2;

    auto fill = [&](int u, const uint2& en) {  // slot u <- entry u * EPB + sub of the round `en`
        c[u] = __shfl(en.x, u * EPB + sub, kWave);
        a[u] = __uint_as_float(__shfl(en.y, u * EPB + sub, kWave));
        if (OFF32) {
            // the 24-bit multiply ignores the mark bits of the column word
            const uint32_t off = __umul24(c[u], pitch) + lane_off;
            h[u] = *reinterpret_cast<const typename F::Raw*>(reinterpret_cast<const char*>(H) + off);
        } else {
            h[u] = *reinterpret_cast<const typename F::Raw*>(
                hbase + (uint64_t)(c[u] & kEntryColMask) * pitch);
        }
    };
    // one round: use the D slots (batches b .. b + D - 1), refilling each from `en` (the entries
    // of the round after).  No early exit: a batch past the end of the range has every lane
    // masked and adds nothing, which keeps the loop free of side exits so that the compiler can
    // count exactly how many younger loads may stay in flight at each use.
    auto round = [&](int b, const uint2& en) {
#pragma unroll
        for (int u = 0; u < D; ++u) {
            const int bb = b + u;
            const int eb = bb * EPB;  // first entry of the batch, relative to the span start
            uint32_t cu = c[u];
            float au = a[u];
            float x[VEC];
            F::widen(h[u], x);
            if (__builtin_expect(bb < b_in0 || bb >= b_in1, 0)) {  // batch straddles the range
                const bool ok = (eb + sub >= es_rel) && (eb + sub < ee_rel);
                if (!ok) {
                    cu = 0;
                    au = 0.f;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) x[i] = 0.f;
                }
            }
            uint64_t m = __ballot((int)cu < 0) & kLane0Mask;  // sub-groups whose entry ends a row
            if (__builtin_expect(m == 0, 1)) {
                pending = pending || bb < b1;
            } else {
                // Rows end in this batch.  t carries the open row's sum so far; each marked
                // sub-group closes one row: the lanes up to and including it add their products,
                // the sub-group sums are combined and the row (or its piece) is written.  acc is
                // only read here and restarts from zero, so the common multiply-add below is
                // the one place that writes it.
                float t[VEC];
#pragma unroll
                for (int i = 0; i < VEC; ++i) t[i] = acc[i];
                int prev = -1;
                while (m) {
                    const int p = (int)(__ffsll((unsigned long long)m) - 1) / LPR;
                    m &= m - 1;
                    if (sub > prev && sub <= p) {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) t[i] = fmaf(au, x[i], t[i]);
                    }
                    reduce_subgroups<LPR, VEC>(t);
                    if (sub == 0 && active) {
                        if (head) {
#pragma unroll
                            for (int i = 0; i < VEC; ++i) part[i] = t[i];
                        } else {
                            if (relu & kEpiAccumulate) add_stored<DT>(t, Z, r * ldz + coff);
                            if (relu & kEpiRelu) {
#pragma unroll
                                for (int i = 0; i < VEC; ++i) t[i] = fmaxf(t[i], 0.f);
                            }
                            if (mask) apply_mask<VEC>(t, mask, ldm, r, coff);
                            store_in_range<DT>(Z, r * ldz, coff, t, c_lo, c_hi);
                        }
                    }
                    head = false;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) t[i] = 0.f;
                    ++r;
                    if (HAS_EMPTY) {
                        while (r + 1 < row_end && rowptr[r + 1] <= gs + eb + p + 1) ++r;
                    }
                    prev = p;
                }
#pragma unroll
                for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
                if (sub <= prev) {  // these lanes' entries went into the rows just closed
                    au = 0.f;
#pragma unroll
                    for (int i = 0; i < VEC; ++i) x[i] = 0.f;
                }
                // entries after the last mark start a new row piece (only real ones count)
                pending = (eb + prev + 1 < ee_rel) && (prev + 1 < EPB);
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[i] = fmaf(au, x[i], acc[i]);
            fill(u, en);  // the batch D later
        }
    };

    ea = rcv[(int64_t)b0 * EPB];         // entries of the round at batch b0
    eb2 = rcv[(int64_t)(b0 + D) * EPB];  // round b0 + D
#pragma unroll
    for (int u = 0; u < D; ++u) fill(u, ea);
    for (int b = b0; b < b1; b += 2 * D) {
        ea = rcv[(int64_t)(b + 2 * D) * EPB];
        round(b, eb2);
        eb2 = rcv[(int64_t)(b + 3 * D) * EPB];
        round(b + D, ea);
    }
    if (pending) {
        reduce_subgroups<LPR, VEC>(acc);
        if (sub == 0 && active) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) part[part_stride + i] = acc[i];
        }
    }
}

// One lane group per span boundary; the group whose boundary is the first one crossed by a row
// adds that row's pieces in span order and writes the row.
template <int GF, int DT>
__global__ __launch_bounds__(kBlock) void aggregate_fixup_kernel(
    const int64_t* __restrict__ rowptr, const uint32_t* __restrict__ grp_row,
    void* __restrict__ Z, int64_t ldz, int c0, int width, int64_t e_begin, int64_t e_end,
    int64_t span, int64_t span_first, int64_t n_spans, const float* __restrict__ partials,
    int relu, const uint32_t* __restrict__ mask, int64_t ldm, int c_lo, int c_hi)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    constexpr int GPB = kBlock / GF;
    constexpr int PS = GF * VEC;  // stride of a partial slot
    const int lg = threadIdx.x % GF;
    const int64_t sk = (int64_t)blockIdx.x * GPB + threadIdx.x / GF + 1;
    if (sk >= n_spans) return;
    const int64_t b = (span_first + sk) * span;  // boundary between spans sk-1 and sk
    if (b <= e_begin || b >= e_end) return;
    const int64_t r = grp_row[b / kGroupNnz];
    const int64_t rs = rowptr[r];
    if (rs >= b) return;                    // a row starts exactly here: nothing crosses
    if ((rs / span + 1) * span != b) return;  // not the first boundary this row crosses
    if (lg * VEC >= width) return;
    const int64_t re = rowptr[r + 1];
    float acc[VEC];
    const float* p = partials + (size_t)(sk - 1) * 2 * PS + PS + (size_t)lg * VEC;  // tail
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = p[i];
    int64_t kk = sk;
    while ((span_first + kk + 1) * span < re) {  // spans that lie wholly inside the row
        p = partials + (size_t)kk * 2 * PS + PS + (size_t)lg * VEC;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] += p[i];
        ++kk;
    }
    p = partials + (size_t)kk * 2 * PS + (size_t)lg * VEC;  // head of the span where it ends
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] += p[i];
    if (relu & kEpiAccumulate) add_stored<DT>(acc, Z, r * ldz + (int64_t)c0 + (int64_t)lg * VEC);
    if (relu & kEpiRelu) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = fmaxf(acc[i], 0.f);
    }
    if (mask) apply_mask<VEC>(acc, mask, ldm, r, (int64_t)c0 + (int64_t)lg * VEC);
    store_in_range<DT>(Z, r * ldz, (int64_t)c0 + (int64_t)lg * VEC, acc, c_lo, c_hi);
}

// Rows without stored entries get no visit from the main kernel: they are set here, to zero, or
// (clamp_only, the accumulating call with ReLU) to max(Z, 0).  A thread looks at one row; the
// wavefront then writes each of its empty rows together, 64 columns at a time, so a graph with
// few empty rows costs one pass over the row pointers and a graph of mostly empty rows is
// written with whole lines.
template <int DT>
__global__ __launch_bounds__(kBlock) void empty_rows_kernel(const int64_t* __restrict__ rowptr,
                                                            void* Z, int64_t ldz, int c0, int width,
                                                            int64_t row_begin, int64_t row_end,
                                                            int clamp_only)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = row_begin + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool empty = r < row_end && rowptr[r + 1] == rowptr[r];
    uint64_t m = __ballot(empty);
    const int64_t wave_row0 = r - lane;
    while (m) {
        const int b = (int)__ffsll((unsigned long long)m) - 1;
        m &= m - 1;
        const int64_t rr = wave_row0 + b;
        for (int c = c0 + lane; c < c0 + width; c += kWave) {
            if (DT == MIXGCN_F32) {
                float* p = reinterpret_cast<float*>(Z) + rr * ldz + c;
                *p = clamp_only ? fmaxf(*p, 0.f) : 0.f;
            } else {
                uint16_t* p = reinterpret_cast<uint16_t*>(Z) + rr * ldz + c;
                if (!clamp_only || !(__uint_as_float((uint32_t)*p << 16) > 0.f)) *p = 0;
            }
        }
    }
}

// Entries per span of a pass: kBatchesPerSpan batches, halved while the launch would have fewer
// than 8192 wavefronts (a small graph is otherwise walked by a handful of long-running
// wavefronts), but never below the kGroupNnz entries that the span-start table resolves.
inline int64_t span_entries(int lpr, int64_t entries, int n_slices)
{
    const int epb = kWave / lpr;
    int64_t batches = kBatchesPerSpan;
    while (batches * epb > kGroupNnz && ceil_div(entries, batches * epb) * n_slices < 8192)
        batches /= 2;
    return batches * epb;
}

template <int LPR, int GF, int DT>
int launch_main(const Csr& m, const uint2* cv, int64_t n_nodes, const void* H, int64_t ldh,
                void* Z, int64_t ldz, int c0, int width,
                int64_t r0, int64_t r1, int64_t e0, int64_t e1, int64_t SPAN, float* partials,
                int relu, const uint32_t* mask, int64_t ldm, int c_lo, int c_hi, hipStream_t s,
                Timer* timer)
{
    constexpr int PW = LPR * Feat<DT>::VEC;
    // timed by the width class of the whole pass
    constexpr int kind = GF == 4 ? kTimeAggG4 : GF == 8 ? kTimeAggG8 : GF == 16 ? kTimeAggG16
                         : GF == 32 ? kTimeAggG32 : kTimeAggG64;
    const int n_slices = (int)ceil_div(width, PW);
    const int64_t span_first = e0 / SPAN;
    const int64_t n_spans = ceil_div(e1, SPAN) - span_first;
    const int64_t grid64 = ceil_div(n_spans, kBlock / kWave) * n_slices;
    if (grid64 > 0x7FFFFFFF) return fail(MIXGCN_EINVAL, "aggregate: grid too large");
    const unsigned grid = (unsigned)grid64;
    // 32-bit gather offsets when the whole feature matrix (as addressed from H) lies within
    // 4 GiB, its pitch fits 24 bits and the column indices fit 24 bits
    const int64_t esz = (int64_t)sizeof(typename Feat<DT>::Raw) / Feat<DT>::VEC;
    const bool off32 = (int64_t)n_nodes * ldh * esz + (int64_t)(c0 + width) * esz < (1ll << 32) &&
                       ldh * esz < (1ll << 24) && n_nodes <= (1ll << 24);
    if (timer) MIXGCN_TRY(timer->begin(kind, s));
#define MIXGCN_AGG_LAUNCH(EMPTY, O32)                                                            \
    hipLaunchKernelGGL((aggregate_kernel<LPR, GF, DT, EMPTY, O32>), dim3(grid), dim3(kBlock), 0, \
                       s, m.rowptr, cv, m.grp_row, H, ldh, Z, ldz, c0, width, r0, r1, e0, e1,  \
                       span_first, n_spans, partials, n_slices, relu, mask, ldm,                 \
                       (int)(SPAN / (kWave / LPR)), c_lo, c_hi)
    if (m.has_empty_rows) {
        if (off32) MIXGCN_AGG_LAUNCH(true, true);
        else MIXGCN_AGG_LAUNCH(true, false);
    } else {
        if (off32) MIXGCN_AGG_LAUNCH(false, true);
        else MIXGCN_AGG_LAUNCH(false, false);
    }
#undef MIXGCN_AGG_LAUNCH
    if (timer) MIXGCN_TRY(timer->end(s));
    return MIXGCN_OK;
}

template <int GF, int DT>
int launch_fixup(const Csr& m, void* Z, int64_t ldz, int c0, int width, int64_t e0, int64_t e1,
                 int64_t span, const float* partials, int relu, const uint32_t* mask,
                 int64_t ldm, int c_lo, int c_hi, hipStream_t s)
{
    constexpr int GPB = kBlock / GF;
    const int64_t span_first = e0 / span;
    const int64_t n_spans = ceil_div(e1, span) - span_first;
    if (n_spans > 1) {
        const unsigned fgrid = (unsigned)ceil_div(n_spans - 1, GPB);
        hipLaunchKernelGGL((aggregate_fixup_kernel<GF, DT>), dim3(fgrid), dim3(kBlock), 0, s,
                           m.rowptr, m.grp_row, Z, ldz, c0, width, e0, e1, span, span_first,
                           n_spans, partials, relu, mask, ldm, c_lo, c_hi);
    }
    return MIXGCN_OK;
}

// Lanes per slice of the main kernel for a pass that `gf` lanes would span (columns per slice
// = lanes * 4 fp32 or * 8 bf16): 8 lanes = one 128-byte line of every gathered row, so a
// 256-column pass has 8 slices, one per XCD.  (Measured best when the row pitch is an odd number
// of 128-byte lines; with a power-of-two pitch a slice's lines fall on few L2 channels.)
constexpr int slice_lanes(int gf) { return gf < 8 ? gf : 8; }

}  // namespace

// Measurement aid (mixgcn_set_aggregate_whole_rows): passes are not cut into column slices, a
// lane group gathers the whole width of the pass from every neighbor row.  That is the gather a
// kernel would have to do that keeps the aggregated tile on the compute unit for the update
// product (it needs every column of its rows), so timing it bounds such a fusion from below.
int g_aggregate_whole_rows = 0;

namespace {

// One pass: column block, width class and span length.
struct Pass { int32_t cb; int w, gf; int64_t span; };

// Width class of a pass of w columns (lanes that would span it), and its span length for a
// range of `entries` stored entries.
inline void plan_pass(int vec, int32_t cb, int w, int64_t entries, Pass* p)
{
    p->cb = cb;
    p->w = w;
    p->gf = 4;  // lanes that span the whole pass: fix-up group and partial-slot stride
    while (p->gf * vec < w) p->gf *= 2;
    const int lpr = g_aggregate_whole_rows ? p->gf : slice_lanes(p->gf);
    p->span = span_entries(lpr, entries, (int)ceil_div(w, lpr * vec));
}

}  // namespace

// Bytes of row-piece scratch a call over n_cols columns and the stored entries [e0, e1) needs:
// the widest of its passes, two slots of the pass's width class per span.
size_t agg_scratch_need(int dtype, int32_t n_cols, int64_t e0, int64_t e1)
{
    const int vec = dtype == MIXGCN_F32 ? 4 : 8;
    size_t need = 0;
    for (int32_t cb = 0; cb < n_cols && e1 > e0; cb += kAggMaxPassCols) {
        Pass p;
        plan_pass(vec, cb, (n_cols - cb) < kAggMaxPassCols ? (n_cols - cb) : kAggMaxPassCols,
                  e1 - e0, &p);
        const int64_t spans = ceil_div(e1, p.span) - e0 / p.span;
        const size_t bytes = (size_t)spans * 2 * p.gf * vec * sizeof(float);
        need = bytes > need ? bytes : need;
    }
    return need;
}

namespace {

template <int DT>
int launch_dt(const mixgcn_graph* g, const Csr& m, const uint2* cv, const void* H, int64_t ldh,
              void* Z, int64_t ldz, int32_t c0, int32_t c1, int64_t r0, int64_t r1, int relu,
              const uint32_t* mask, int64_t ldm, float* P, size_t P_bytes, hipStream_t s,
              Timer* timer)
{
    constexpr int VEC = Feat<DT>::VEC;
    const int64_t e0 = m.h_rowptr[(size_t)r0], e1 = m.h_rowptr[(size_t)r1];
    // the lanes work on whole 16-byte groups: the passes start at the group that holds the first
    // column, and the stores leave out what lies outside [c_lo, c_hi)
    const int32_t c_lo = c0, c_hi = c1;
    c0 = c0 / VEC * VEC;
    // the row pieces of every pass must fit the scratch: checked before anything is launched
    const size_t need = agg_scratch_need(DT, c1 - c0, e0, e1);
    if (need > P_bytes)
        return fail(MIXGCN_EINVAL, "aggregate: " + std::to_string(e1 - e0) + " stored entries at " +
                                       std::to_string(c1 - c0) + " columns need " +
                                       std::to_string(need) + " bytes of scratch for row pieces, " +
                                       std::to_string(P_bytes) + " are there");
    // an empty row adds nothing to an accumulating call, but a ReLU still clamps what it holds
    const bool acc_only = (relu & kEpiAccumulate) && !(relu & kEpiRelu);
    if (m.has_empty_rows && !acc_only && r1 > r0)
        hipLaunchKernelGGL((empty_rows_kernel<DT>), dim3((unsigned)ceil_div(r1 - r0, kBlock)),
                           dim3(kBlock), 0, s, m.rowptr, Z, ldz, c_lo, c_hi - c_lo, r0, r1,
                           (relu & kEpiAccumulate) ? 1 : 0);
    if (e1 <= e0) return MIXGCN_OK;
    for (int32_t cbk = c0; cbk < c1; cbk += kAggMaxPassCols) {
        Pass p;
        plan_pass(VEC, cbk, (c1 - cbk) < kAggMaxPassCols ? (c1 - cbk) : kAggMaxPassCols, e1 - e0, &p);
        const int32_t cb = p.cb;
        const int w = p.w;
        const int64_t span = p.span;
#define MIXGCN_AGG_PASS(GG)                                                                      \
    if (g_aggregate_whole_rows)                                                                  \
        MIXGCN_TRY((launch_main<GG, GG, DT>(m, cv, (int64_t)g->n, H, ldh, Z, ldz, cb, w, r0, r1, e0, \
                                            e1, span, P, relu, mask, ldm, c_lo, c_hi, s, timer))); \
    else                                                                                         \
        MIXGCN_TRY((launch_main<slice_lanes(GG), GG, DT>(m, cv, (int64_t)g->n, H, ldh, Z, ldz, cb, w, \
                                                         r0, r1, e0, e1, span, P, relu, mask,     \
                                                         ldm, c_lo, c_hi, s, timer)));            \
    MIXGCN_TRY((launch_fixup<GG, DT>(m, Z, ldz, cb, w, e0, e1, span, P, relu, mask, ldm, c_lo, c_hi, s)))
        switch (p.gf) {
        case 4: MIXGCN_AGG_PASS(4); break;
        case 8: MIXGCN_AGG_PASS(8); break;
        case 16: MIXGCN_AGG_PASS(16); break;
        case 32: MIXGCN_AGG_PASS(32); break;
        default: MIXGCN_AGG_PASS(64); break;
        }
#undef MIXGCN_AGG_PASS
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

// bit c % 32 of bits[r * ldb + c / 32] = X[r, c] > 0.  A lane takes the 16 bytes that hold
// columns [VEC q, VEC q + VEC) of one row, 32 / VEC neighboring lanes combine their bits into
// one word with OR-shuffles and the first of them writes it.  words = words written per row.
template <int DT>
__global__ __launch_bounds__(kBlock) void relu_bitmap_kernel(const void* __restrict__ X,
                                                             int64_t ldx, int64_t n, int cols,
                                                             int words, uint32_t* __restrict__ bits,
                                                             int64_t ldb)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;       // 4 fp32 or 8 bf16 per lane
    constexpr int LPW = 32 / VEC;     // lanes per word
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int qpr = words * LPW;      // lanes per row
    const int64_t r = i / qpr;
    const int q = (int)(i % qpr);
    const int c = q * VEC;
    uint32_t nib = 0;
    if (r < n && c < cols) {
        float x[VEC];
        F::widen(*F::ptr(X, r * ldx + c), x);
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            if (c + e < cols && x[e] > 0.f) nib |= 1u << e;
    }
    uint32_t w = nib << (VEC * (q % LPW));
#pragma unroll
    for (int o = 1; o < LPW; o <<= 1) w |= __shfl_xor(w, o, kWave);
    if (q % LPW == 0 && r < n) bits[r * ldb + q / LPW] = w;
}

// Dropout mask as a bitmap (forward use of the S-SpMM, Sec. 3.2.1).  Element (r, c) of the
// n x cols tensor is kept iff the upper half of output number r * cols + c of the SplitMix64
// generator started at `seed` is below `threshold` (= keep probability * 2^32).  One thread per
// word; every word of a row up to ldb is written, bits past `cols` are clear.
__device__ inline uint64_t splitmix64_at(uint64_t seed, uint64_t i)
{
    uint64_t z = seed + (i + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__global__ __launch_bounds__(kBlock) void dropout_bitmap_kernel(uint64_t seed, int64_t n, int cols,
                                                                uint64_t threshold,
                                                                uint32_t* __restrict__ bits,
                                                                int64_t ldb)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * ldb) return;
    const int64_t r = i / ldb;
    const int c0 = (int)(i % ldb) * 32;
    uint32_t w = 0;
#pragma unroll 8
    for (int b = 0; b < 32; ++b) {
        const int c = c0 + b;
        if (c < cols && (splitmix64_at(seed, (uint64_t)(r * cols + c)) >> 32) < threshold)
            w |= 1u << b;
    }
    bits[i] = w;
}

// X <- X (.) M for a bitmap M: a lane owns 16 bytes of a row (VEC columns, which lie in one
// mask word because VEC divides 32).
template <int DT>
__global__ __launch_bounds__(kBlock) void apply_bitmap_kernel(void* __restrict__ X, int64_t ldx,
                                                              int64_t n, int cols,
                                                              const uint32_t* __restrict__ bits,
                                                              int64_t ldb)
{
    using F = Feat<DT>;
    constexpr int VEC = F::VEC;
    const int vpr = (cols + VEC - 1) / VEC;  // vectors per row (the last may reach into the padding)
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * vpr) return;
    const int64_t r = i / vpr;
    const int c = (int)(i % vpr) * VEC;
    float x[VEC];
    F::widen(*F::ptr(X, r * ldx + c), x);
    apply_mask<VEC>(x, bits, ldb, r, c);
    F::store(X, r * ldx + c, x);
}

}  // namespace

int launch_apply_bitmap(int dtype, void* X, int64_t ldx, int64_t n, int32_t cols,
                        const uint32_t* bits, int64_t ldb, hipStream_t s)
{
    const int vec = dtype == MIXGCN_F32 ? 4 : 8;
    const int64_t total = n * ((cols + vec - 1) / vec);
    if (total == 0) return MIXGCN_OK;
    const dim3 grid((unsigned)ceil_div(total, kBlock));
    if (dtype == MIXGCN_F32)
        hipLaunchKernelGGL(apply_bitmap_kernel<MIXGCN_F32>, grid, dim3(kBlock), 0, s, X, ldx, n, cols,
                           bits, ldb);
    else
        hipLaunchKernelGGL(apply_bitmap_kernel<MIXGCN_BF16>, grid, dim3(kBlock), 0, s, X, ldx, n, cols,
                           bits, ldb);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

int launch_dropout_bitmap(uint64_t seed, int64_t n, int32_t cols, uint64_t threshold,
                          uint32_t* bits, int64_t ldb, hipStream_t s)
{
    const int64_t total = n * ldb;
    if (total == 0) return MIXGCN_OK;
    hipLaunchKernelGGL(dropout_bitmap_kernel, dim3((unsigned)ceil_div(total, kBlock)), dim3(kBlock),
                       0, s, seed, n, cols, threshold, bits, ldb);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

int launch_relu_bitmap(int dtype, const void* X, int64_t ldx, int64_t n, int32_t cols,
                       uint32_t* bits, int64_t ldb, hipStream_t s)
{
    if (n == 0) return MIXGCN_OK;
    // every word of a row up to ldb is written (zero past cols); a row takes whole lane groups,
    // and kBlock is a multiple of the group size, so a group never straddles a wavefront
    const int words = (int)ldb;
    const int es = dtype == MIXGCN_F32 ? 4 : 2;
    const int lanes_per_word = 32 / (16 / es);
    const int64_t total = n * (int64_t)words * lanes_per_word;
    const dim3 grid((unsigned)ceil_div(total, kBlock));
    if (dtype == MIXGCN_F32)
        hipLaunchKernelGGL(relu_bitmap_kernel<MIXGCN_F32>, grid, dim3(kBlock), 0, s, X, ldx, n, cols,
                           words, bits, ldb);
    else
        hipLaunchKernelGGL(relu_bitmap_kernel<MIXGCN_BF16>, grid, dim3(kBlock), 0, s, X, ldx, n,
                           cols, words, bits, ldb);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

int launch_aggregate(const mixgcn_graph* g, const Csr& m, const uint2* cv, int dtype, const void* H,
                     int64_t ldh, void* Z, int64_t ldz, int32_t c0, int32_t c1, int64_t r0,
                     int64_t r1, int epilogue, const uint32_t* mask, int64_t ldm, float* partials,
                     size_t partials_bytes, hipStream_t s, Timer* timer)
{
    if (dtype == MIXGCN_F32)
        return launch_dt<MIXGCN_F32>(g, m, cv, H, ldh, Z, ldz, c0, c1, r0, r1, epilogue, mask, ldm,
                                     partials, partials_bytes, s, timer);
    return launch_dt<MIXGCN_BF16>(g, m, cv, H, ldh, Z, ldz, c0, c1, r0, r1, epilogue, mask, ldm,
                                  partials, partials_bytes, s, timer);
}

// Upper bound of the row-piece scratch of one call on a graph with nnz stored entries: over
// both storage types and every pass width, the spans of the longest possible entry range times
// the two slots of a span.  A range is cut into spans of span_entries(); when that rule has
// halved the span at least once, the span count stays below 2 * 8192 / slices + 1.
size_t agg_scratch_bound(int64_t nnz)
{
    size_t best = 0;
    for (int vec = 4; vec <= 8; vec *= 2) {
        for (int w = 1; w <= kAggMaxPassCols; ++w) {
            Pass p;
            plan_pass(vec, 0, w, nnz, &p);
            const int lpr = g_aggregate_whole_rows ? p.gf : slice_lanes(p.gf);
            const int n_slices = (int)ceil_div(w, lpr * vec);
            const int64_t full = (int64_t)kBatchesPerSpan * (kWave / lpr);
            int64_t spans = ceil_div(nnz, full) + 1;  // a range need not start on a span boundary
            int64_t small = 2 * 8192 / n_slices + 2;
            // and no span is shorter than the kGroupNnz entries the span-start table resolves
            const int64_t most = ceil_div(nnz, kGroupNnz) + 1;
            if (small > most) small = most;
            if (small > spans) spans = small;
            const size_t bytes = (size_t)spans * 2 * p.gf * vec * sizeof(float);
            best = bytes > best ? bytes : best;
        }
    }
    return best;
}

// Row-piece scratch for the entry point that may not allocate: a fixed array in device memory
// (every GPU the library runs on holds its own copy until the process ends).  Host code never
// uses the array's name as an address: the device address is looked up once per device, with
// that device current, and kept.
constexpr size_t kStaticAggBytes = (size_t)64 << 20;
static __device__ __align__(256) float scratch[kStaticAggBytes / sizeof(float)];

namespace {
constexpr int kStaticDevices = 16;
float* g_static_ptr[kStaticDevices] = {};
std::mutex g_static_mu;
}  // namespace

int static_agg_scratch(float** p, size_t* bytes)
{
    int dev = 0;
    MIXGCN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStaticDevices) return fail(MIXGCN_EINVAL, "aggregate_static: device index");
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
        void* q = nullptr;
        MIXGCN_HIP_TRY(hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)));
        if (!q) return fail(MIXGCN_EHIP, "aggregate_static: no device address for the scratch array");
        g_static_ptr[dev] = reinterpret_cast<float*>(q);
    }
    *p = g_static_ptr[dev];
    *bytes = kStaticAggBytes;
    return MIXGCN_OK;
}

}  // namespace mixgcn
