// C ABI entry points: argument validation, object lifetime, the two-stream row-chunk
// pipeline that overlaps the aggregation of chunk k with the update of chunk k-1, and its
// cross-layer form
// (paper Sec. 3.2.2, fine-grain pipeline between the sparse and the dense half of a layer).
#include <cmath>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <new>

#include "internal.h"

namespace mixgcn {

static thread_local std::string g_last_error;

int g_update_arith = MIXGCN_ARITH_FP32;

void set_error(const std::string& msg) { g_last_error = msg; }
int fail(int code, const std::string& msg)
{
    g_last_error = msg;
    return code;
}

// Grow-only device scratch for entry points that carry no handle (split-K partials of the
// weight gradient, block partials of the loss).  One buffer per purpose and device.
namespace {
struct Scratch {
    void* p = nullptr;
    size_t bytes = 0;
};
constexpr int kMaxDevices = 16;
constexpr int kScratchKinds = 4;  // wgrad slabs, loss partials, split weights, small results
Scratch g_scratch[kMaxDevices][kScratchKinds];
std::mutex g_scratch_mu;
}  // namespace

int get_scratch(int which, size_t bytes, void** out)
{
    int dev = 0;
    MIXGCN_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices || which < 0 || which >= kScratchKinds)
        return fail(MIXGCN_EINVAL, "scratch: bad device or kind");
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    Scratch& sc = g_scratch[dev][which];
    if (bytes > sc.bytes) {
        if (sc.p) {
            MIXGCN_HIP_TRY(hipDeviceSynchronize());  // earlier kernels may still use the old buffer
            (void)hipFree(sc.p);
        }
        sc.p = nullptr;
        sc.bytes = 0;
        // The first allocation is large enough for the usual case, so that a later call (one
        // recorded into a HIP graph, say) does not have to grow it: the slab partials of the
        // weight gradient never exceed 1024 tiles of 128 x 128 fp32.
        const size_t floor_bytes = which == 0 ? ((size_t)64 << 20) : ((size_t)1 << 20);
        size_t want = bytes + bytes / 4 + 256;
        if (want < floor_bytes) want = floor_bytes;
        MIXGCN_HIP_TRY(hipMalloc(&sc.p, want));
        sc.bytes = want;
    }
    *out = sc.p;
    return MIXGCN_OK;
}

// Creates the per-device work buffers at their default sizes (a no-op once they exist).
static int reserve_default_scratch()
{
    void* unused = nullptr;
    for (int which = 0; which < kScratchKinds; ++which) MIXGCN_TRY(get_scratch(which, 1, &unused));
    return MIXGCN_OK;
}

// The row-piece scratch of graph g for work on `stream` (see mixgcn_graph::agg_slots).  The
// usual call finds the stream's slot and touches no HIP API.
static int acquire_agg_slot(const mixgcn_graph* g, hipStream_t stream, float** out)
{
    std::lock_guard<std::mutex> lock(g->agg_mu);
    AggSlot* slots = g->agg_slots;
    AggSlot* pick = nullptr;
    for (int i = 0; i < kAggSlots && !pick; ++i)
        if (slots[i].bound && slots[i].stream == stream) pick = &slots[i];
    if (!pick) {
        // a free slot, one that is already allocated first
        for (int i = 0; i < kAggSlots && !pick; ++i)
            if (!slots[i].bound && slots[i].p) pick = &slots[i];
        for (int i = 0; i < kAggSlots && !pick; ++i)
            if (!slots[i].bound) pick = &slots[i];
        if (!pick) {
            // every slot belongs to another stream: take over the one unused for longest, after
            // its work has finished (more streams than slots is not a case worth an event pool)
            pick = &slots[0];
            for (int i = 1; i < kAggSlots; ++i)
                if (slots[i].last_use < pick->last_use) pick = &slots[i];
            MIXGCN_HIP_TRY(hipDeviceSynchronize());
        }
        if (!pick->p) MIXGCN_HIP_TRY(hipMalloc((void**)&pick->p, g->agg_slot_bytes));
        pick->stream = stream;
        pick->bound = true;
    }
    pick->last_use = ++g->agg_tick;
    *out = pick->p;
    return MIXGCN_OK;
}

int Timer::begin(int kind, hipStream_t s)
{
    if (used == recs.size()) {
        Rec r;
        MIXGCN_HIP_TRY(hipEventCreate(&r.a));
        MIXGCN_HIP_TRY(hipEventCreate(&r.b));
        recs.push_back(r);
    }
    recs[used].kind = kind;
    MIXGCN_HIP_TRY(hipEventRecord(recs[used].a, s));
    return MIXGCN_OK;
}

int Timer::end(hipStream_t s)
{
    MIXGCN_HIP_TRY(hipEventRecord(recs[used].b, s));
    ++used;
    return MIXGCN_OK;
}

void Timer::destroy()
{
    for (Rec& r : recs) {
        if (r.a) (void)hipEventDestroy(r.a);
        if (r.b) (void)hipEventDestroy(r.b);
    }
    recs.clear();
    used = 0;
}

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int elem_size(int dtype) { return dtype == MIXGCN_BF16 ? 2 : 4; }

int check_matrix(const char* what, const void* p, int64_t ld, int64_t cols, int esize)
{
    if (!p) return fail(MIXGCN_EINVAL, std::string(what) + ": null pointer");
    if (!aligned16(p)) return fail(MIXGCN_EINVAL, std::string(what) + ": not 16-byte aligned");
    if (ld < cols) return fail(MIXGCN_EINVAL, std::string(what) + ": ld < columns");
    if ((ld * esize) % 16 != 0)
        return fail(MIXGCN_EINVAL, std::string(what) + ": ld * sizeof(element) not a multiple of 16");
    return MIXGCN_OK;
}

}  // namespace
}  // namespace mixgcn

using namespace mixgcn;

extern "C" {

int mixgcn_version(void) { return MIXGCN_VERSION; }

const char* mixgcn_last_error(void) { return g_last_error.c_str(); }

const char* mixgcn_strerror(int code)
{
    switch (code) {
    case MIXGCN_OK: return "ok";
    case MIXGCN_EINVAL: return "invalid argument";
    case MIXGCN_ENOMEM: return "out of memory";
    case MIXGCN_EHIP: return "HIP runtime error";
    case MIXGCN_ESTATE: return "call order violated";
    case MIXGCN_EUNSUPPORTED: return "not supported by this build";
    default: return "unknown error";
    }
}

int mixgcn_build_csr(const uint32_t* src, const uint32_t* dst, uint64_t n_edges, uint32_t n_nodes,
                     uint32_t flags, void* stream, mixgcn_graph** out)
{
    if (!out) return fail(MIXGCN_EINVAL, "build_csr: out is null");
    *out = nullptr;
    if (n_nodes == 0) return fail(MIXGCN_EINVAL, "build_csr: n_nodes == 0");
    if (n_nodes > 0x40000000u) return fail(MIXGCN_EINVAL, "build_csr: n_nodes > 2^30");
    if (n_edges > 0 && (!src || !dst)) return fail(MIXGCN_EINVAL, "build_csr: null edge list");
    if (n_edges > (1ull << 40)) return fail(MIXGCN_EINVAL, "build_csr: n_edges too large");
    if (flags & ~(uint32_t)(MIXGCN_SYMMETRIZE | MIXGCN_ADD_SELF_LOOPS | MIXGCN_BUILD_TRANSPOSE |
                            MIXGCN_INPUT_ON_HOST))
        return fail(MIXGCN_EINVAL, "build_csr: unknown flag");
    hipStream_t s = (hipStream_t)stream;
    const bool sym = flags & MIXGCN_SYMMETRIZE, loops = flags & MIXGCN_ADD_SELF_LOOPS;

    uint32_t* d_src = nullptr;
    uint32_t* d_dst = nullptr;
    const uint32_t* use_src = src;
    const uint32_t* use_dst = dst;
    int rc = MIXGCN_OK;
    mixgcn_graph* g = new (std::nothrow) mixgcn_graph();
    if (!g) return fail(MIXGCN_ENOMEM, "build_csr: host allocation failed");
    do {
        if (hipGetDevice(&g->device) != hipSuccess) { rc = fail(MIXGCN_EHIP, "hipGetDevice"); break; }
        if ((flags & MIXGCN_INPUT_ON_HOST) && n_edges > 0) {
            if (hipMalloc((void**)&d_src, n_edges * 4) != hipSuccess ||
                hipMalloc((void**)&d_dst, n_edges * 4) != hipSuccess) {
                rc = fail(MIXGCN_ENOMEM, "build_csr: staging the host edge list");
                break;
            }
            if (hipMemcpy(d_src, src, n_edges * 4, hipMemcpyHostToDevice) != hipSuccess ||
                hipMemcpy(d_dst, dst, n_edges * 4, hipMemcpyHostToDevice) != hipSuccess) {
                rc = fail(MIXGCN_EHIP, "build_csr: copying the host edge list");
                break;
            }
            use_src = d_src;
            use_dst = d_dst;
        }
        g->n = n_nodes;
        g->flags = flags;
        rc = csr_from_edges(use_src, use_dst, n_edges, n_nodes, sym, loops, false, &g->fwd, s);
        if (rc != MIXGCN_OK) break;
        if ((flags & MIXGCN_BUILD_TRANSPOSE) && !sym) {
            rc = csr_from_edges(use_src, use_dst, n_edges, n_nodes, false, loops, true, &g->tr, s);
            if (rc != MIXGCN_OK) break;
            g->has_transpose = true;
        }
    } while (0);
    if (d_src) (void)hipFree(d_src);
    if (d_dst) (void)hipFree(d_dst);
    if (rc != MIXGCN_OK) {
        mixgcn_graph_free(g);
        return rc;
    }
    *out = g;
    return MIXGCN_OK;
}

int mixgcn_graph_free(mixgcn_graph* g)
{
    if (!g) return MIXGCN_OK;
    csr_free(&g->fwd);
    csr_free(&g->tr);
    if (g->deg) (void)hipFree(g->deg);
    if (g->dinv) (void)hipFree(g->dinv);
    for (AggSlot& slot : g->agg_slots)
        if (slot.p) (void)hipFree(slot.p);
    delete g;
    return MIXGCN_OK;
}

int mixgcn_normalize(mixgcn_graph* g, int mode, void* stream)
{
    if (!g) return fail(MIXGCN_EINVAL, "normalize: graph is null");
    return mixgcn_normalize_mode(g, mode, 0.f, stream);
}

int mixgcn_normalize_mode(mixgcn_graph* g, int mode, float eps, void* stream)
{
    if (!g) return fail(MIXGCN_EINVAL, "normalize: graph is null");
    if (mode != MIXGCN_NORM_SYM && mode != MIXGCN_NORM_MEAN && mode != MIXGCN_NORM_SUM)
        return fail(MIXGCN_EINVAL, "normalize: unknown mode");
    if (!(eps == eps) || fabsf(eps) > 3.0e38f) return fail(MIXGCN_EINVAL, "normalize: eps");
    MIXGCN_TRY(normalize_graph(g, mode, mode == MIXGCN_NORM_SUM ? eps : 0.f, (hipStream_t)stream));
    // the row-piece scratch of the aggregation: sized once from the entry count, first slot here
    if (!g->agg_slot_bytes) g->agg_slot_bytes = agg_scratch_bound(g->fwd.nnz);
    if (!g->agg_slots[0].p)
        MIXGCN_HIP_TRY(hipMalloc((void**)&g->agg_slots[0].p, g->agg_slot_bytes));
    return MIXGCN_OK;
}

int mixgcn_graph_reserve_streams(mixgcn_graph* g, int32_t n_streams)
{
    if (!g) return fail(MIXGCN_EINVAL, "graph_reserve_streams: graph is null");
    if (!g->normalized) return fail(MIXGCN_ESTATE, "graph_reserve_streams: call mixgcn_normalize first");
    if (n_streams < 1 || n_streams > kAggSlots)
        return fail(MIXGCN_EINVAL, "graph_reserve_streams: between 1 and 16 streams");
    std::lock_guard<std::mutex> lock(g->agg_mu);
    int ready = 0, free_slots = 0;
    for (const AggSlot& slot : g->agg_slots) {
        if (slot.bound) continue;
        ++free_slots;
        if (slot.p) ++ready;
    }
    if (free_slots < n_streams)
        return fail(MIXGCN_EINVAL, "graph_reserve_streams: fewer slots than that are unowned");
    for (int i = 0; i < kAggSlots && ready < n_streams; ++i) {
        AggSlot& slot = g->agg_slots[i];
        if (slot.bound || slot.p) continue;
        MIXGCN_HIP_TRY(hipMalloc((void**)&slot.p, g->agg_slot_bytes));
        ++ready;
    }
    return MIXGCN_OK;
}

int64_t mixgcn_aggregate_scratch_bytes(int64_t nnz)
{
    if (nnz < 0) return 0;
    return (int64_t)agg_scratch_bound(nnz);
}

int64_t mixgcn_aggregate_scratch_need(int dtype, int32_t n_cols, int64_t entry_begin,
                                      int64_t entry_end)
{
    if ((dtype != MIXGCN_F32 && dtype != MIXGCN_BF16) || n_cols < 0 || entry_begin < 0 ||
        entry_end < entry_begin)
        return -1;
    return (int64_t)agg_scratch_need(dtype, n_cols, entry_begin, entry_end);
}

int mixgcn_graph_info(const mixgcn_graph* g, mixgcn_graph_view* out)
{
    if (!g || !out) return fail(MIXGCN_EINVAL, "graph_info: null argument");
    std::memset(out, 0, sizeof(*out));
    out->n_nodes = g->n;
    out->flags = g->flags;
    out->nnz = g->fwd.nnz;
    out->rowptr = g->fwd.rowptr;
    out->col = g->fwd.col;
    out->val = g->normalized ? g->fwd.val : nullptr;
    out->deg = g->normalized ? g->deg : nullptr;
    out->dinv = g->normalized ? g->dinv : nullptr;
    const mixgcn::Csr* t = nullptr;
    if (g->flags & MIXGCN_SYMMETRIZE) t = &g->fwd;
    else if (g->has_transpose) t = &g->tr;
    if (t) {
        out->t_rowptr = t->rowptr;
        out->t_col = t->col;
        const bool own = t == &g->fwd && g->norm_mode == MIXGCN_NORM_MEAN && t->val_t;
        out->t_val = g->normalized ? (own ? t->val_t : t->val) : nullptr;
    }
    return MIXGCN_OK;
}

static int aggregate_impl(const mixgcn_graph* g, int transpose, int dtype, const void* H,
                          int64_t ldh, void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                          int64_t row_begin, int64_t row_end, int epilogue, hipStream_t stream,
                          Timer* timer, const uint32_t* mask = nullptr, int64_t ld_mask = 0,
                          bool static_scratch = false)
{
    if (!g) return fail(MIXGCN_EINVAL, "aggregate: graph is null");
    if (!g->normalized) return fail(MIXGCN_ESTATE, "aggregate: call mixgcn_normalize first");
    if (dtype != MIXGCN_F32 && dtype != MIXGCN_BF16) return fail(MIXGCN_EINVAL, "aggregate: dtype");
    if (epilogue & ~(MIXGCN_EPI_RELU | MIXGCN_EPI_ACCUMULATE))
        return fail(MIXGCN_EINVAL, "aggregate: unknown epilogue flag");
    const int es = elem_size(dtype), vec = 16 / es;
    if (col_begin < 0 || col_end < col_begin) return fail(MIXGCN_EINVAL, "aggregate: column range");
    if (row_begin < 0 || row_end < row_begin || row_end > (int64_t)g->n)
        return fail(MIXGCN_EINVAL, "aggregate: row range");
    MIXGCN_TRY(check_matrix("aggregate: H", H, ldh, col_end, es));
    MIXGCN_TRY(check_matrix("aggregate: Z", Z, ldz, col_end, es));
    // The kernels read and write whole 16-byte groups of a row; a row pitch is a whole number of
    // groups (checked above), so the groups that hold [col_begin, col_end) lie inside the row, and
    // the stores leave out the elements of the first and last group that are outside the range.
    const int64_t up = ((int64_t)col_end + vec - 1) / vec * vec;
    {
        const char* h0 = (const char*)H;
        const char* h1 = h0 + (size_t)g->n * ldh * es;
        const char* z0 = (const char*)Z;
        const char* z1 = z0 + (size_t)g->n * ldz * es;
        if (h0 < z1 && z0 < h1) {
            // Two column blocks of one row-major buffer (same pitch) may interleave: the
            // columns [0, up) seen from H and from Z must be disjoint within a row.
            const int64_t pitch = ldh * es;
            int64_t shift = ((z0 - h0) % pitch + pitch) % pitch;
            const bool disjoint = ldh == ldz && shift >= up * es && shift + up * es <= pitch;
            if (!disjoint) return fail(MIXGCN_EINVAL, "aggregate: H and Z overlap");
        }
    }
    const mixgcn::Csr* m = &g->fwd;
    const uint2* cv = g->fwd.cv;
    if (transpose) {
        if (g->flags & MIXGCN_SYMMETRIZE) {
            if (g->norm_mode == MIXGCN_NORM_MEAN) cv = g->fwd.cv_t;
        } else {
            if (!g->has_transpose)
                return fail(MIXGCN_ESTATE, "aggregate: transpose needs MIXGCN_BUILD_TRANSPOSE");
            m = &g->tr;
            cv = g->tr.cv;
        }
    }
    if (!cv) return fail(MIXGCN_ESTATE, "aggregate: values of the transpose are missing");
    if (mask && ld_mask < ((int64_t)col_end + 31) / 32)
        return fail(MIXGCN_EINVAL, "aggregate: ld_mask shorter than ceil(col_end / 32) words");
    if (row_end == row_begin || col_end == col_begin) return MIXGCN_OK;
    float* partials = nullptr;
    size_t partials_bytes = g->agg_slot_bytes;
    if (static_scratch) MIXGCN_TRY(static_agg_scratch(&partials, &partials_bytes));
    else MIXGCN_TRY(acquire_agg_slot(g, stream, &partials));
    return launch_aggregate(g, *m, cv, dtype, H, ldh, Z, ldz, col_begin, col_end, row_begin,
                            row_end, epilogue, mask, ld_mask, partials, partials_bytes, stream,
                            timer);
}

int mixgcn_aggregate(const mixgcn_graph* g, int transpose, int dtype, const void* H, int64_t ldh,
                     void* Z, int64_t ldz, int32_t col_begin, int32_t col_end, int64_t row_begin,
                     int64_t row_end, void* stream)
{
    return aggregate_impl(g, transpose, dtype, H, ldh, Z, ldz, col_begin, col_end, row_begin,
                          row_end, 0, (hipStream_t)stream, nullptr);
}

int mixgcn_aggregate_static(const mixgcn_graph* g, int transpose, int dtype, const void* H,
                            int64_t ldh, void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                            int64_t row_begin, int64_t row_end, void* stream)
{
    return aggregate_impl(g, transpose, dtype, H, ldh, Z, ldz, col_begin, col_end, row_begin,
                          row_end, 0, (hipStream_t)stream, nullptr, nullptr, 0, true);
}

int mixgcn_aggregate_ex(const mixgcn_graph* g, int transpose, int dtype, const void* H, int64_t ldh,
                        void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                        int64_t row_begin, int64_t row_end, int epilogue, void* stream)
{
    return aggregate_impl(g, transpose, dtype, H, ldh, Z, ldz, col_begin, col_end, row_begin,
                          row_end, epilogue, (hipStream_t)stream, nullptr);
}

int mixgcn_aggregate_masked(const mixgcn_graph* g, int transpose, int dtype, const void* H,
                            int64_t ldh, void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                            int64_t row_begin, int64_t row_end, const uint32_t* mask,
                            int64_t ld_mask, void* stream)
{
    if (!mask) return fail(MIXGCN_EINVAL, "aggregate_masked: mask is null");
    return aggregate_impl(g, transpose, dtype, H, ldh, Z, ldz, col_begin, col_end, row_begin,
                          row_end, 0, (hipStream_t)stream, nullptr, mask, ld_mask);
}

int mixgcn_relu_bitmap(int dtype, const void* X, int64_t ldx, int64_t n_rows, int32_t n_cols,
                       uint32_t* mask, int64_t ld_mask, void* stream)
{
    if (dtype != MIXGCN_F32 && dtype != MIXGCN_BF16)
        return fail(MIXGCN_EINVAL, "relu_bitmap: dtype");
    if (n_rows < 0 || n_cols <= 0) return fail(MIXGCN_EINVAL, "relu_bitmap: sizes");
    if (!mask) return fail(MIXGCN_EINVAL, "relu_bitmap: null pointer");
    MIXGCN_TRY(check_matrix("relu_bitmap: X", X, ldx, n_cols, elem_size(dtype)));
    if (ld_mask < ((int64_t)n_cols + 31) / 32)
        return fail(MIXGCN_EINVAL, "relu_bitmap: ld_mask shorter than ceil(n_cols / 32) words");
    return launch_relu_bitmap(dtype, X, ldx, n_rows, n_cols, mask, ld_mask, (hipStream_t)stream);
}

static int update_impl(int op, int dtype, const void* A, int64_t lda, const void* B, int64_t ldb,
                       void* C, int64_t ldc, int64_t n_rows, int32_t k, int32_t m,
                       const void* relu_ref, int64_t ldr, float beta, hipStream_t stream,
                       Timer* timer)
{
    if (op < MIXGCN_OP_FWD || op > MIXGCN_OP_WGRAD) return fail(MIXGCN_EINVAL, "update: op");
    if (dtype != MIXGCN_F32 && dtype != MIXGCN_BF16) return fail(MIXGCN_EINVAL, "update: dtype");
    if (n_rows < 0 || k <= 0 || m <= 0) return fail(MIXGCN_EINVAL, "update: sizes");
    if (beta != 0.f && beta != 1.f) return fail(MIXGCN_EINVAL, "update: beta must be 0 or 1");
    const int es = elem_size(dtype);
    switch (op) {
    case MIXGCN_OP_FWD:
    case MIXGCN_OP_FWD_RELU:
        MIXGCN_TRY(check_matrix("update: A", A, lda, k, es));
        MIXGCN_TRY(check_matrix("update: B", B, ldb, m, 4));
        MIXGCN_TRY(check_matrix("update: C", C, ldc, m, es));
        break;
    case MIXGCN_OP_DGRAD:
        MIXGCN_TRY(check_matrix("update: A", A, lda, m, es));
        MIXGCN_TRY(check_matrix("update: B", B, ldb, m, 4));
        MIXGCN_TRY(check_matrix("update: C", C, ldc, k, es));
        if (relu_ref) MIXGCN_TRY(check_matrix("update: relu_ref", relu_ref, ldr, m, es));
        break;
    default:
        MIXGCN_TRY(check_matrix("update: A", A, lda, k, es));
        MIXGCN_TRY(check_matrix("update: B", B, ldb, m, es));
        MIXGCN_TRY(check_matrix("update: C", C, ldc, m, 4));
        if (relu_ref) MIXGCN_TRY(check_matrix("update: relu_ref", relu_ref, ldr, m, es));
        break;
    }
    return launch_update(op, dtype, A, lda, B, ldb, C, ldc, n_rows, k, m, relu_ref,
                         ldr, beta, stream, timer);
}

int mixgcn_apply_bitmap(int dtype, void* X, int64_t ldx, int64_t n_rows, int32_t n_cols,
                        const uint32_t* mask, int64_t ld_mask, void* stream)
{
    if (dtype != MIXGCN_F32 && dtype != MIXGCN_BF16)
        return fail(MIXGCN_EINVAL, "apply_bitmap: dtype");
    if (n_rows < 0 || n_cols <= 0) return fail(MIXGCN_EINVAL, "apply_bitmap: sizes");
    if (!mask) return fail(MIXGCN_EINVAL, "apply_bitmap: null pointer");
    MIXGCN_TRY(check_matrix("apply_bitmap: X", X, ldx, n_cols, elem_size(dtype)));
    if (ld_mask < ((int64_t)n_cols + 31) / 32)
        return fail(MIXGCN_EINVAL, "apply_bitmap: ld_mask shorter than ceil(n_cols / 32) words");
    return launch_apply_bitmap(dtype, X, ldx, n_rows, n_cols, mask, ld_mask, (hipStream_t)stream);
}

int mixgcn_dropout_bitmap(uint64_t seed, int64_t n_rows, int32_t n_cols, double keep_probability,
                          uint32_t* mask, int64_t ld_mask, void* stream)
{
    if (n_rows < 0 || n_cols <= 0) return fail(MIXGCN_EINVAL, "dropout_bitmap: sizes");
    if (!mask) return fail(MIXGCN_EINVAL, "dropout_bitmap: null pointer");
    if (!(keep_probability >= 0.0 && keep_probability <= 1.0))
        return fail(MIXGCN_EINVAL, "dropout_bitmap: keep_probability outside [0, 1]");
    if (ld_mask < ((int64_t)n_cols + 31) / 32)
        return fail(MIXGCN_EINVAL, "dropout_bitmap: ld_mask shorter than ceil(n_cols / 32) words");
    if (n_rows > 0 && (uint64_t)n_rows > (1ull << 62) / (uint64_t)n_cols)
        return fail(MIXGCN_EINVAL, "dropout_bitmap: n_rows * n_cols too large");
    const uint64_t threshold = (uint64_t)(keep_probability * 4294967296.0);
    return launch_dropout_bitmap(seed, n_rows, n_cols, threshold, mask, ld_mask,
                                 (hipStream_t)stream);
}

int mixgcn_update(int op, int dtype, const void* A, int64_t lda, const void* B, int64_t ldb,
                  void* C, int64_t ldc, int64_t n_rows, int32_t k, int32_t m,
                  const void* relu_ref, int64_t ldr, float beta, void* stream)
{
    return update_impl(op, dtype, A, lda, B, ldb, C, ldc, n_rows, k, m, relu_ref, ldr, beta,
                       (hipStream_t)stream, nullptr);
}

int mixgcn_set_update_arith(int mode)
{
    if (mode != MIXGCN_ARITH_FP32 && mode != MIXGCN_ARITH_BF16X3)
        return fail(MIXGCN_EINVAL, "set_update_arith: unknown mode");
    g_update_arith = mode;
    return MIXGCN_OK;
}

int mixgcn_set_aggregate_whole_rows(int on)
{
    g_aggregate_whole_rows = on ? 1 : 0;
    return MIXGCN_OK;
}

int mixgcn_softmax_xent(int dtype, const void* logits, int64_t ldl, const int32_t* labels,
                        int64_t n, int32_t n_classes, void* dlogits, int64_t ldd, double* loss,
                        void* stream)
{
    if (dtype != MIXGCN_F32 && dtype != MIXGCN_BF16) return fail(MIXGCN_EINVAL, "softmax_xent: dtype");
    if (!logits || !labels || !dlogits || !loss) return fail(MIXGCN_EINVAL, "softmax_xent: null");
    if (n <= 0 || n_classes <= 0 || ldl < n_classes || ldd < n_classes)
        return fail(MIXGCN_EINVAL, "softmax_xent: sizes");
    return launch_softmax_xent(dtype, logits, ldl, labels, n, n_classes, dlogits, ldd, loss,
                               (hipStream_t)stream);
}

int mixgcn_stream_create_cu_subset(int lo, int hi, int groups, void** stream)
{
    if (!stream) return fail(MIXGCN_EINVAL, "stream_create_cu_subset: null");
    *stream = nullptr;
    if (groups < 1 || groups > 8 || lo < 0 || hi > groups || lo >= hi)
        return fail(MIXGCN_EINVAL, "stream_create_cu_subset: need 0 <= lo < hi <= groups <= 8");
    int dev = 0, n_cu = 0;
    MIXGCN_HIP_TRY(hipGetDevice(&dev));
    MIXGCN_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
    std::vector<uint32_t> mask((size_t)(n_cu + 31) / 32, 0u);
    // CU c is enabled iff (c / 8) % groups lies in [lo, hi): blocks of 8 consecutive CU indices
    // alternate between the subsets, which selects the same share of every XCD whether the
    // runtime numbers the CUs XCD by XCD or round-robin across the XCDs.
    for (int c = 0; c < n_cu; ++c) {
        const int gsel = (c / 8) % groups;
        if (gsel >= lo && gsel < hi) mask[(size_t)c / 32] |= 1u << (c % 32);
    }
    hipStream_t s = nullptr;
    MIXGCN_HIP_TRY(hipExtStreamCreateWithCUMask(&s, (uint32_t)mask.size(), mask.data()));
    *stream = (void*)s;
    return MIXGCN_OK;
}

int mixgcn_stream_destroy(void* stream)
{
    if (!stream) return MIXGCN_OK;
    MIXGCN_HIP_TRY(hipStreamDestroy((hipStream_t)stream));
    return MIXGCN_OK;
}

int mixgcn_pipeline_create(void* primary_stream, void* secondary_stream, mixgcn_pipeline** out)
{
    if (!out) return fail(MIXGCN_EINVAL, "pipeline_create: out is null");
    *out = nullptr;
    mixgcn_pipeline* p = new (std::nothrow) mixgcn_pipeline();
    if (!p) return fail(MIXGCN_ENOMEM, "pipeline_create: host allocation failed");
    p->primary = (hipStream_t)primary_stream;
    p->secondary = (hipStream_t)secondary_stream;
    // the work buffers of the update products and of the loss exist from here on, so that the
    // first step of a pipeline allocates nothing
    {
        const int rc = reserve_default_scratch();
        if (rc != MIXGCN_OK) {
            delete p;
            return rc;
        }
    }
    if (hipEventCreateWithFlags(&p->ev_start, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&p->ev_done, hipEventDisableTiming) != hipSuccess) {
        mixgcn_pipeline_destroy(p);
        return fail(MIXGCN_EHIP, "pipeline_create: hipEventCreate");
    }
    *out = p;
    return MIXGCN_OK;
}

int mixgcn_pipeline_destroy(mixgcn_pipeline* p)
{
    if (!p) return MIXGCN_OK;
    for (hipEvent_t e : p->events) (void)hipEventDestroy(e);
    if (p->ev_start) (void)hipEventDestroy(p->ev_start);
    if (p->ev_done) (void)hipEventDestroy(p->ev_done);
    p->timer.destroy();
    delete p;
    return MIXGCN_OK;
}

int mixgcn_pipeline_timing(mixgcn_pipeline* p, int enable)
{
    if (!p) return fail(MIXGCN_EINVAL, "pipeline_timing: null pipeline");
    p->timer.enabled = enable != 0;
    p->timer.reset();
    return MIXGCN_OK;
}

int mixgcn_pipeline_timing_read(mixgcn_pipeline* p, int kind, double* total_ms, int64_t* launches)
{
    if (!p || !total_ms || !launches) return fail(MIXGCN_EINVAL, "pipeline_timing_read: null");
    if (kind < 0 || kind >= kTimeKinds) return fail(MIXGCN_EINVAL, "pipeline_timing_read: kind");
    MIXGCN_HIP_TRY(hipStreamSynchronize(p->primary));
    MIXGCN_HIP_TRY(hipStreamSynchronize(p->secondary));
    double sum = 0.0;
    int64_t cnt = 0;
    for (size_t i = 0; i < p->timer.used; ++i) {
        const Timer::Rec& r = p->timer.recs[i];
        if (r.kind != kind) continue;
        float ms = 0.f;
        MIXGCN_HIP_TRY(hipEventElapsedTime(&ms, r.a, r.b));
        sum += ms;
        ++cnt;
    }
    *total_ms = sum;
    *launches = cnt;
    return MIXGCN_OK;
}

}  // extern "C"

namespace {

int ensure_events(mixgcn_pipeline* p, size_t count)
{
    while (p->events.size() < count) {
        hipEvent_t e;
        MIXGCN_HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        p->events.push_back(e);
    }
    return MIXGCN_OK;
}

// Chunk boundaries: multiples of 128 rows (the update kernels' row tile), last chunk ragged.
int64_t chunk_bound(int64_t n, int n_chunks, int i)
{
    if (i >= n_chunks) return n;
    int64_t b = (n * i / n_chunks + 127) / 128 * 128;
    return b < n ? b : n;
}

int check_layer(const char* who, const mixgcn_graph* g, const mixgcn_layer_desc* d,
                const mixgcn_pipeline* p)
{
    if (!g || !d || !p) return fail(MIXGCN_EINVAL, std::string(who) + ": null argument");
    if (!g->normalized) return fail(MIXGCN_ESTATE, std::string(who) + ": graph not normalized");
    if (d->f_in <= 0 || d->f_out <= 0 || d->n_chunks <= 0 || d->n_chunks > 65536)
        return fail(MIXGCN_EINVAL, std::string(who) + ": bad layer sizes");
    if (d->dtype != MIXGCN_F32 && d->dtype != MIXGCN_BF16)
        return fail(MIXGCN_EINVAL, std::string(who) + ": dtype");
    if (d->order != MIXGCN_AGG_FIRST && d->order != MIXGCN_UPDATE_FIRST)
        return fail(MIXGCN_EINVAL, std::string(who) + ": order");
    return MIXGCN_OK;
}

}  // namespace

extern "C" {

int mixgcn_layer_fwd(const mixgcn_graph* g, const mixgcn_layer_desc* d, const void* H,
                     const float* W, void* Z, void* Hout, mixgcn_pipeline* p)
{
    MIXGCN_TRY(check_layer("layer_fwd", g, d, p));
    if (!H || !W || !Z || !Hout) return fail(MIXGCN_EINVAL, "layer_fwd: null tensor");
    const int64_t n = g->n;
    const int es = elem_size(d->dtype);
    const int op = d->relu ? MIXGCN_OP_FWD_RELU : MIXGCN_OP_FWD;
    const int nc = d->n_chunks;
    Timer* tm = p->timer.enabled ? &p->timer : nullptr;
    if (d->order == MIXGCN_UPDATE_FIRST) {
        // Z = H W on the dense stream, then Hout = sigma(A_hat Z): the gather needs all of Z
        MIXGCN_TRY(update_impl(MIXGCN_OP_FWD, d->dtype, H, d->ld_h, W, d->ld_w, Z, d->ld_z, n,
                               d->f_in, d->f_out, nullptr, 0, 0.f, p->primary, tm));
        return aggregate_impl(g, 0, d->dtype, Z, d->ld_z, Hout, d->ld_out, 0, d->f_out, 0, n,
                              d->relu, p->primary, tm);
    }
    if (nc == 1 || p->secondary == p->primary) {
        MIXGCN_TRY(aggregate_impl(g, 0, d->dtype, H, d->ld_h, Z, d->ld_z, 0, d->f_in, 0, n, 0,
                                  p->primary, tm));
        return update_impl(op, d->dtype, Z, d->ld_z, W, d->ld_w, Hout, d->ld_out, n, d->f_in,
                           d->f_out, nullptr, 0, 0.f, p->primary, tm);
    }
    MIXGCN_TRY(ensure_events(p, (size_t)nc));
    // the dense stream may not start before everything queued on the sparse stream so far
    MIXGCN_HIP_TRY(hipEventRecord(p->ev_start, p->primary));
    MIXGCN_HIP_TRY(hipStreamWaitEvent(p->secondary, p->ev_start, 0));
    for (int c = 0; c < nc; ++c) {
        const int64_t r0 = chunk_bound(n, nc, c), r1 = chunk_bound(n, nc, c + 1);
        if (r1 <= r0) continue;
        MIXGCN_TRY(aggregate_impl(g, 0, d->dtype, H, d->ld_h, Z, d->ld_z, 0, d->f_in, r0, r1, 0,
                                  p->primary, tm));
        MIXGCN_HIP_TRY(hipEventRecord(p->events[(size_t)c], p->primary));
        MIXGCN_HIP_TRY(hipStreamWaitEvent(p->secondary, p->events[(size_t)c], 0));
        const char* zc = (const char*)Z + (size_t)r0 * d->ld_z * es;
        char* oc = (char*)Hout + (size_t)r0 * d->ld_out * es;
        MIXGCN_TRY(update_impl(op, d->dtype, zc, d->ld_z, W, d->ld_w, oc, d->ld_out, r1 - r0,
                               d->f_in, d->f_out, nullptr, 0, 0.f, p->secondary, tm));
    }
    MIXGCN_HIP_TRY(hipEventRecord(p->ev_done, p->secondary));
    MIXGCN_HIP_TRY(hipStreamWaitEvent(p->primary, p->ev_done, 0));
    return MIXGCN_OK;
}

int mixgcn_layer_bwd(const mixgcn_graph* g, const mixgcn_layer_desc* d, const void* H, void* Z,
                     const void* Hout, const float* W, void* G, float* dW, void* dH,
                     mixgcn_pipeline* p)
{
    MIXGCN_TRY(check_layer("layer_bwd", g, d, p));
    if (!Z || !W || !G || !dW) return fail(MIXGCN_EINVAL, "layer_bwd: null tensor");
    if (d->relu && !Hout) return fail(MIXGCN_EINVAL, "layer_bwd: relu layer needs Hout");
    const int64_t n = g->n;
    const void* R = d->relu ? Hout : nullptr;
    Timer* tm = p->timer.enabled ? &p->timer : nullptr;
    if (d->order == MIXGCN_UPDATE_FIRST) {
        if (!H) return fail(MIXGCN_EINVAL, "layer_bwd: update-first layer needs H");
        if (R) MIXGCN_TRY(launch_relu_mask(d->dtype, G, d->ld_out, R, d->ld_out, n, d->f_out,
                                           p->primary));
        // dQ = A_hat^T dP into the workspace, then the two dense products
        MIXGCN_TRY(aggregate_impl(g, 1, d->dtype, G, d->ld_out, Z, d->ld_z, 0, d->f_out, 0, n, 0,
                                  p->primary, tm));
        MIXGCN_TRY(update_impl(MIXGCN_OP_WGRAD, d->dtype, H, d->ld_h, Z, d->ld_z, dW, d->ld_w, n,
                               d->f_in, d->f_out, nullptr, 0, 0.f, p->primary, tm));
        if (dH)
            MIXGCN_TRY(update_impl(MIXGCN_OP_DGRAD, d->dtype, Z, d->ld_z, W, d->ld_w, dH, d->ld_h, n,
                                   d->f_in, d->f_out, nullptr, 0, 0.f, p->primary, tm));
        return MIXGCN_OK;
    }
    const bool two = p->secondary != p->primary && d->n_chunks > 1;
    hipStream_t dense = two ? p->secondary : p->primary;
    if (two) {
        MIXGCN_HIP_TRY(hipEventRecord(p->ev_start, p->primary));
        MIXGCN_HIP_TRY(hipStreamWaitEvent(p->secondary, p->ev_start, 0));
    }
    // dW = Z^T dP must read Z before dZ overwrites it
    MIXGCN_TRY(update_impl(MIXGCN_OP_WGRAD, d->dtype, Z, d->ld_z, G, d->ld_out, dW, d->ld_w, n,
                           d->f_in, d->f_out, R, d->ld_out, 0.f, dense, tm));
    if (dH) {
        MIXGCN_TRY(update_impl(MIXGCN_OP_DGRAD, d->dtype, G, d->ld_out, W, d->ld_w, Z, d->ld_z, n,
                               d->f_in, d->f_out, R, d->ld_out, 0.f, dense, tm));
        if (two) {
            MIXGCN_HIP_TRY(hipEventRecord(p->ev_done, p->secondary));
            MIXGCN_HIP_TRY(hipStreamWaitEvent(p->primary, p->ev_done, 0));
        }
        MIXGCN_TRY(aggregate_impl(g, 1, d->dtype, Z, d->ld_z, dH, d->ld_h, 0, d->f_in, 0, n, 0,
                                  p->primary, tm));
    } else if (two) {
        MIXGCN_HIP_TRY(hipEventRecord(p->ev_done, p->secondary));
        MIXGCN_HIP_TRY(hipStreamWaitEvent(p->primary, p->ev_done, 0));
    }
    return MIXGCN_OK;
}

}  // extern "C"

namespace {

// One operation of a chain of layers, applied to the row chunks in order.  A windowed operation
// (an aggregation) reads rows [r0 - b, r1 + b) of what the operation before it wrote, any other
// only its own rows [r0, r1).
struct ChainOp {
    bool sparse;    // issued on the primary (sparse) stream, else on the secondary (dense) one
    bool windowed;
    std::function<int(int64_t r0, int64_t r1, hipStream_t s)> run;
};

// Chunks [first, last] of the producer that chunk c of a windowed consumer reads.
void chunk_window(int64_t n, int nc, int64_t b, int c, int* first, int* last)
{
    const int64_t r0 = chunk_bound(n, nc, c), r1 = chunk_bound(n, nc, c + 1);
    const int64_t lo = r0 - b > 0 ? r0 - b : 0;
    const int64_t hi = r1 + b < n ? r1 + b : n;  // exclusive
    int f = c, l = c;
    while (f > 0 && chunk_bound(n, nc, f) > lo) --f;
    while (l + 1 < nc && chunk_bound(n, nc, l + 1) < hi) ++l;
    *first = f;
    *last = l;
}

// Issues the chain operation by operation, chunk by chunk.  Both streams run their work in
// issue order, so a chunk only has to wait for the LAST chunk it reads of the operation before
// it, and only when that one runs on the other stream (Sec. 3.2.2: the first batch of the next
// aggregation starts as soon as the batches it depends on are there, not when the layer is).
int run_chain(const mixgcn_graph* g, mixgcn_pipeline* p, int nc, int64_t b,
              const std::vector<ChainOp>& ops)
{
    const int64_t n = g->n;
    const bool two = p->secondary != p->primary;
    MIXGCN_TRY(ensure_events(p, ops.size() * (size_t)nc));
    if (two) {
        MIXGCN_HIP_TRY(hipEventRecord(p->ev_start, p->primary));
        MIXGCN_HIP_TRY(hipStreamWaitEvent(p->secondary, p->ev_start, 0));
    }
    for (size_t k = 0; k < ops.size(); ++k) {
        const ChainOp& op = ops[k];
        hipStream_t s = (op.sparse || !two) ? p->primary : p->secondary;
        const bool cross = two && k > 0 && ops[k - 1].sparse != op.sparse;
        int waited = -1;  // highest chunk of the producer this stream already waits for
        for (int c = 0; c < nc; ++c) {
            const int64_t r0 = chunk_bound(n, nc, c), r1 = chunk_bound(n, nc, c + 1);
            if (cross) {
                int first = c, last = c;
                if (op.windowed) chunk_window(n, nc, b, c, &first, &last);
                if (last > waited) {
                    MIXGCN_HIP_TRY(hipStreamWaitEvent(s, p->events[(k - 1) * (size_t)nc + (size_t)last], 0));
                    waited = last;
                }
            }
            if (r1 > r0) MIXGCN_TRY(op.run(r0, r1, s));
            if (two) MIXGCN_HIP_TRY(hipEventRecord(p->events[k * (size_t)nc + (size_t)c], s));
        }
    }
    if (two) {
        MIXGCN_HIP_TRY(hipEventRecord(p->ev_done, p->secondary));
        MIXGCN_HIP_TRY(hipStreamWaitEvent(p->primary, p->ev_done, 0));
    }
    return MIXGCN_OK;
}

int check_chain(const char* who, const mixgcn_graph* g, int32_t n_layers,
                const mixgcn_layer_desc* d, int64_t bandwidth, const mixgcn_pipeline* p)
{
    if (n_layers <= 0 || n_layers > 1024) return fail(MIXGCN_EINVAL, std::string(who) + ": n_layers");
    for (int l = 0; l < n_layers; ++l) {
        MIXGCN_TRY(check_layer(who, g, d ? d + l : nullptr, p));
        if (d[l].n_chunks != d[0].n_chunks || d[l].dtype != d[0].dtype)
            return fail(MIXGCN_EINVAL, std::string(who) + ": layers differ in n_chunks or dtype");
        if (l > 0 && (d[l].f_in != d[l - 1].f_out || d[l].ld_h != d[l - 1].ld_out))
            return fail(MIXGCN_EINVAL, std::string(who) + ": layer input does not match the output before it");
    }
    if (bandwidth < 0) return fail(MIXGCN_EINVAL, std::string(who) + ": bandwidth");
    // the window must cover the graph as stored: a smaller one would let an aggregation read
    // rows that are not written yet
    if (g->bandwidth < 0) {
        int64_t bw = 0;
        MIXGCN_TRY(mixgcn_bandwidth(g, nullptr, &bw, p->primary));
        g->bandwidth = bw;
    }
    if (bandwidth < g->bandwidth)
        return fail(MIXGCN_EINVAL, std::string(who) + ": bandwidth is smaller than the graph's (" +
                                       std::to_string(g->bandwidth) + ")");
    return MIXGCN_OK;
}

inline const char* row_ptr(const void* base, int64_t r, int64_t ld, int es)
{
    return (const char*)base + (size_t)r * (size_t)ld * (size_t)es;
}
inline char* row_ptr(void* base, int64_t r, int64_t ld, int es)
{
    return (char*)base + (size_t)r * (size_t)ld * (size_t)es;
}

}  // namespace

extern "C" {

int mixgcn_pipeline_window(int64_t n_nodes, int32_t n_chunks, int64_t bandwidth, int32_t chunk,
                           int64_t* row_begin, int64_t* row_end, int32_t* first, int32_t* last)
{
    if (n_nodes < 0 || n_chunks <= 0 || bandwidth < 0 || chunk < 0 || chunk >= n_chunks)
        return fail(MIXGCN_EINVAL, "pipeline_window: arguments");
    if (row_begin) *row_begin = chunk_bound(n_nodes, n_chunks, chunk);
    if (row_end) *row_end = chunk_bound(n_nodes, n_chunks, chunk + 1);
    int f = chunk, l = chunk;
    chunk_window(n_nodes, n_chunks, bandwidth, chunk, &f, &l);
    if (first) *first = f;
    if (last) *last = l;
    return MIXGCN_OK;
}

int mixgcn_forward_pipelined(const mixgcn_graph* g, int32_t n_layers, const mixgcn_layer_desc* d,
                             const void* H0, const float* const* W, void* const* Z,
                             void* const* Hout, int64_t bandwidth, mixgcn_pipeline* p)
{
    MIXGCN_TRY(check_chain("forward_pipelined", g, n_layers, d, bandwidth, p));
    if (!H0 || !W || !Z || !Hout) return fail(MIXGCN_EINVAL, "forward_pipelined: null argument");
    for (int l = 0; l < n_layers; ++l)
        if (!W[l] || !Z[l] || !Hout[l]) return fail(MIXGCN_EINVAL, "forward_pipelined: null tensor");
    Timer* tm = p->timer.enabled ? &p->timer : nullptr;
    const int es = elem_size(d[0].dtype);
    std::vector<ChainOp> ops;
    for (int l = 0; l < n_layers; ++l) {
        const mixgcn_layer_desc L = d[l];
        const void* in = l == 0 ? H0 : Hout[l - 1];
        const float* w = W[l];
        void* z = Z[l];
        void* out = Hout[l];
        const int op = L.relu ? MIXGCN_OP_FWD_RELU : MIXGCN_OP_FWD;
        if (L.order == MIXGCN_AGG_FIRST) {
            ops.push_back({true, true, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               return aggregate_impl(g, 0, L.dtype, in, L.ld_h, z, L.ld_z, 0, L.f_in,
                                                     r0, r1, 0, s, tm);
                           }});
            ops.push_back({false, false, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               return update_impl(op, L.dtype, row_ptr(z, r0, L.ld_z, es), L.ld_z, w,
                                                  L.ld_w, row_ptr(out, r0, L.ld_out, es), L.ld_out,
                                                  r1 - r0, L.f_in, L.f_out, nullptr, 0, 0.f, s, tm);
                           }});
        } else {
            ops.push_back({false, false, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               return update_impl(MIXGCN_OP_FWD, L.dtype, row_ptr(in, r0, L.ld_h, es),
                                                  L.ld_h, w, L.ld_w, row_ptr(z, r0, L.ld_z, es),
                                                  L.ld_z, r1 - r0, L.f_in, L.f_out, nullptr, 0, 0.f,
                                                  s, tm);
                           }});
            ops.push_back({true, true, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               return aggregate_impl(g, 0, L.dtype, z, L.ld_z, out, L.ld_out, 0,
                                                     L.f_out, r0, r1, L.relu, s, tm);
                           }});
        }
    }
    return run_chain(g, p, d[0].n_chunks, bandwidth, ops);
}

int mixgcn_backward_pipelined(const mixgcn_graph* g, int32_t n_layers, const mixgcn_layer_desc* d,
                              const void* H0, void* const* Z, const void* const* Hout,
                              const float* const* W, void* const* G, float* const* dW, void* dH0,
                              int64_t bandwidth, mixgcn_pipeline* p)
{
    MIXGCN_TRY(check_chain("backward_pipelined", g, n_layers, d, bandwidth, p));
    if (!Z || !Hout || !W || !G || !dW) return fail(MIXGCN_EINVAL, "backward_pipelined: null argument");
    for (int l = 0; l < n_layers; ++l) {
        if (!Z[l] || !W[l] || !G[l] || !dW[l])
            return fail(MIXGCN_EINVAL, "backward_pipelined: null tensor");
        if (d[l].relu && !Hout[l]) return fail(MIXGCN_EINVAL, "backward_pipelined: relu layer needs Hout");
        if (d[l].order == MIXGCN_UPDATE_FIRST && !(l == 0 ? H0 : Hout[l - 1]))
            return fail(MIXGCN_EINVAL, "backward_pipelined: update-first layer needs its input");
    }
    Timer* tm = p->timer.enabled ? &p->timer : nullptr;
    const int es = elem_size(d[0].dtype);
    std::vector<ChainOp> ops;
    // first = 1 until the weight gradient of a layer has been started (beta = 0), one per layer
    auto started = std::make_shared<std::vector<char>>((size_t)n_layers, 0);
    for (int l = n_layers - 1; l >= 0; --l) {
        const mixgcn_layer_desc L = d[l];
        const void* in = l == 0 ? H0 : Hout[l - 1];
        const void* R = L.relu ? Hout[l] : nullptr;
        const float* w = W[l];
        void* z = Z[l];
        void* grad = G[l];
        float* dw = dW[l];
        void* dh = l == 0 ? dH0 : G[l - 1];
        if (L.order == MIXGCN_AGG_FIRST) {
            // dW += Z^T dP and dZ = dP W^T for the chunk (dZ over Z, after dW has read it)
            ops.push_back({false, false, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               const float beta = (*started)[(size_t)l] ? 1.f : 0.f;
                               (*started)[(size_t)l] = 1;
                               const void* rc = R ? row_ptr(R, r0, L.ld_out, es) : nullptr;
                               MIXGCN_TRY(update_impl(MIXGCN_OP_WGRAD, L.dtype,
                                                      row_ptr(z, r0, L.ld_z, es), L.ld_z,
                                                      row_ptr(grad, r0, L.ld_out, es), L.ld_out, dw,
                                                      L.ld_w, r1 - r0, L.f_in, L.f_out, rc, L.ld_out,
                                                      beta, s, tm));
                               if (!dh) return (int)MIXGCN_OK;
                               return update_impl(MIXGCN_OP_DGRAD, L.dtype,
                                                  row_ptr(grad, r0, L.ld_out, es), L.ld_out, w, L.ld_w,
                                                  row_ptr(z, r0, L.ld_z, es), L.ld_z, r1 - r0, L.f_in,
                                                  L.f_out, rc, L.ld_out, 0.f, s, tm);
                           }});
            if (dh)
                ops.push_back({true, true, [=](int64_t r0, int64_t r1, hipStream_t s) {
                                   return aggregate_impl(g, 1, L.dtype, z, L.ld_z, dh, L.ld_h, 0,
                                                         L.f_in, r0, r1, 0, s, tm);
                               }});
        } else {
            if (R)
                ops.push_back({false, false, [=](int64_t r0, int64_t r1, hipStream_t s) {
                                   return launch_relu_mask(L.dtype, row_ptr(grad, r0, L.ld_out, es),
                                                           L.ld_out, row_ptr(R, r0, L.ld_out, es),
                                                           L.ld_out, r1 - r0, L.f_out, s);
                               }});
            ops.push_back({true, true, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               return aggregate_impl(g, 1, L.dtype, grad, L.ld_out, z, L.ld_z, 0,
                                                     L.f_out, r0, r1, 0, s, tm);
                           }});
            ops.push_back({false, false, [=](int64_t r0, int64_t r1, hipStream_t s) {
                               const float beta = (*started)[(size_t)l] ? 1.f : 0.f;
                               (*started)[(size_t)l] = 1;
                               MIXGCN_TRY(update_impl(MIXGCN_OP_WGRAD, L.dtype,
                                                      row_ptr(in, r0, L.ld_h, es), L.ld_h,
                                                      row_ptr(z, r0, L.ld_z, es), L.ld_z, dw, L.ld_w,
                                                      r1 - r0, L.f_in, L.f_out, nullptr, 0, beta, s,
                                                      tm));
                               if (!dh) return (int)MIXGCN_OK;
                               return update_impl(MIXGCN_OP_DGRAD, L.dtype, row_ptr(z, r0, L.ld_z, es),
                                                  L.ld_z, w, L.ld_w, row_ptr(dh, r0, L.ld_h, es),
                                                  L.ld_h, r1 - r0, L.f_in, L.f_out, nullptr, 0, 0.f,
                                                  s, tm);
                           }});
        }
    }
    return run_chain(g, p, d[0].n_chunks, bandwidth, ops);
}

}  // extern "C"
