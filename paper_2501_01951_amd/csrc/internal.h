// Internal declarations shared by the HIP sources of libmixgcn (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>
#include <string>
#include <vector>

#include "mixgcn.h"

namespace mixgcn {

// ---- error plumbing ---------------------------------------------------------------------------
void set_error(const std::string& msg);
int fail(int code, const std::string& msg);

#define MIXGCN_HIP_TRY(expr)                                                                  \
    do {                                                                                      \
        hipError_t _e = (expr);                                                               \
        if (_e != hipSuccess)                                                                 \
            return ::mixgcn::fail(_e == hipErrorOutOfMemory ? MIXGCN_ENOMEM : MIXGCN_EHIP,    \
                                  std::string(#expr) + ": " + hipGetErrorString(_e));         \
    } while (0)

#define MIXGCN_TRY(expr)         \
    do {                         \
        int _rc = (expr);        \
        if (_rc != MIXGCN_OK) return _rc; \
    } while (0)

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- graph ------------------------------------------------------------------------------------
// Granularity (in stored entries) of the table that maps an entry index to its row.
constexpr int kGroupNnz = 256;
// Padding of the kernel's entry array beyond nnz: the widest span one wavefront walks plus the
// prefetch distance of its software pipeline.
constexpr int kEntryPad = 8192;
// Bits of an entry's column word that are not part of the column index.
constexpr uint32_t kEntryEndBit = 0x80000000u;  // last stored entry of its row
constexpr uint32_t kEntryColMask = 0x3FFFFFFFu;

// Widest pass of the aggregation kernel in columns (fp32 and bf16 alike), and the bytes of row
// pieces one call can need on a graph with `nnz` stored entries, whatever its ranges.
constexpr int kAggMaxPassCols = 256;
extern int g_aggregate_whole_rows;  // measurement aid, see mixgcn_set_aggregate_whole_rows
size_t agg_scratch_bound(int64_t nnz);
size_t agg_scratch_need(int dtype, int32_t n_cols, int64_t e0, int64_t e1);

constexpr int kAggSlots = 16;
struct AggSlot {
    float* p = nullptr;
    hipStream_t stream = nullptr;
    bool bound = false;      // `stream` is meaningful (the null stream is a valid owner)
    uint64_t last_use = 0;
};

struct Csr {
    int64_t nnz = 0;
    int64_t nnz_padded = 0;          // allocation length of cv
    int64_t n_groups = 0;            // ceil(nnz / kGroupNnz)
    int64_t* rowptr = nullptr;       // [n + 1]
    uint32_t* col = nullptr;         // [nnz]  (public form: plain ascending columns)
    float* val = nullptr;            // [nnz]  (public form)
    // The aggregation kernel's form: entry e = { col | end-of-row mark, val bits }, zero padded.
    uint2* cv = nullptr;             // [nnz_padded]
    // Values of the TRANSPOSED matrix on this same pattern (symmetrised graph whose weights are
    // not symmetric, i.e. the mean mode); null otherwise.
    uint2* cv_t = nullptr;           // [nnz_padded]
    float* val_t = nullptr;          // [nnz]
    uint32_t* grp_row = nullptr;     // [n_groups + 1] row that holds entry g * kGroupNnz
    std::vector<int64_t> h_rowptr;   // host copy of rowptr
    bool has_empty_rows = false;
};

}  // namespace mixgcn

struct mixgcn_graph {
    uint32_t n = 0;
    uint32_t flags = 0;
    int device = 0;
    bool normalized = false;
    int norm_mode = 0;           // MIXGCN_NORM_* of the last normalisation
    bool has_transpose = false;  // a separate transpose CSR is stored in `tr`
    mixgcn::Csr fwd;
    mixgcn::Csr tr;
    uint32_t* deg = nullptr;
    float* dinv = nullptr;
    // Scratch of the aggregation kernels (pieces of the rows that cross span boundaries).  A
    // slot is bound to the stream that first asks for one and stays with it, so calls on one
    // stream share a slot (stream order keeps them apart) and calls on different streams never
    // do.  Every slot has the same size, fixed by mixgcn_normalize from the entry count (enough
    // for any row and column range); slot 0 is allocated there, further slots when a further
    // stream first aggregates this graph or ahead of time by mixgcn_graph_reserve_streams.
    mutable mixgcn::AggSlot agg_slots[mixgcn::kAggSlots];
    mutable std::mutex agg_mu;
    mutable uint64_t agg_tick = 0;
    size_t agg_slot_bytes = 0;
    // max |u - v| over the stored entries, computed on first use by the cross-layer pipeline
    mutable int64_t bandwidth = -1;
};

namespace mixgcn {

// Optional per-launch timing with HIP events recorded on the stream of the launch.
enum TimerKind {
    kTimeAggG4 = 0,  // aggregation main kernel by lane-group size: 4, 8, 16, 32, 64
    kTimeAggG8,
    kTimeAggG16,
    kTimeAggG32,
    kTimeAggG64,
    kTimeUpdateFwd,
    kTimeUpdateDgrad,
    kTimeUpdateWgrad,
    kTimeKinds
};

struct Timer {
    struct Rec {
        hipEvent_t a = nullptr, b = nullptr;
        int kind = 0;
    };
    bool enabled = false;
    std::vector<Rec> recs;
    size_t used = 0;
    int begin(int kind, hipStream_t s);
    int end(hipStream_t s);
    void reset() { used = 0; }
    void destroy();
};

}  // namespace mixgcn

struct mixgcn_pipeline {
    mixgcn::Timer timer;
    hipStream_t primary = nullptr;
    hipStream_t secondary = nullptr;
    std::vector<hipEvent_t> events;
    hipEvent_t ev_start = nullptr;
    hipEvent_t ev_done = nullptr;
};

namespace mixgcn {

// ---- device primitives (scan.hip, sort.hip) ---------------------------------------------------
// Exclusive prefix sum of n uint32 counts into uint64 offsets; total (optional, device) gets
// the sum.  tmp must hold scan_tmp_bytes(n).
size_t scan_tmp_bytes(int64_t n);
int exclusive_scan_u32_to_u64(const uint32_t* in, uint64_t* out, int64_t n, uint64_t* total,
                              void* tmp, hipStream_t s);

// Stable LSD radix sort of 64-bit keys on bits [0, n_bits).  Result ends in *sorted (either
// keys or alt).  tmp must hold sort_tmp_bytes(n).
size_t sort_tmp_bytes(int64_t n);
int radix_sort_u64(uint64_t* keys, uint64_t* alt, int64_t n, int n_bits, uint64_t** sorted,
                   void* tmp, hipStream_t s);

// ---- scratch shared by entry points without a handle --------------------------------------------
int get_scratch(int which, size_t bytes, void** out);

// ---- kernels behind the entry points ----------------------------------------------------------
int csr_from_edges(const uint32_t* d_src, const uint32_t* d_dst, uint64_t n_edges, uint32_t n,
                   bool symmetrize, bool self_loops, bool transposed, Csr* out, hipStream_t s);
void csr_free(Csr* c);
int normalize_graph(mixgcn_graph* g, int mode, float eps, hipStream_t s);

// mask: optional bitmap applied to the written outputs (bit c % 32 of mask[r * ldm + c / 32])
// cv: the entry array to walk (m.cv, or m.cv_t for the transpose of a symmetrised graph with
// unsymmetric weights); epilogue: MIXGCN_EPI_* flags
// partials / partials_bytes: scratch for the row pieces (device); a call that would need more is
// refused with MIXGCN_EINVAL before anything is launched
int launch_aggregate(const mixgcn_graph* g, const Csr& m, const uint2* cv, int dtype, const void* H,
                     int64_t ldh, void* Z, int64_t ldz, int32_t c0, int32_t c1, int64_t r0,
                     int64_t r1, int epilogue, const uint32_t* mask, int64_t ldm, float* partials,
                     size_t partials_bytes, hipStream_t s, Timer* timer);
// The aggregation scratch that lives in a fixed device array of the library (one copy per
// device), for the entry point that may not allocate.
int static_agg_scratch(float** p, size_t* bytes);

// bits[r * ldb + c / 32] bit c % 32 = X[r, c] > 0; every word of a row up to ldb is written
int launch_relu_bitmap(int dtype, const void* X, int64_t ldx, int64_t n, int32_t cols,
                       uint32_t* bits, int64_t ldb, hipStream_t s);
// X <- X (.) M (bitmap M); rows are padded to 16 bytes, so the last vector is in bounds
int launch_apply_bitmap(int dtype, void* X, int64_t ldx, int64_t n, int32_t cols,
                        const uint32_t* bits, int64_t ldb, hipStream_t s);
// bit of (r, c) = upper half of SplitMix64 output r * cols + c (seed) < threshold
int launch_dropout_bitmap(uint64_t seed, int64_t n, int32_t cols, uint64_t threshold,
                          uint32_t* bits, int64_t ldb, hipStream_t s);

// G <- G (.) 1[R > 0] in place (ReLU derivative taken from the stored activation R).
int launch_relu_mask(int dtype, void* G, int64_t ldg, const void* R, int64_t ldr, int64_t n,
                     int32_t m, hipStream_t s);

int launch_update(int op, int dtype, const void* A, int64_t lda, const void* B, int64_t ldb,
                  void* C, int64_t ldc, int64_t n, int32_t k, int32_t m, const void* R,
                  int64_t ldr, float beta, hipStream_t s, Timer* timer);

// bf16-stored features on the bf16 matrix cores (weights stay fp32, split into two bf16 terms)
int launch_update_bf16(int op, const uint16_t* A, int64_t lda, const void* B, int64_t ldb, void* C,
                       int64_t ldc, int64_t n, int32_t k, int32_t m, const uint16_t* R,
                       int64_t ldr, float beta, hipStream_t s, Timer* timer);

// fp32 features on the bf16 matrix cores (every operand as three bf16 terms, six partial products);
// chosen by mixgcn_set_update_arith, and only where update_split_applies says so
extern int g_update_arith;
bool update_split_applies(int op, int64_t lda, int64_t ldb, int64_t ldr, int64_t n, int32_t k,
                          int32_t m);
// W: the weights (forward, data gradient) or the upstream gradient (weight gradient, whose row
// count must be a multiple of 16)
int launch_update_split(int op, const float* A, int64_t lda, const float* W, int64_t ldw, float* C,
                        int64_t ldc, int64_t n, int32_t k, int32_t m, const float* R, int64_t ldr,
                        float beta, hipStream_t s, Timer* timer);

// dW = beta dW + sum of the slab partials P[slab][cells], in slab order in fp64
int launch_wgrad_reduce(const float* P, int64_t n_slabs, int64_t cells, int32_t m, float* dW,
                        int64_t ldw, float beta, hipStream_t s);

int launch_softmax_xent(int dtype, const void* logits, int64_t ldl, const int32_t* labels,
                        int64_t n, int32_t c, void* dlogits, int64_t ldd, double* loss,
                        hipStream_t s);

}  // namespace mixgcn
