/*
 * mixgcn.h -- C ABI of the MI355X (gfx950) GCN layer path.
 *
 * One GPU's share of full-graph GCN training under the paper's mixture of parallelism
 * (Algorithm 2): neighbor aggregation  Z = A_hat H  over all nodes on a slice of feature
 * columns, node update  H' = sigma(Z W), and their backward passes, with the sparse and dense
 * halves overlapped on row chunks (Sec. 3.2.2, fine-grain pipeline).
 *
 * Conventions
 *  - Matrices are node x feature, row-major, with leading dimensions in ELEMENTS.  (The paper
 *    writes feature x node matrices; Eq. 3 with W here = the paper's W^T is H' = sigma(A_hat H W).)
 *  - Every pointer is a DEVICE pointer unless its comment says host.  The caller owns all
 *    tensors and streams; the library owns only mixgcn_graph / mixgcn_pipeline objects.
 *  - `stream` arguments are hipStream_t passed as void* (NULL = the default stream).  All work
 *    is asynchronous on that stream except where stated.
 *  - Base pointers must be 16-byte aligned and ld * sizeof(element) a multiple of 16.
 *  - Every call returns 0 on success or a negative MIXGCN_E* code; mixgcn_last_error() gives a
 *    thread-local message.  Bad arguments are rejected before anything is launched.
 *  - dtype: MIXGCN_F32 = fp32 storage and arithmetic; MIXGCN_BF16 = bf16 storage of every
 *    n x F feature tensor (inputs, aggregates, layer outputs including the logits, and the
 *    gradients of all of these) with fp32 accumulation; the weights, the A_hat values, the loss
 *    and dW stay fp32.
 */
#ifndef MIXGCN_H
#define MIXGCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIXGCN_VERSION 100

enum {
    MIXGCN_OK = 0,
    MIXGCN_EINVAL = -1,       /* bad argument (null, range, alignment, ld < columns ...) */
    MIXGCN_ENOMEM = -2,       /* device or host allocation failed */
    MIXGCN_EHIP = -3,         /* a HIP runtime call failed; message has hipGetErrorString */
    MIXGCN_ESTATE = -4,       /* call order violated (e.g. aggregate before normalize) */
    MIXGCN_EUNSUPPORTED = -5  /* valid request that this build does not implement */
};

/* mixgcn_build_csr flags */
enum {
    MIXGCN_SYMMETRIZE = 1,      /* also insert (v,u) for every input (u,v) */
    MIXGCN_ADD_SELF_LOOPS = 2,  /* A_tilde = A + I: one diagonal entry in every row */
    MIXGCN_BUILD_TRANSPOSE = 4, /* also keep the CSR of the transpose (needed for backward when
                                   SYMMETRIZE is not set; with SYMMETRIZE the matrix is its own
                                   transpose and nothing extra is stored) */
    MIXGCN_INPUT_ON_HOST = 8    /* src/dst are host pointers (copied synchronously) */
};

/* Aggregation matrices (mixgcn_normalize_mode).  SYM is the paper's GCN (Sec. 2.1); MEAN and
 * SUM are the neighbor aggregations of the two other architectures the paper evaluates (Sec. 4,
 * experimental setting: GraphSAGE and GIN), taken from the works it cites for them. */
enum {
    MIXGCN_NORM_SYM = 0,  /* A_hat = D^-1/2 A_tilde D^-1/2                                      */
    MIXGCN_NORM_MEAN = 1, /* A_hat = D^-1 A: mean over the stored row (GraphSAGE, mean form)   */
    MIXGCN_NORM_SUM = 2   /* A_hat = A + eps I on the stored pattern: 1 off the diagonal,
                             1 + eps on it (GIN; build the graph with self-loops)               */
};
/* Epilogue flags of mixgcn_aggregate_ex. */
enum {
    MIXGCN_EPI_RELU = 1,      /* Z = max(A_hat H, 0)                                            */
    MIXGCN_EPI_ACCUMULATE = 2 /* Z = Z + A_hat H (applied before the ReLU if both are set)     */
};
enum { MIXGCN_F32 = 0, MIXGCN_BF16 = 1 };

/* mixgcn_update ops */
enum {
    MIXGCN_OP_FWD = 0,      /* C[n x m] = A[n x k] B[k x m]                                  */
    MIXGCN_OP_FWD_RELU = 1, /* C = max(A B, 0)                                               */
    MIXGCN_OP_DGRAD = 2,    /* C[n x k] = (A (.) 1[R > 0])[n x m]  B[k x m]^T                */
    MIXGCN_OP_WGRAD = 3     /* C[k x m] = beta C + A[n x k]^T (B (.) 1[R > 0])[n x m]        */
};

/* mixgcn_set_update_arith: how the update products of fp32 features use the matrix cores */
enum {
    MIXGCN_ARITH_FP32 = 0,  /* fp32 MFMA (the default)                                        */
    MIXGCN_ARITH_BF16X3 = 1 /* every fp32 operand as the exact sum of three bf16 terms, six   */
                            /* bf16 MFMAs per product, fp32 accumulation                      */
};

typedef struct mixgcn_graph mixgcn_graph;
typedef struct mixgcn_pipeline mixgcn_pipeline;

/* Read-only view of a graph's device arrays (valid until mixgcn_graph_free). */
typedef struct mixgcn_graph_view {
    uint32_t n_nodes;
    uint32_t flags;        /* the build flags */
    int64_t nnz;           /* stored entries of A_tilde, self-loops included */
    const int64_t* rowptr; /* [n_nodes + 1] */
    const uint32_t* col;   /* [nnz], ascending within a row */
    const float* val;      /* [nnz] A_hat values, NULL before mixgcn_normalize */
    const uint32_t* deg;   /* [n_nodes] D_tilde_uu, NULL before mixgcn_normalize */
    const float* dinv;     /* [n_nodes] D_tilde_uu^-1/2, NULL before mixgcn_normalize */
    const int64_t* t_rowptr; /* transpose CSR; equal to rowptr/col/val pointers when the   */
    const uint32_t* t_col;   /* graph was symmetrised; NULL if no transpose is available   */
    const float* t_val;
} mixgcn_graph_view;

/* One GCN layer for mixgcn_layer_fwd / mixgcn_layer_bwd. */
typedef struct mixgcn_layer_desc {
    int32_t f_in;     /* d^(l): width of H and Z */
    int32_t f_out;    /* d^(l+1): width of H' */
    int64_t ld_h;     /* leading dimension of H (input features) and of dH */
    int64_t ld_z;     /* leading dimension of Z and dZ */
    int64_t ld_out;   /* leading dimension of Hout and G */
    int64_t ld_w;     /* leading dimension of W and dW (fp32, f_in x f_out) */
    int32_t dtype;    /* MIXGCN_F32 or MIXGCN_BF16 (storage of H, Z, Hout, G, dH) */
    int32_t relu;     /* 1: Hout = relu(Z W); 0: Hout = Z W (last layer) */
    int32_t n_chunks; /* row chunks of the fine-grain pipeline; 1 = no overlap */
    int32_t order;    /* MIXGCN_AGG_FIRST (Algorithm 2) or MIXGCN_UPDATE_FIRST */
} mixgcn_layer_desc;

/*
 * Eq. 3 is associative: sigma((A_hat H) W) = sigma(A_hat (H W)).  Algorithm 2 aggregates first;
 * when a layer narrows (f_out < f_in) updating first makes the aggregation f_in / f_out times
 * cheaper.  Both orders give the same result up to rounding.
 */
enum { MIXGCN_AGG_FIRST = 0, MIXGCN_UPDATE_FIRST = 1 };

/*
 * Sec. 2.1: A_tilde = A + I for a binary adjacency A.  Builds the sorted CSR of A_tilde from a
 * directed edge list: (optionally) symmetrise, drop u == v, drop duplicates, (optionally) add
 * the diagonal, order by (row, column).
 *   src, dst  : [n_edges] node ids (device, or host with MIXGCN_INPUT_ON_HOST); not modified.
 *   out       : receives a new graph, released with mixgcn_graph_free.
 * Synchronises `stream` (nnz must be known to size the arrays).  An endpoint >= n_nodes gives
 * MIXGCN_EINVAL and no graph.
 */
int mixgcn_build_csr(const uint32_t* src, const uint32_t* dst, uint64_t n_edges, uint32_t n_nodes,
                     uint32_t flags, void* stream, mixgcn_graph** out);

/*
 * Sec. 2.1: D_tilde_uu = sum_v A_tilde_uv and A_hat = D_tilde^-1/2 A_tilde D_tilde^-1/2.
 * Fills deg (row sums, exact integers), dinv = (float)(1/sqrt((double)deg)) and
 * val[e] = dinv[row(e)] * dinv[col[e]] (one fp32 multiply, so val is symmetric bit for bit),
 * for the transpose as well if it is stored.  Asynchronous on `stream`.
 */
int mixgcn_normalize(mixgcn_graph* g, int mode, void* stream);
/*
 * The same with the aggregation matrix of another architecture (MIXGCN_NORM_*); mixgcn_normalize
 * is this call with eps = 0.  deg is always the stored row count.
 *   MEAN: dinv = (float)(1 / (double)deg) (0 for an empty row), val[e] = dinv[row(e)].  The
 *         transpose has other values (dinv[col]) on the same pattern; they are kept beside the
 *         matrix, and transpose = 1 of the aggregate calls uses them.
 *   SUM:  val[e] = 1, and (float)1 + eps where row == col (entries that are not stored stay
 *         zero: without self-loops in the graph eps has no effect).  eps must be finite.
 */
int mixgcn_normalize_mode(mixgcn_graph* g, int mode, float eps, void* stream);

/*
 * Algorithm 2, aggregation phase (and its adjoint for the backward pass):
 *   Z[r, c] = sum_{e in row r of M} val[e] * H[col[e], c],
 *   r in [row_begin, row_end), c in [col_begin, col_end),  M = A_hat (transpose = 0) or
 *   A_hat^T (transpose = 1).
 * [col_begin, col_end) is the worker's feature slice [floor(d i/m), floor(d (i+1)/m));
 * [row_begin, row_end) is a pipeline chunk.  H and Z are indexed with absolute columns; entries
 * of Z outside the ranges are not touched: the bounds need not be multiples of anything, so the
 * slice bounds floor(d i/m) of Algorithm 2 can be passed as they are (the kernel works on
 * 16-byte groups of a row; of the first and the last group of a range it writes only the
 * elements inside the range, one by one; H is read in whole groups, which always lie inside the
 * row pitch).  H and Z must not overlap.
 *
 * Concurrency.  Rows that are cut by the kernel's work split are completed through a scratch
 * buffer that belongs to the graph and to the stream of the call: calls on one stream share it
 * in stream order, calls on different streams use different buffers, so the column slices of one
 * graph may be aggregated on several streams at once.  The buffer of the first stream is
 * allocated by mixgcn_normalize; each further stream that aggregates the graph gets its own on
 * its first call (one hipMalloc of mixgcn_aggregate_scratch_bytes(nnz), no synchronisation), or
 * ahead of time through mixgcn_graph_reserve_streams.  Up to 16 streams per graph are served
 * this way; a 17th takes over the least recently used buffer after a device synchronisation.
 * Otherwise the call allocates nothing and does not synchronise.
 */
int mixgcn_aggregate(const mixgcn_graph* g, int transpose, int dtype, const void* H, int64_t ldh,
                     void* Z, int64_t ldz, int32_t col_begin, int32_t col_end, int64_t row_begin,
                     int64_t row_end, void* stream);

/*
 * Makes sure that `n_streams` (1..16) scratch buffers of the aggregation are allocated and not
 * yet owned by a stream, so that the next n_streams streams that aggregate this graph for the
 * first time allocate nothing (a stream keeps its buffer, so later calls on it never do).
 * After mixgcn_normalize; MIXGCN_EINVAL if fewer than n_streams of the 16 slots are unowned.
 * mixgcn_aggregate_scratch_bytes: size of one such buffer for a graph with nnz stored entries
 * (host arithmetic): enough for any row and column range of any call.
 * mixgcn_aggregate_scratch_need: what one call over n_cols columns actually uses when its rows
 * hold the stored entries [entry_begin, entry_end) (host arithmetic; -1 for bad arguments).
 */
int mixgcn_graph_reserve_streams(mixgcn_graph* g, int32_t n_streams);
int64_t mixgcn_aggregate_scratch_bytes(int64_t nnz);
int64_t mixgcn_aggregate_scratch_need(int dtype, int32_t n_cols, int64_t entry_begin,
                                      int64_t entry_end);

/*
 * mixgcn_aggregate for callers that cannot allocate device memory or tolerate a library that
 * does (work recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc):
 * the same kernels and the same result bit for bit, but the scratch for the rows cut by the
 * work split is a fixed 64 MiB array in device memory that the library holds on every GPU it
 * runs on until the process ends.  The call makes no hipMalloc / hipFree and no call that does.
 * A call that needs more scratch than the array has (mixgcn_aggregate_scratch_need: about one
 * byte per stored entry of the row range at 256 fp32 columns, half of that at 128; 67 million
 * entries fit at 256 columns) is refused with MIXGCN_EINVAL before anything is launched.  All
 * calls on one GPU share the array, whatever the graph: calls that overlap in time (different
 * streams with no ordering between them) race; calls on one stream are safe.  Nothing in the
 * array has to be cleared between calls: every slot a call reads it has written before.
 */
int mixgcn_aggregate_static(const mixgcn_graph* g, int transpose, int dtype, const void* H,
                            int64_t ldh, void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                            int64_t row_begin, int64_t row_end, void* stream);

/*
 * mixgcn_aggregate with an epilogue (MIXGCN_EPI_* flags, 0 = none), for the layer forms that
 * combine a node's own features with the aggregate (GraphSAGE's concatenation, whose backward
 * pass is dH = dX_self + A_hat^T dX_neigh):
 *   ACCUMULATE adds the row sums to what Z holds (a row without stored entries adds nothing);
 *   RELU clamps the result at zero, also on the rows without entries.
 * H and Z may be two column blocks of ONE row-major buffer: same ld, and the column ranges
 * [0, col_end) counted from the H pointer and from the Z pointer do not meet within a row
 * (H = X, Z = X + F with F >= col_end rounded up to a whole 16-byte group, 2 F <= ld).
 */
int mixgcn_aggregate_ex(const mixgcn_graph* g, int transpose, int dtype, const void* H, int64_t ldh,
                        void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                        int64_t row_begin, int64_t row_end, int epilogue, void* stream);

/*
 * Sec. 3.2.1, Eq. 4 (S-SpMM): Z = (M_op H) (.) mask on the same ranges as mixgcn_aggregate, the
 * output mask given in bitmap form: column c of row r is bit (c mod 32) of the uint32 word
 * mask[r * ld_mask + c / 32] (device memory, ld_mask >= ceil(col_end / 32) words).  An output
 * whose bit is clear is written as zero; one whose bit is set is the full neighbor sum.  In the
 * backward pass with mask = 1[H > 0] of the layer input this produces the masked gradient dP of
 * the layer below directly.
 */
int mixgcn_aggregate_masked(const mixgcn_graph* g, int transpose, int dtype, const void* H,
                            int64_t ldh, void* Z, int64_t ldz, int32_t col_begin, int32_t col_end,
                            int64_t row_begin, int64_t row_end, const uint32_t* mask,
                            int64_t ld_mask, void* stream);

/*
 * The output sparsity of a ReLU layer in the bitmap form above (Sec. 3.2.1): bit (c mod 32) of
 * mask[r * ld_mask + c / 32] = X[r, c] > 0 for c < n_cols; every word of a row up to ld_mask is
 * written, bits past n_cols are clear.  X is n_rows x n_cols (device, fp32 or bf16, 16-byte
 * aligned, ldx a whole number of 16-byte groups like every feature matrix here).
 */
int mixgcn_relu_bitmap(int dtype, const void* X, int64_t ldx, int64_t n_rows, int32_t n_cols,
                       uint32_t* mask, int64_t ld_mask, void* stream);

/*
 * The mask of the S-SpMM's forward use (Sec. 3.2.1: dropout drops about half of the outputs of
 * the aggregation), as a bitmap for mixgcn_aggregate_masked.  The paper specifies no random
 * numbers, so the mask is defined here: element (r, c) of the n_rows x n_cols tensor is kept
 * (bit set) iff the upper 32 bits of output number r * n_cols + c (counting from 0) of the
 * SplitMix64 generator started at `seed` are below keep_probability * 2^32.  A pure function of
 * (seed, r, c): the same call gives the same mask, and the backward pass can regenerate it
 * instead of storing it.  Every word of a row up to ld_mask is written; bits past n_cols are
 * clear.  No scaling by 1 / keep_probability is implied: Eq. 4 multiplies by the 0/1 mask.
 */
int mixgcn_dropout_bitmap(uint64_t seed, int64_t n_rows, int32_t n_cols, double keep_probability,
                          uint32_t* mask, int64_t ld_mask, void* stream);

/*
 * X <- X (.) M in place for a bitmap M (layout as above): the backward pass of an aggregation
 * whose output was masked multiplies the gradient by the same mask before A_hat^T (Eq. 4; the
 * mask is a constant of the step).  X: n_rows x n_cols, 16-byte aligned rows.  A masked-off
 * element becomes +0; the elements of the row padding up to the next 16 bytes are rewritten too
 * (zero where the mask bit past n_cols is clear, as the two mask generators leave it).
 */
int mixgcn_apply_bitmap(int dtype, void* X, int64_t ldx, int64_t n_rows, int32_t n_cols,
                        const uint32_t* mask, int64_t ld_mask, void* stream);

/*
 * Algorithm 2, update phase, and the two products of its backward pass (see MIXGCN_OP_*).
 *   A, B, C    : operands as listed per op; n_rows = n, k = d^(l), m = d^(l+1).
 *   relu_ref   : R, the stored layer output H' whose sign gives the ReLU derivative
 *                (1[R > 0], 0 at 0); NULL = no mask.  Only DGRAD and WGRAD read it.
 *   beta       : WGRAD only, 0 or 1.
 * FWD, FWD_RELU, DGRAD: B is the weight matrix W[k x m], fp32, row-major.  WGRAD: A = Z
 * [n x k], B = the upstream gradient [n x m], C = dW [k x m] fp32.
 * Two per-device work buffers are shared by all calls: the slab partials of WGRAD, and the weight
 * terms of the products with W for bf16 features and under MIXGCN_ARITH_BF16X3.  Calls that use
 * the same one must not overlap: issue them on one stream, or order the streams with events (the
 * layer and pipeline entry points do).
 */
int mixgcn_update(int op, int dtype, const void* A, int64_t lda, const void* B, int64_t ldb,
                  void* C, int64_t ldc, int64_t n_rows, int32_t k, int32_t m,
                  const void* relu_ref, int64_t ldr, float beta, void* stream);

/*
 * Chooses the arithmetic of the update products (Algorithm 2, update phase) for fp32 features in
 * every later call of this process, whichever entry point launches them; bf16 features are not
 * affected.  MIXGCN_ARITH_BF16X3 applies to the forward product and the data gradient when the
 * output is wider than 64 columns, the reduction depth (k forward, m backward) is a multiple of
 * 16 and at least 64, to the weight gradient when k and m are multiples of 128 (its last
 * n_rows % 16 rows are added by the fp32 kernel), and only with pitches below 2^22 elements;
 * every other product keeps the fp32 MFMA.  Its error per product term is bounded by
 * 2^-23 |a| |b| (the three dropped partial products), the size of an fp32 rounding; non-finite
 * inputs, and magnitudes that round to infinity as bf16 (above 3.39e38), give NaN where the fp32
 * path gives an infinity or a finite value.  The accumulation is the bf16 MFMA's own: over the
 * long reduction of the weight gradient it is somewhat coarser than the fp32 MFMA's (measured
 * relative error of dW at 2^20 rows: 2.5e-6 against 8e-7), over the short ones of the other two
 * products it is not.  Not thread safe: set it before
 * launching work.  MIXGCN_EINVAL for an unknown mode.
 */
int mixgcn_set_update_arith(int mode);

/*
 * One layer forward, Eq. 3.
 *   MIXGCN_AGG_FIRST (order of Algorithm 2):  Z = A_hat H [n x f_in];  Hout = sigma(Z W), run as
 *     d->n_chunks row chunks with the aggregation of chunk k overlapping the update of chunk
 *     k-1 on the pipeline's two streams (Sec. 3.2.2).  Z is kept for the backward pass.
 *   MIXGCN_UPDATE_FIRST:  Z = H W [n x f_out, ld_z >= f_out] (workspace);  Hout = sigma(A_hat Z).
 *     The backward pass needs H instead of Z.
 * On return the work is enqueued; the pipeline's primary stream is ordered after all of it.
 */
int mixgcn_layer_fwd(const mixgcn_graph* g, const mixgcn_layer_desc* d, const void* H,
                     const float* W, void* Z, void* Hout, mixgcn_pipeline* p);

/*
 * One layer backward: the chain rule of Eq. 3 in the order of Algorithm 2's backward line
 * ("perform backward propagation", which Sec. 3.1.2 describes as the forward workflow run in
 * reverse).  With dP = G (.) 1[Hout > 0] (d->relu) or dP = G:
 *   MIXGCN_AGG_FIRST:     dW = Z^T dP;   dZ = dP W^T (written over Z);   dH = A_hat^T dZ.
 *                         H is not read (may be NULL).
 *   MIXGCN_UPDATE_FIRST:  dQ = A_hat^T dP [n x f_out] (written to the workspace Z);
 *                         dW = H^T dQ;   dH = dQ W^T.  H is the layer's input [n x f_in, ld_h].
 * G may be overwritten.  dH == NULL skips the input gradient (first layer when none is wanted).
 * dW is fp32 [f_in x f_out] with leading dimension d->ld_w.
 * The backward pass is not cut into row chunks: with d->n_chunks > 1 and two streams the two
 * dense products run on the secondary stream and the transposed aggregation, which needs all
 * of dZ, follows on the primary one.
 */
int mixgcn_layer_bwd(const mixgcn_graph* g, const mixgcn_layer_desc* d, const void* H, void* Z,
                     const void* Hout, const float* W, void* G, float* dW, void* dH,
                     mixgcn_pipeline* p);

/*
 * Sec. 3.2.2, Proposition 3.5: several layers as one fine-grain pipeline.  The nodes are processed
 * in s = n_chunks batches of consecutive rows (the same s, dtype and graph for every layer; batch
 * boundaries are multiples of 128 rows, see mixgcn_pipeline_window).  With bandwidth b of the
 * graph as numbered, batch c of an aggregation reads only rows [r0 - b, r1 + b) of its input, so
 * it is started as soon as the dense operation before it has written those batches, while that
 * operation is still working on later ones; aggregations are issued on the pipeline's primary
 * stream, updates on its secondary stream.  With b >= n - 1 every aggregation waits for the whole
 * operation before it and the schedule is the layer-by-layer one.  By Proposition 3.5 the first
 * batch of the next aggregation never waits for the last batch of the update before it once
 * s >= mixgcn_pipeline_stages(n, b).
 *   d[l]     : descriptor of layer l; d[l].f_in == d[l-1].f_out and d[l].ld_h == d[l-1].ld_out.
 *   H0       : input of layer 0; the input of layer l > 0 is Hout[l-1].
 *   W, Z, Hout, G, dW : host arrays of n_layers device pointers, used per layer exactly as by
 *              mixgcn_layer_fwd / mixgcn_layer_bwd.  G[n_layers-1] holds the loss gradient on
 *              entry; G[l-1] receives the input gradient of layer l (the dH of
 *              mixgcn_layer_bwd); dH0 (may be NULL: not computed) that of layer 0.
 *   bandwidth: b; a value below the stored graph's own bandwidth (computed once per graph, which
 *              synchronises the primary stream on the first call) is MIXGCN_EINVAL.
 * The weight gradient of a layer is accumulated batch by batch (beta = 1 after the first), so it
 * agrees with mixgcn_layer_bwd up to the order of summation.  On return the work is enqueued and
 * the primary stream is ordered after all of it.
 *
 * mixgcn_pipeline_window (host arithmetic): rows [*row_begin, *row_end) of batch `chunk`, and the
 * batches [*first, *last] of its input that a windowed operation on that batch reads.  Any
 * output pointer may be NULL.
 */
int mixgcn_forward_pipelined(const mixgcn_graph* g, int32_t n_layers, const mixgcn_layer_desc* d,
                             const void* H0, const float* const* W, void* const* Z,
                             void* const* Hout, int64_t bandwidth, mixgcn_pipeline* p);
int mixgcn_backward_pipelined(const mixgcn_graph* g, int32_t n_layers, const mixgcn_layer_desc* d,
                              const void* H0, void* const* Z, const void* const* Hout,
                              const float* const* W, void* const* G, float* const* dW, void* dH0,
                              int64_t bandwidth, mixgcn_pipeline* p);
int mixgcn_pipeline_window(int64_t n_nodes, int32_t n_chunks, int64_t bandwidth, int32_t chunk,
                           int64_t* row_begin, int64_t* row_end, int32_t* first, int32_t* last);

/*
 * Loss glue (Algorithm 2, loss line): mean softmax cross-entropy over n nodes and its gradient
 * dlogits = (softmax - onehot) / n (may alias logits).  logits and dlogits are stored as
 * `dtype` (the arithmetic is fp32, the loss sum fp64).  loss: one device double.
 */
int mixgcn_softmax_xent(int dtype, const void* logits, int64_t ldl, const int32_t* labels,
                        int64_t n, int32_t n_classes, void* dlogits, int64_t ldd, double* loss,
                        void* stream);

/* Helpers. */
int mixgcn_graph_info(const mixgcn_graph* g, mixgcn_graph_view* out);
int mixgcn_graph_free(mixgcn_graph* g);
/*
 * A stream whose kernels run on a subset of the compute units, for splitting the GPU between
 * the sparse and the dense half of the pipeline: CU c is enabled iff (c / 8) % groups lies in
 * [lo, hi).  Default priority.  Destroy with mixgcn_stream_destroy (after its work is done).
 */
int mixgcn_stream_create_cu_subset(int lo, int hi, int groups, void** stream);
int mixgcn_stream_destroy(void* stream);
/* Two streams for the chunk pipeline: `primary` runs the aggregation, `secondary` the update. */
int mixgcn_pipeline_create(void* primary_stream, void* secondary_stream, mixgcn_pipeline** out);
int mixgcn_pipeline_destroy(mixgcn_pipeline* p);
/*
 * Per-launch timing for benchmarks: while enabled, mixgcn_layer_fwd / mixgcn_layer_bwd record a
 * HIP event pair around every launch of the aggregation kernel and of the update kernels, on
 * the stream of that launch.  mixgcn_pipeline_timing(p, enable) switches it and clears what was
 * recorded.  mixgcn_pipeline_timing_read synchronises both streams and returns the summed
 * duration (ms) and the number of launches of one kind (host pointers):
 *   0..4  aggregation kernel with lane groups of 4, 8, 16, 32, 64 lanes (slice widths up to
 *         16, 32, 64, 128, 256 fp32 columns; twice that for bf16)
 *   5 update forward, 6 update dgrad, 7 update wgrad (split-K slab kernel).
 */
enum { MIXGCN_TIME_AGG_G4 = 0, MIXGCN_TIME_AGG_G8 = 1, MIXGCN_TIME_AGG_G16 = 2,
       MIXGCN_TIME_AGG_G32 = 3, MIXGCN_TIME_AGG_G64 = 4, MIXGCN_TIME_UPDATE_FWD = 5,
       MIXGCN_TIME_UPDATE_DGRAD = 6, MIXGCN_TIME_UPDATE_WGRAD = 7 };
int mixgcn_pipeline_timing(mixgcn_pipeline* p, int enable);
int mixgcn_pipeline_timing_read(mixgcn_pipeline* p, int kind, double* total_ms, int64_t* launches);
/*
 * Sec. 3.2.2 (pipeline scheduler with node reordering).  mixgcn_reorder_rcm writes the position
 * p_v of every node in a reverse Cuthill-McKee processing sequence to pos[v] (device, n_nodes
 * uint32), computed from the stored rows of the graph (for a symmetrised graph: its undirected
 * form).  The rule is deterministic: degree = stored entries of the row; a component starts
 * from the unvisited node of smallest (degree, id); nodes are visited in queue order and the
 * unvisited neighbors of the visited node join the queue in increasing (degree, id); the
 * sequence is the visiting order reversed.  Synchronises the stream.  Levels with a small
 * frontier (up to 1024 nodes holding up to 4096 stored entries) are walked on the device by one
 * resident workgroup, a few microseconds each; only wider levels cost a launch and a read-back.
 *
 * mixgcn_bandwidth: b = max over stored entries (u, v) of |p_v - p_u| (the paper's graph
 * bandwidth); pos == NULL takes the identity sequence.  *bandwidth is a host pointer.
 *
 * mixgcn_pipeline_stages: Proposition 3.5 - the smallest number of batches s with
 * (n - b) / (2 n) >= 1 / s, i.e. ceil(2 n / (n - b)); 0 if b >= n (no such s).  Host arithmetic.
 *
 * mixgcn_relabel_edges: src_out[i] = pos[src[i]], dst_out[i] = pos[dst[i]] (device arrays; the
 * outputs may alias the inputs), the edge list of the same graph in the new numbering.
 * mixgcn_permute_rows: Y[pos[v], :] = X[v, :] for an n_rows x n_cols feature matrix (device,
 * 16-byte aligned, ld a whole number of 16-byte groups; X and Y must not overlap).
 */
int mixgcn_reorder_rcm(const mixgcn_graph* g, uint32_t* pos, void* stream);
int mixgcn_bandwidth(const mixgcn_graph* g, const uint32_t* pos, int64_t* bandwidth, void* stream);
int64_t mixgcn_pipeline_stages(int64_t n_nodes, int64_t bandwidth);
int mixgcn_relabel_edges(const uint32_t* src, const uint32_t* dst, uint64_t n_edges,
                         const uint32_t* pos, uint32_t n_nodes, uint32_t* src_out,
                         uint32_t* dst_out, void* stream);
int mixgcn_permute_rows(int dtype, const void* X, int64_t ldx, void* Y, int64_t ldy, int64_t n_rows,
                        int32_t n_cols, const uint32_t* pos, void* stream);

/*
 * Measurement aid, not part of the training path: the rates this device sustains on a 4 GiB
 * streaming read and a 4 GiB streaming copy (GB/s; the copy counts read + write), on random
 * 128-byte gathers (16 bytes per lane, 8 lanes per line, nothing else in the kernel) from a
 * 2 MiB buffer that every L2 holds and from a 4 GiB buffer in HBM, and on register-only MFMA
 * chains in fp32 (32x32x2) and bf16 (32x32x16), in TFLOP/s, for comparison with the published
 * peaks that the roofline fractions are quoted against.  Outputs are host pointers.  Allocates
 * and frees 8 GiB of device memory; synchronises the stream.
 */
int mixgcn_measure_peaks(double* read_gbs, double* copy_gbs, double* gather_l2_gbs,
                         double* gather_hbm_gbs, double* mfma_f32_tflops,
                         double* mfma_bf16_tflops, void* stream);
/*
 * Measurement aid, not part of the training path: with on != 0 every later aggregation of this
 * process gathers whole rows (no column slices pinned to XCDs), which is what a kernel would have
 * to do that keeps the aggregated tile on the compute unit for the update product (Sec. 3.2.2,
 * the fine-grain pipeline in its tightest form).  Same results, other speed; timing it bounds
 * such a fusion from below.  Process-wide and not thread safe; set it BEFORE mixgcn_normalize of
 * the graphs it is used with (it changes the size of their aggregation scratch).
 */
int mixgcn_set_aggregate_whole_rows(int on);
const char* mixgcn_strerror(int code);
const char* mixgcn_last_error(void);
int mixgcn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MIXGCN_H */
