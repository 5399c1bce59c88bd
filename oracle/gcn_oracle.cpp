/*
 * CPU oracle for full-graph GCN training (MixGCN paper, Sec. 2.1, Eq. 3, Algorithm 2).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is the plain, slow definition of what the
 * HIP path must compute, written with explicit loops and double precision throughout.  It
 * shares no code with the HIP library and nothing in the product path may call it.
 *
 * Layout convention: node x feature, row-major, with explicit leading dimensions.  The paper
 * stores feature x node matrices and writes a layer as  H'^T = sigma(A_hat H^T W^T)  (Eq. 3);
 * with W here = the paper's W^T this is  H' = sigma(A_hat H W), the same computation.
 *
 * What is pinned by tests that do not use this file's own formulas: CSR/degrees against a
 * dense boolean matrix built independently; A_hat values against regular graphs, complete
 * graphs, edgeless graphs and the eigenvector identity A_hat d^(1/2) = d^(1/2); the products
 * against dense brute force and adjoint identities; the loss against ln C at W = 0; the whole
 * forward+backward against central finite differences and the linear-activation closed form;
 * the masked aggregation (S-SpMM) against a dense masked product, the complement identity
 * Z(M) + Z(not M) = A_hat H, and Z = M on regular graphs with H = 1; the bitmap against numpy;
 * the reverse Cuthill-McKee sequence against a hand-worked example, closed forms (path, cycle,
 * star, complete graph, grid) and the brute-force optimum on 7-node graphs; the dropout mask
 * against the generator's published test vector and its density.  The GraphSAGE and GIN steps
 * (numpy, in the Python module beside this file) are pinned by node-by-node definitions,
 * special cases that reduce to a perceptron and finite differences.  No function here is
 * "parity unpinned".
 */
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

#if defined(_OPENMP)
#include <omp.h>
#include <parallel/algorithm>
#define ORACLE_SORT __gnu_parallel::sort
#else
#define ORACLE_SORT std::sort
#endif

namespace {

/* Storage rounding applied where a tensor is written back (never inside a sum).
 * 0: keep double; 1: round to fp32; 2: round to bf16 (round-to-nearest-even). */
inline double quantize(double x, int q)
{
    if (q == 0) return x;
    float f = (float)x;
    if (q == 1) return (double)f;
    uint32_t u;
    std::memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) != 0x7F800000u) { /* finite: RNE to the upper 16 bits */
        u += 0x7FFFu + ((u >> 16) & 1u);
    }
    u &= 0xFFFF0000u;
    std::memcpy(&f, &u, 4);
    return (double)f;
}

}  // namespace

extern "C" {

int oracle_num_threads()
{
#if defined(_OPENMP)
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#if defined(_OPENMP)
    omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * A_tilde = A + I as a sorted CSR (Sec. 2.1: A_tilde = A + I; the adjacency is binary).
 * From a directed edge list: optionally add the reverse of every edge, drop u == v, drop
 * duplicates, then (optionally) put exactly one diagonal entry in every row.  Columns ascend
 * within a row.  col must have room for (symmetrize ? 2 : 1) * n_edges + n_nodes entries.
 * Returns nnz, or -1 if an endpoint is out of range.
 */
int64_t oracle_build_csr(const uint32_t* src, const uint32_t* dst, uint64_t n_edges,
                         uint32_t n_nodes, int symmetrize, int add_self_loops,
                         int64_t* rowptr, uint32_t* col)
{
    std::vector<uint64_t> pairs;
    pairs.reserve((symmetrize ? 2 : 1) * n_edges + (add_self_loops ? n_nodes : 0));
    for (uint64_t i = 0; i < n_edges; ++i) {
        uint64_t u = src[i], v = dst[i];
        if (u >= n_nodes || v >= n_nodes) return -1;
        if (u == v) continue;
        pairs.push_back((u << 32) | v);
        if (symmetrize) pairs.push_back((v << 32) | u);
    }
    if (add_self_loops)
        for (uint64_t u = 0; u < n_nodes; ++u) pairs.push_back((u << 32) | u);
    ORACLE_SORT(pairs.begin(), pairs.end());
    pairs.erase(std::unique(pairs.begin(), pairs.end()), pairs.end());

    for (uint64_t u = 0; u <= n_nodes; ++u) rowptr[u] = 0;
    for (uint64_t p : pairs) rowptr[(p >> 32) + 1] += 1;
    for (uint64_t u = 0; u < n_nodes; ++u) rowptr[u + 1] += rowptr[u];
    for (size_t e = 0; e < pairs.size(); ++e) col[e] = (uint32_t)(pairs[e] & 0xFFFFFFFFull);
    return (int64_t)pairs.size();
}

/*
 * D_tilde_uu = sum_v A_tilde_uv (a count, since A_tilde is binary) and
 * A_hat_uv = A_tilde_uv / sqrt(D_uu D_vv)   (Sec. 2.1).
 * deg: row sums.  dinv: D^(-1/2) in double.  val: A_hat in double, by the definition.
 * val_f32 (optional): the fp32 encoding  float(dinv[u]) * float(dinv[v])  rounded once,
 * which is symmetric in (u, v) bit for bit.
 */
void oracle_normalize(const int64_t* rowptr, const uint32_t* col, uint32_t n_nodes,
                      uint32_t* deg, double* dinv, double* val, float* val_f32)
{
    for (uint32_t u = 0; u < n_nodes; ++u) {
        uint32_t d = 0;
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) d += 1; /* sum of ones */
        deg[u] = d;
        dinv[u] = d ? 1.0 / std::sqrt((double)d) : 0.0;
    }
    for (uint32_t u = 0; u < n_nodes; ++u)
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            uint32_t v = col[e];
            /* A zero row sum can only occur without the diagonal (the paper always adds I);
             * D^(-1/2) is then undefined and the entry is taken as 0. */
            val[e] = (deg[u] && deg[v]) ? 1.0 / std::sqrt((double)deg[u] * (double)deg[v]) : 0.0;
            if (val_f32) val_f32[e] = (float)dinv[u] * (float)dinv[v];
        }
}

/*
 * CSR of the transpose of a (rowptr, col, val) matrix whose scaling vector is unchanged:
 * entry (u, v, x) becomes (v, u, x).  Columns ascend within each output row.
 */
void oracle_transpose(const int64_t* rowptr, const uint32_t* col, const double* val,
                      uint32_t n_nodes, int64_t* t_rowptr, uint32_t* t_col, double* t_val)
{
    const int64_t nnz = rowptr[n_nodes];
    for (uint64_t u = 0; u <= n_nodes; ++u) t_rowptr[u] = 0;
    for (int64_t e = 0; e < nnz; ++e) t_rowptr[col[e] + 1] += 1;
    for (uint64_t u = 0; u < n_nodes; ++u) t_rowptr[u + 1] += t_rowptr[u];
    std::vector<int64_t> cursor(t_rowptr, t_rowptr + n_nodes);
    for (uint32_t u = 0; u < n_nodes; ++u) /* ascending u keeps the output columns sorted */
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            int64_t p = cursor[col[e]]++;
            t_col[p] = u;
            t_val[p] = val[e];
        }
}

/*
 * Neighbor aggregation on a column slice and a row range (Algorithm 2, aggregation phase):
 *   Z[v, j] = sum_{e in row v} val[e] * H[col[e], c0 + j],  v in [r0, r1), j in [0, c1 - c0).
 * H is indexed with the absolute column c0 + j; Z likewise (Z[v*ldz + c0 + j]).
 */
void oracle_spmm(const int64_t* rowptr, const uint32_t* col, const double* val,
                 const double* H, int64_t ldh, double* Z, int64_t ldz, int64_t c0, int64_t c1,
                 int64_t r0, int64_t r1, int q)
{
#pragma omp parallel
    {
        std::vector<double> acc((size_t)(c1 - c0));
#pragma omp for schedule(dynamic, 64)
        for (int64_t v = r0; v < r1; ++v) {
            std::fill(acc.begin(), acc.end(), 0.0);
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e) { /* neighbors in column order */
                const double a = val[e];
                const double* h = H + (int64_t)col[e] * ldh;
                for (int64_t j = c0; j < c1; ++j) acc[j - c0] += a * h[j];
            }
            for (int64_t j = c0; j < c1; ++j) Z[v * ldz + j] = quantize(acc[j - c0], q);
        }
    }
}

/*
 * Output sparsity in bitmap form (Sec. 3.2.1: the mask of a ReLU layer is kept as a bitmap):
 * bit (j mod 32) of bits[v * ldb + j / 32] is set iff X[v, j] > 0.  Bits past column m are clear.
 */
void oracle_relu_bitmap(const double* X, int64_t ldx, int64_t n, int64_t m, uint32_t* bits,
                        int64_t ldb)
{
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t w = 0; w < ldb; ++w) bits[v * ldb + w] = 0u;
        for (int64_t j = 0; j < m; ++j)
            if (X[v * ldx + j] > 0.0) bits[v * ldb + j / 32] |= 1u << (j % 32);
    }
}

/*
 * The forward use of the output mask (Sec. 3.2.1: about half of the aggregation's outputs are
 * dropped by dropout in the forward pass).  The paper gives no random-number specification, so the
 * mask is defined here: element (v, j) of an n x m tensor is KEPT iff the upper 32 bits of
 * splitmix64(seed, v * m + j) are below keep * 2^32, where splitmix64(seed, i) is output i
 * (counting from 0) of the SplitMix64 generator (Steele, Lea, Flood, OOPSLA 2014) started at
 * `seed`: z = seed + (i + 1) * 0x9E3779B97F4A7C15, then two xor-shift-multiply rounds and a final
 * xor-shift.  A pure function of (seed, index), so any number of threads produce the same mask.
 */
uint64_t oracle_splitmix64(uint64_t seed, uint64_t i)
{
    uint64_t z = seed + (i + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* keep in [0, 1]; bitmap layout as oracle_relu_bitmap (bits past column m are clear). */
void oracle_dropout_bitmap(uint64_t seed, int64_t n, int64_t m, double keep, uint32_t* bits,
                           int64_t ldb)
{
    double t = keep * 4294967296.0;
    if (t < 0.0) t = 0.0;
    if (t > 4294967296.0) t = 4294967296.0;
    const uint64_t threshold = (uint64_t)t;
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t w = 0; w < ldb; ++w) bits[v * ldb + w] = 0u;
        for (int64_t j = 0; j < m; ++j)
            if ((oracle_splitmix64(seed, (uint64_t)(v * m + j)) >> 32) < threshold)
                bits[v * ldb + j / 32] |= 1u << (j % 32);
    }
}

/*
 * S-SpMM (Sec. 3.2.1, Eq. 4):  Z = (A H) (.) M  with the mask M given as a bitmap (layout as
 * above).  Every output is the full neighbor sum of the plain aggregation, kept where the mask
 * bit is set and zero elsewhere.
 */
void oracle_sspmm(const int64_t* rowptr, const uint32_t* col, const double* val, const double* H,
                  int64_t ldh, double* Z, int64_t ldz, int64_t c0, int64_t c1, int64_t r0,
                  int64_t r1, const uint32_t* bits, int64_t ldb, int q)
{
    for (int64_t v = r0; v < r1; ++v)
        for (int64_t j = c0; j < c1; ++j) {
            double acc = 0.0;
            for (int64_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
                acc += val[e] * H[(int64_t)col[e] * ldh + j];
            const bool keep = (bits[v * ldb + j / 32] >> (j % 32)) & 1u;
            Z[v * ldz + j] = keep ? quantize(acc, q) : 0.0;
        }
}

/*
 * Node reordering (Sec. 3.2.2): reverse Cuthill-McKee positions.  pos[v] = place of node v in
 * the processing sequence (the paper's p_v).  The rule, made deterministic:
 *   - the degree of a node is the number of stored entries of its row;
 *   - a component is started from the unvisited node with the smallest (degree, id);
 *   - nodes are visited in queue order, and the unvisited neighbors of the node being visited
 *     join the queue in increasing (degree, id);
 *   - the final sequence is the visiting sequence reversed.
 */
void oracle_rcm(const int64_t* rowptr, const uint32_t* col, uint32_t n, uint32_t* pos)
{
    std::vector<uint32_t> by_deg(n), order;
    order.reserve(n);
    for (uint32_t v = 0; v < n; ++v) by_deg[v] = v;
    auto deg = [&](uint32_t v) { return rowptr[v + 1] - rowptr[v]; };
    auto less = [&](uint32_t a, uint32_t b) {
        return deg(a) != deg(b) ? deg(a) < deg(b) : a < b;
    };
    std::sort(by_deg.begin(), by_deg.end(), less);
    std::vector<char> seen(n, 0);
    std::vector<uint32_t> nb;
    size_t head = 0;
    for (uint32_t root : by_deg) {
        if (seen[root]) continue;
        seen[root] = 1;
        order.push_back(root);
        while (head < order.size()) {
            const uint32_t u = order[head++];
            nb.clear();
            for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e)
                if (!seen[col[e]]) {
                    seen[col[e]] = 1;
                    nb.push_back(col[e]);
                }
            std::sort(nb.begin(), nb.end(), less);
            order.insert(order.end(), nb.begin(), nb.end());
        }
    }
    for (uint32_t i = 0; i < n; ++i) pos[order[i]] = n - 1 - i;
}

/* Graph bandwidth under a processing sequence (Sec. 3.2.2): b = max over stored entries (u, v)
 * of |p_v - p_u|; pos == NULL means the identity sequence. */
int64_t oracle_bandwidth(const int64_t* rowptr, const uint32_t* col, uint32_t n,
                         const uint32_t* pos)
{
    int64_t b = 0;
    for (uint32_t u = 0; u < n; ++u)
        for (int64_t e = rowptr[u]; e < rowptr[u + 1]; ++e) {
            const int64_t pu = pos ? pos[u] : u, pv = pos ? pos[col[e]] : col[e];
            b = std::max<int64_t>(b, pu > pv ? pu - pv : pv - pu);
        }
    return b;
}

/* Proposition 3.5: the idleness of the fine-grain pipeline can be removed when
 * (n - b) / (2 n) >= 1 / s; the smallest such number of batches s, or 0 if there is none
 * (b >= n). */
int64_t oracle_pipeline_stages(int64_t n, int64_t b)
{
    if (n <= 0 || b >= n) return 0;
    for (int64_t s = 1;; ++s)  /* by definition: first s that satisfies the inequality */
        if ((n - b) * s >= 2 * n) return s;
}

/* Node update (Algorithm 2, update phase):  P = Z W  (n x k times k x m), then optional ReLU. */
void oracle_update_fwd(const double* Z, int64_t ldz, const double* W, int64_t ldw, double* Hout,
                       int64_t ldo, int64_t n, int64_t k, int64_t m, int relu, int q)
{
#pragma omp parallel
    {
        std::vector<double> acc((size_t)m);
#pragma omp for schedule(static)
        for (int64_t v = 0; v < n; ++v) {
            std::fill(acc.begin(), acc.end(), 0.0);
            for (int64_t i = 0; i < k; ++i) { /* every acc[j] sums over i in ascending order */
                const double z = Z[v * ldz + i];
                for (int64_t j = 0; j < m; ++j) acc[j] += z * W[i * ldw + j];
            }
            for (int64_t j = 0; j < m; ++j) {
                double s = acc[j];
                if (relu && !(s > 0.0)) s = 0.0;
                Hout[v * ldo + j] = quantize(s, q);
            }
        }
    }
}

/* dP = G (.) 1[Href > 0]  (ReLU derivative, 0 at 0).  Href == NULL means identity. */
void oracle_relu_grad(const double* G, int64_t ldg, const double* Href, int64_t ldr, double* dP,
                      int64_t ldp, int64_t n, int64_t m, int q)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t j = 0; j < m; ++j) {
            double g = G[v * ldg + j];
            if (Href && !(Href[v * ldr + j] > 0.0)) g = 0.0;
            dP[v * ldp + j] = quantize(g, q);
        }
}

/* dZ = dP W^T :  dZ[v, i] = sum_j dP[v, j] W[i, j]. */
void oracle_update_dgrad(const double* dP, int64_t ldp, const double* W, int64_t ldw, double* dZ,
                         int64_t ldz, int64_t n, int64_t k, int64_t m, int q)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t i = 0; i < k; ++i) {
            double s = 0.0;
            for (int64_t j = 0; j < m; ++j) s += dP[v * ldp + j] * W[i * ldw + j];
            dZ[v * ldz + i] = quantize(s, q);
        }
}

/* dW = Z^T dP :  dW[i, j] = sum_v Z[v, i] dP[v, j]  (always kept in double). */
void oracle_update_wgrad(const double* Z, int64_t ldz, const double* dP, int64_t ldp, double* dW,
                         int64_t ldw, int64_t n, int64_t k, int64_t m)
{
    /* Rows are summed in fixed blocks of 4096 (each block in row order) and the block sums are
     * added in block order, so the result does not depend on the number of threads. */
    const int64_t RB = 4096;
    const int64_t nb = (n + RB - 1) / RB;
    std::vector<double> part((size_t)nb * k * m, 0.0);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t b = 0; b < nb; ++b) {
        double* p = part.data() + (size_t)b * k * m;
        const int64_t v1 = std::min(n, (b + 1) * RB);
        for (int64_t v = b * RB; v < v1; ++v)
            for (int64_t i = 0; i < k; ++i) {
                const double z = Z[v * ldz + i];
                for (int64_t j = 0; j < m; ++j) p[i * m + j] += z * dP[v * ldp + j];
            }
    }
    for (int64_t i = 0; i < k; ++i)
        for (int64_t j = 0; j < m; ++j) {
            double s = 0.0;
            for (int64_t b = 0; b < nb; ++b) s += part[(size_t)b * k * m + i * m + j];
            dW[i * ldw + j] = s;
        }
}

/*
 * Mean softmax cross-entropy over all n nodes and its gradient:
 *   loss = -(1/n) sum_v log softmax(logits_v)[y_v],   dlogits = (softmax - onehot) / n.
 * dlogits may be NULL.
 */
double oracle_softmax_xent(const double* logits, int64_t ldl, const int32_t* labels, int64_t n,
                           int64_t c, double* dlogits, int64_t ldd)
{
    std::vector<double> nll((size_t)n);
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        const double* x = logits + v * ldl;
        double mx = x[0];
        for (int64_t j = 1; j < c; ++j) mx = std::max(mx, x[j]);
        double se = 0.0;
        for (int64_t j = 0; j < c; ++j) se += std::exp(x[j] - mx);
        double lse = mx + std::log(se);
        nll[v] = lse - x[labels[v]];
        if (dlogits)
            for (int64_t j = 0; j < c; ++j)
                dlogits[v * ldd + j] =
                    (std::exp(x[j] - lse) - (j == labels[v] ? 1.0 : 0.0)) / (double)n;
    }
    double total = 0.0; /* summed in node order, independent of the thread count */
    for (int64_t v = 0; v < n; ++v) total += nll[v];
    return total / (double)n;
}

/*
 * L-layer GCN, one forward + backward pass in the order of Algorithm 2 (aggregate, then
 * update; ReLU between layers, none after the last; no bias; no dropout):
 *   Z_l = A_hat H_l;  P_l = Z_l W_l;  H_{l+1} = relu(P_l) for l < L-1, = P_l for l = L-1.
 * Backward (derived from Eq. 3 by the chain rule):
 *   dP_{L-1} = (softmax - onehot)/n;  dW_l = Z_l^T dP_l;  dZ_l = dP_l W_l^T;
 *   dH_l = A_hat^T dZ_l;  dP_{l-1} = dH_l (.) 1[H_l > 0].
 * dims has L+1 entries.  All matrices are dense row-major with ld == their column count.
 * W[l]: dims[l] x dims[l+1].  Zs[l]: n x dims[l].  Hs[l] (l = 1..L): n x dims[l] with Hs[L] =
 * logits; Hs[0] is not written.  dW[l] like W[l].  dX (n x dims[0]) may be NULL.
 * linear != 0 replaces every ReLU by the identity.  q != 0 rounds every stored n x F tensor
 * (Z_l, H_l including the logits, the loss gradient, dZ_l, dH_l, dP_l) to fp32 / bf16 where it
 * is written; weights, A_hat, the loss and dW stay in double.  Returns the loss.
 * relu_sign (may be NULL, and so may any entry): relu_sign[l], l = 1..L-1, is an n x dims[l]
 * array that stands in for H_l where the backward pass takes the ReLU derivative,
 * dP_{l-1} = dH_l (.) 1[relu_sign[l] > 0].  The derivative is a 0/1 decision taken from a
 * floating-point value; a caller that compares another implementation's gradients passes that
 * implementation's stored activations here, so that both sides take every decision from the
 * same numbers (an activation within rounding error of zero is a coin toss that neither side
 * gets wrong).  The forward pass is not affected.
 */
double oracle_gcn_step(const int64_t* rowptr, const uint32_t* col, const double* val,
                       const int64_t* t_rowptr, const uint32_t* t_col, const double* t_val,
                       int64_t n, int n_layers, const int64_t* dims, const double* X,
                       const double* const* W, const int32_t* labels, double* const* Zs,
                       double* const* Hs, double* const* dW, double* dX, int linear, int q,
                       const double* const* relu_sign)
{
    const int L = n_layers;
    const double* Hin = X;
    for (int l = 0; l < L; ++l) {
        oracle_spmm(rowptr, col, val, Hin, dims[l], Zs[l], dims[l], 0, dims[l], 0, n, q);
        int relu = (l < L - 1) && !linear;
        oracle_update_fwd(Zs[l], dims[l], W[l], dims[l + 1], Hs[l + 1], dims[l + 1], n, dims[l],
                          dims[l + 1], relu, q);
        Hin = Hs[l + 1];
    }
    const int64_t C = dims[L];
    std::vector<double> dP((size_t)n * C);
    double loss = oracle_softmax_xent(Hs[L], C, labels, n, C, dP.data(), C);
    if (!dW) return loss;
    if (q)  /* the loss gradient is a stored n x C tensor like every other one */
        for (size_t i = 0; i < dP.size(); ++i) dP[i] = quantize(dP[i], q);
    for (int l = L - 1; l >= 0; --l) {
        const int64_t k = dims[l], m = dims[l + 1];
        oracle_update_wgrad(Zs[l], k, dP.data(), m, dW[l], m, n, k, m);
        if (l == 0 && !dX) break;
        std::vector<double> dZ((size_t)n * k);
        oracle_update_dgrad(dP.data(), m, W[l], m, dZ.data(), k, n, k, m, q);
        std::vector<double> dH((size_t)n * k);
        oracle_spmm(t_rowptr, t_col, t_val, dZ.data(), k, dH.data(), k, 0, k, 0, n, q);
        if (l == 0) {
            std::memcpy(dX, dH.data(), sizeof(double) * (size_t)n * k);
            break;
        }
        dP.assign((size_t)n * k, 0.0);
        const double* sign = (relu_sign && relu_sign[l]) ? relu_sign[l] : Hs[l];
        oracle_relu_grad(dH.data(), k, linear ? nullptr : sign, k, dP.data(), k, n, k, q);
    }
    return loss;
}

}  // extern "C"
