// Node update, data gradient and weight gradient of fp32 features (paper Algorithm 2, update
// phase) on the bf16 matrix cores; opt-in (mixgcn_set_update_arith), wide layers only.  Every fp32 operand is
// written as the exact sum of three bf16 terms (round to nearest at each stage),
//     x = x0 + x1 + x2,   |x1| <= 2^-8 |x|,   |x2| <= 2^-16 |x|,
// and a product a b is accumulated in fp32 from the six partial products of order 2^-16 and
// above: a2 b0, a0 b2, a1 b1, a1 b0, a0 b1, a0 b0, smallest first.  The three dropped ones are
// together below 2^-23 |a| |b|, the size of one fp32 rounding, so the result is as good as the
// fp32 MFMA's (the tests measure it slightly better).  On this part a 32x32x16 bf16 MFMA does
// eight times the work of the 32x32x2 fp32 MFMA in half its time, so the six of them cost 3/8 of
// the fp32 path's matrix-core time.
//
// Weights are split once per call, into the order the kernel walks them: the three terms of one
// step (16 reduction indices) of one column tile are contiguous, so a step's weights are three
// coalesced 16-byte loads per thread.  Features are split on their way from global memory to
// LDS: two conversions, four unpacks and four subtractions per term and four elements.  Vector
// instructions do not overlap with MFMAs on a SIMD, so the staging path carries nothing else:
// scalar bases plus fixed per-thread offsets, rows beyond the matrix are read from its last row
// (their results are never stored), and the reduction depth must be whole steps (the caller
// keeps the fp32 MFMA kernels otherwise).  Non-finite inputs give NaN.
//
// Pipeline of a tile: global loads run two steps ahead in two register sets; LDS is double
// buffered; the MFMA operands are themselves double buffered in registers, read from LDS one
// step before their MFMAs, so the only thing between a barrier and the next MFMA is the issue of
// those reads.  The main loop has no conditional load or store, which lets every wait on a load
// leave the other register set's loads in flight.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uintx2 lds_uintx2;
typedef __attribute__((address_space(3))) uintx4 lds_uintx4;

constexpr int BKS = 16;       // reduction depth per step = one MFMA
constexpr int LDR = BKS + 8;  // LDS row stride in bf16: 48 bytes, 16 consecutive rows hit all banks
constexpr int kPlanes = 3;

template <int WM_, int WN_, int TM_, int TN_>
struct Shape {
    static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
    static constexpr int BM = WM * TM * 32;
    static constexpr int BN = WN * TN * 32;
    static_assert(WM * WN == 4, "four waves per block");
};
using Shape128x128 = Shape<2, 2, 2, 2>;

__device__ inline unsigned xcd_local_index(unsigned bid, unsigned grid)
{
    const unsigned q = grid / 8, rem = grid % 8, x = bid % 8;
    return x * q + (x < rem ? x : rem) + bid / 8;
}

// two fp32 -> two bf16 (round to nearest even), first argument in the low half
__device__ inline uint32_t pack_bf16(float a, float b)
{
    const floatx2 v = {a, b};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &h, 4);
    return u;
}
__device__ inline float low_half(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float high_half(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// The three terms of the operand Wop[kk][j] = transpose ? W[kk][j] : W[j][kk], zero outside W, in
// the order the row-block kernel walks them: out[column tile][step][term][j % bn][kk % 16], so
// that the weights of one step of one tile are 3 * bn * 32 contiguous bytes.
__global__ __launch_bounds__(kBlock) void split3_weights_kernel(
    const float* __restrict__ W, int64_t ldw, int rows_w, int cols_w, int transpose,
    uint16_t* __restrict__ out, int out_rows, int out_cols, int bn)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= out_rows * out_cols) return;
    const int j = idx / out_cols, kk = idx % out_cols;
    const int r = transpose ? kk : j, c = transpose ? j : kk;
    float x = (r < rows_w && c < cols_w) ? W[(int64_t)r * ldw + c] : 0.f;
    const int nk = out_cols / BKS;
    const size_t tile = ((size_t)(j / bn) * nk + kk / BKS) * kPlanes;
#pragma unroll
    for (int p = 0; p < kPlanes; ++p) {
        const uint32_t h = pack_bf16(x, 0.f);
        out[((tile + p) * bn + j % bn) * BKS + kk % BKS] = (uint16_t)h;
        x -= low_half(h);
        if (!(fabsf(x) <= 3.0e38f)) x = 0.f;  // infinities and NaNs stay in the first term only
    }
}

// Four fp32 of a row on their way to LDS: the three bf16 planes of the (masked) values.
template <bool MASK>
__device__ inline void split_store(const float4& a, const float4& r, uint16_t* p0, uint16_t* p1,
                                   uint16_t* p2)
{
    float4 x = a;
    if (MASK) {
        x.x = r.x > 0.f ? x.x : 0.f;
        x.y = r.y > 0.f ? x.y : 0.f;
        x.z = r.z > 0.f ? x.z : 0.f;
        x.w = r.w > 0.f ? x.w : 0.f;
    }
    const uintx2 t0 = {pack_bf16(x.x, x.y), pack_bf16(x.z, x.w)};
    x.x -= low_half(t0.x);
    x.y -= high_half(t0.x);
    x.z -= low_half(t0.y);
    x.w -= high_half(t0.y);
    const uintx2 t1 = {pack_bf16(x.x, x.y), pack_bf16(x.z, x.w)};
    x.x -= low_half(t1.x);
    x.y -= high_half(t1.x);
    x.z -= low_half(t1.y);
    x.w -= high_half(t1.y);
    const uintx2 t2 = {pack_bf16(x.x, x.y), pack_bf16(x.z, x.w)};
    *(lds_uintx2*)p0 = t0;
    *(lds_uintx2*)p1 = t1;
    *(lds_uintx2*)p2 = t2;
}

// What one thread moves per step: two 16-byte pieces of the A tile (rows prow and prow + 64,
// four columns), the same of the mask reference, and one 16-byte piece of each weight plane.
template <class S, bool MASK>
struct Stage {
    float4 a[2], r[2];
    uint4 b[kPlanes];

    __device__ inline void load(const char* a0, const char* r0, const char* b0, const uint32_t* aoff,
                                const uint32_t* roff, uint32_t boff)
    {
        // every thread issues the same number of loads on every step, so that the wait for a
        // register set can leave the loads of the other set in flight
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            a[p] = *reinterpret_cast<const float4*>(a0 + aoff[p]);
            if (MASK) r[p] = *reinterpret_cast<const float4*>(r0 + roff[p]);
        }
#pragma unroll
        for (int p = 0; p < kPlanes; ++p)
            b[p] = *reinterpret_cast<const uint4*>(b0 + p * (S::BN * BKS * 2) + boff);
    }
    __device__ inline void store(uint16_t* as, uint16_t* bs, int apos, int bpos, bool b_on) const
    {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            uint16_t* q = as + apos + p * 64 * LDR;
            split_store<MASK>(a[p], r[p], q, q + S::BM * LDR, q + 2 * S::BM * LDR);
        }
        if (b_on) {
#pragma unroll
            for (int p = 0; p < kPlanes; ++p) {
                const uintx4 v = {b[p].x, b[p].y, b[p].z, b[p].w};
                *(lds_uintx4*)(bs + p * S::BN * LDR + bpos) = v;
            }
        }
    }
};

// C[n x MD] = act((A (.) 1[R > 0])[n x KD] * Bop[KD x MD]); Bop is given as three bf16 terms in
// the layout of split3_weights_kernel (bn = BN), KD a multiple of BKS.
template <class S, bool RELU, bool MASK>
__global__ __launch_bounds__(kBlock, 2) void rowblock_split_kernel(
    const float* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bp, float* __restrict__ C, int64_t ldc, int64_t n, int KD, int MD,
    const float* __restrict__ R, int64_t ldr, int n_col_tiles)
{
    static_assert(S::BM == 128, "the staging maps 256 threads onto 128 rows of 16 columns");
    __shared__ __attribute__((aligned(16))) uint16_t As[2][kPlanes * S::BM * LDR];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][kPlanes * S::BN * LDR];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / S::WN, wn = wave % S::WN;
    const unsigned lid = xcd_local_index(blockIdx.x, gridDim.x);
    const int64_t row0 = (int64_t)(lid / n_col_tiles) * S::BM;
    const int col0 = (int)(lid % n_col_tiles) * S::BN;

    floatx16 acc[S::TM][S::TN];
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

    // staging: thread -> (row tid / 4 [+ 64], columns 4 (tid % 4) ..) of A, (row tid / 2, half
    // tid % 2) of the weight planes
    // Rows are dealt to the lanes so that one LDS write cycle (16 lanes of 8 bytes, 8 lanes of 16)
    // covers rows 0, 2, 4, 6 or 1, 3, 5, 7 of a group of eight: at 12 banks per row these start at
    // banks 0, 24, 16, 8 (12, 4, 28, 20) and do not collide.
    auto dealt = [](int q) { return (q & ~7) | ((q & 3) << 1) | ((q >> 2) & 1); };
    const int prow = dealt(tid >> 2), pk = 4 * (tid & 3);
    uint32_t aoff[2], roff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        int64_t rr = row0 + p * 64 + prow;
        if (rr > n - 1) rr = n - 1;
        aoff[p] = (uint32_t)(rr - row0) * (uint32_t)lda * 4u + 4u * pk;
        roff[p] = MASK ? (uint32_t)(rr - row0) * (uint32_t)ldr * 4u + 4u * pk : 0u;
    }
    const int apos = prow * LDR + pk;
    // threads beyond a narrow weight tile load a row of it again and store nothing
    const int brow = dealt(tid >> 1), bhalf = tid & 1;
    const bool b_on = 2 * S::BN >= kBlock || brow < S::BN;
    const uint32_t boff = ((uint32_t)(brow % S::BN) * BKS + 8u * bhalf) * 2u;
    const int bpos = (brow % S::BN) * LDR + 8 * bhalf;

    const char* a0 = reinterpret_cast<const char*>(A + row0 * lda);
    const char* r0 = MASK ? reinterpret_cast<const char*>(R + row0 * ldr) : nullptr;
    const int nk = KD / BKS;
    const char* b0 = reinterpret_cast<const char*>(
        Bp + (size_t)(lid % n_col_tiles) * nk * (kPlanes * S::BN * BKS));

    const int li = lane & 31, lk = lane >> 5;
    struct Operands {
        bf16x8 a[kPlanes][S::TM], b[kPlanes][S::TN];
    };
    auto read_operands = [&](Operands& o, const uint16_t* as, const uint16_t* bs) {
#pragma unroll
        for (int p = 0; p < kPlanes; ++p) {
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
                o.a[p][tm] = *reinterpret_cast<const bf16x8*>(
                    &as[p * S::BM * LDR + ((wm * S::TM + tm) * 32 + li) * LDR + 8 * lk]);
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn)
                o.b[p][tn] = *reinterpret_cast<const bf16x8*>(
                    &bs[p * S::BN * LDR + ((wn * S::TN + tn) * 32 + li) * LDR + 8 * lk]);
        }
    };
    auto mma = [&](const Operands& o) {
        // smallest partial products first; consecutive MFMAs go to different accumulators
        constexpr int pa[6] = {2, 0, 1, 1, 0, 0};
        constexpr int pb[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
        for (int q = 0; q < 6; ++q)
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < S::TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        o.a[pa[q]][tm], o.b[pb[q]][tn], acc[tm][tn], 0, 0, 0);
    };

    // The MFMAs of step i run on operands that were read from LDS during step i - 1, while the
    // operands of step i + 1 are read and the tiles of step i + 2 are split and written over the
    // buffer that step i came from.  Two steps per trip keep every buffer and register set static.
    Stage<S, MASK> s0, s1;
    Operands o0, o1;
    // a step beyond the last one loads the last one again (never stored): no branch around loads
    auto load = [&](Stage<S, MASK>& st, int step) {
        const int sc = step < nk ? step : nk - 1;
        const size_t oa = (size_t)sc * (BKS * 4), ob = (size_t)sc * (kPlanes * S::BN * BKS * 2);
        st.load(a0 + oa, r0 + oa, b0 + ob, aoff, roff, boff);
    };
    load(s0, 0);
    load(s1, 1);
    s0.store(As[0], Bs[0], apos, bpos, b_on);
    load(s0, 2);
    if (nk > 1) s1.store(As[1], Bs[1], apos, bpos, b_on);
    load(s1, 3);
    __syncthreads();
    read_operands(o0, As[0], Bs[0]);
    __syncthreads();
    // main trips: both steps have two successors, so nothing in them is conditional and every
    // wait can be counted (a set's loads are awaited with the other set's five still in flight)
    int i = 0;
    for (; i + 3 < nk; i += 2) {
        read_operands(o1, As[1], Bs[1]);
        mma(o0);
        s0.store(As[0], Bs[0], apos, bpos, b_on);
        load(s0, i + 4);
        __syncthreads();
        read_operands(o0, As[0], Bs[0]);
        mma(o1);
        s1.store(As[1], Bs[1], apos, bpos, b_on);
        load(s1, i + 5);
        __syncthreads();
    }
    // the last one to three steps
    const int rem = nk - i;
    if (rem >= 2) read_operands(o1, As[1], Bs[1]);
    mma(o0);
    if (rem >= 3) s0.store(As[0], Bs[0], apos, bpos, b_on);
    if (rem >= 2) {
        __syncthreads();
        if (rem >= 3) read_operands(o0, As[0], Bs[0]);
        mma(o1);
        if (rem >= 3) mma(o0);
    }

    // D layout: lane l, register v -> row 8 (v / 4) + 4 (l / 32) + v % 4, col l % 32
    const int wmu = __builtin_amdgcn_readfirstlane(wm), wnu = __builtin_amdgcn_readfirstlane(wn);
    const uint32_t lane_off = (uint32_t)(4 * lk) * (uint32_t)ldc + (uint32_t)li;
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn) {
            const int ct = col0 + (wnu * S::TN + tn) * 32;
            const int64_t rt = row0 + (wmu * S::TM + tm) * 32;
            float* tile = C + rt * ldc + ct;
            if (rt + 32 <= n && ct + 32 <= MD && ldc < (1 << 22)) {
                // nothing to clip: a scalar base per register, one 32-bit lane offset
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    // as signed integers, max(bits, 0) clears exactly the values with the sign set
                    int x = __float_as_int(acc[tm][tn][v]);
                    if (RELU) x = x > 0 ? x : 0;
                    tile[(int64_t)(8 * (v / 4) + (v % 4)) * ldc + lane_off] = __int_as_float(x);
                }
            } else if (ct + li < MD) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t r = rt + 8 * (v / 4) + 4 * lk + (v % 4);
                    if (r < n) {
                        float x = acc[tm][tn][v];
                        if (RELU) x = x > 0.f ? x : 0.f;
                        C[r * ldc + ct + li] = x;
                    }
                }
            }
        }
}

// ---- weight gradient: P[slab][KD x MD] = A[rows of slab][KD]^T * (B (.) 1[R > 0])[rows][MD] -----
// The reduction runs over node rows, the slow index of both operands in memory, while the bf16
// MFMA wants eight consecutive reduction indices per lane.  The tiles are therefore staged as
// they lie (row-major [node row][feature], three bf16 planes each, plain 8-byte writes) and the
// transposition is done by the LDS read: ds_read_b64_tr_b16 hands lane i of a group of 16 lanes
// element i % 4 of the 8 bytes addressed by lanes i / 4, i / 4 + 4, i / 4 + 8 and i / 4 + 12, so
// with lane s of the group pointing at row s / 4, features 4 (s % 4) .. + 3, every lane receives
// its own feature at four consecutive rows; two such reads are one MFMA operand.
// LDS rows are 320 bytes (128 features + pad): two groups of 16 lanes are served together (64
// banks), that is four rows of 64 bytes, which a pitch of 16 banks modulo 64 keeps apart (with
// 288-byte rows a third of the LDS cycles were bank conflicts).
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
constexpr int LDW = 128 + 32;            // halfwords per staged row
constexpr int kWPlane = BKS * LDW;       // halfwords per plane of a tile

__device__ inline bf16x8 read_transposed(const uint16_t* p)
{
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)p);
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(p + 4 * LDW));
    const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    bf16x8 o;
    __builtin_memcpy(&o, &v, 16);
    return o;
}

template <bool MASK>
__global__ __launch_bounds__(kBlock, 2) void wgrad_split_kernel(
    const float* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb,
    const float* __restrict__ R, int64_t ldr, float* __restrict__ P, int KD, int MD,
    int64_t rows_per_slab, int64_t n_rows, int n_i_tiles, int n_j_tiles)
{
    constexpr int TM = 2, TN = 2;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][kPlanes * kWPlane];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][kPlanes * kWPlane];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int tiles = n_i_tiles * n_j_tiles;
    const unsigned lid = xcd_local_index(blockIdx.x, gridDim.x);
    const int64_t slab = lid / tiles;
    const int t = (int)(lid % tiles);
    const int i0 = (t / n_j_tiles) * 128, j0 = (t % n_j_tiles) * 128;
    const int64_t r_begin = slab * rows_per_slab;
    const int64_t r_end = (r_begin + rows_per_slab) < n_rows ? (r_begin + rows_per_slab) : n_rows;
    const int nk = (int)((r_end - r_begin) / BKS);  // whole steps: the caller sees to it

    floatx16 acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

    // staging: thread -> rows tid / 32 and tid / 32 + 8 of the step, features 4 (tid % 32) .. + 3
    const int srow = tid >> 5, scol = 4 * (tid & 31);
    uint32_t aoff[2], boff[2], roff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
        aoff[p] = (uint32_t)(srow + 8 * p) * (uint32_t)lda * 4u + 4u * scol;
        boff[p] = (uint32_t)(srow + 8 * p) * (uint32_t)ldb * 4u + 4u * scol;
        roff[p] = MASK ? (uint32_t)(srow + 8 * p) * (uint32_t)ldr * 4u + 4u * scol : 0u;
    }
    const int spos = srow * LDW + scol;
    const char* a0 = reinterpret_cast<const char*>(A + r_begin * lda + i0);
    const char* b0 = reinterpret_cast<const char*>(B + r_begin * ldb + j0);
    const char* m0 = MASK ? reinterpret_cast<const char*>(R + r_begin * ldr + j0) : nullptr;
    const size_t step_a = (size_t)BKS * 4 * (size_t)lda, step_b = (size_t)BKS * 4 * (size_t)ldb,
                 step_r = (size_t)BKS * 4 * (size_t)ldr;

    struct Regs {
        float4 a[2], b[2], r[2];
    };
    // a step beyond the last one loads the last one again (never stored): no branch around loads
    auto load = [&](Regs& g, int step) {
        const size_t sc = (size_t)(step < nk ? step : nk - 1);
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            g.a[p] = *reinterpret_cast<const float4*>(a0 + sc * step_a + aoff[p]);
            g.b[p] = *reinterpret_cast<const float4*>(b0 + sc * step_b + boff[p]);
            if (MASK) g.r[p] = *reinterpret_cast<const float4*>(m0 + sc * step_r + roff[p]);
        }
    };
    auto store = [&](const Regs& g, uint16_t* as, uint16_t* bs) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            uint16_t* qa = as + spos + p * 8 * LDW;
            split_store<false>(g.a[p], g.a[p], qa, qa + kWPlane, qa + 2 * kWPlane);
            uint16_t* qb = bs + spos + p * 8 * LDW;
            split_store<MASK>(g.b[p], g.r[p], qb, qb + kWPlane, qb + 2 * kWPlane);
        }
    };
    // operand reads: lane -> 16-lane group (feature block, reduction half), place in the group
    const int grp = lane >> 4, gs = lane & 15;
    const int rpos = (8 * (grp >> 1) + (gs >> 2)) * LDW + 16 * (grp & 1) + 4 * (gs & 3);
    struct Operands {
        bf16x8 a[kPlanes][TM], b[kPlanes][TN];
    };
    auto read_operands = [&](Operands& o, const uint16_t* as, const uint16_t* bs) {
#pragma unroll
        for (int p = 0; p < kPlanes; ++p) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
                o.a[p][tm] = read_transposed(as + p * kWPlane + rpos + (wm * TM + tm) * 32);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                o.b[p][tn] = read_transposed(bs + p * kWPlane + rpos + (wn * TN + tn) * 32);
        }
    };
    auto mma = [&](const Operands& o) {
        constexpr int pa[6] = {2, 0, 1, 1, 0, 0};
        constexpr int pb[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
        for (int q = 0; q < 6; ++q)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        o.a[pa[q]][tm], o.b[pb[q]][tn], acc[tm][tn], 0, 0, 0);
    };

    if (nk > 0) {
        // the pipeline of the row-block kernel: MFMAs of step i on operands read during step
        // i - 1, operands of step i + 1 read, tiles of step i + 2 split and written, loads two
        // more steps ahead
        Regs g0, g1;
        Operands o0, o1;
        load(g0, 0);
        load(g1, 1);
        store(g0, As[0], Bs[0]);
        load(g0, 2);
        if (nk > 1) store(g1, As[1], Bs[1]);
        load(g1, 3);
        __syncthreads();
        read_operands(o0, As[0], Bs[0]);
        __syncthreads();
        int i = 0;
        for (; i + 3 < nk; i += 2) {
            read_operands(o1, As[1], Bs[1]);
            mma(o0);
            store(g0, As[0], Bs[0]);
            load(g0, i + 4);
            __syncthreads();
            read_operands(o0, As[0], Bs[0]);
            mma(o1);
            store(g1, As[1], Bs[1]);
            load(g1, i + 5);
            __syncthreads();
        }
        const int rem = nk - i;
        if (rem >= 2) read_operands(o1, As[1], Bs[1]);
        mma(o0);
        if (rem >= 3) store(g0, As[0], Bs[0]);
        if (rem >= 2) {
            __syncthreads();
            if (rem >= 3) read_operands(o0, As[0], Bs[0]);
            mma(o1);
            if (rem >= 3) mma(o0);
        }
    }

    // D layout: lane l, register v -> row 8 (v / 4) + 4 (l / 32) + v % 4, col l % 32
    const int li = lane & 31, lk = lane >> 5;
    float* out = P + (size_t)slab * KD * MD;
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int j = j0 + (wn * TN + tn) * 32 + li;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + (wm * TM + tm) * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                out[(size_t)i * MD + j] = acc[tm][tn][v];
            }
        }
}

// C[n x out_dim] = (A (.) mask)[n x red_dim] * Wop, Wop[kk][j] = transpose_w ? W[kk][j] : W[j][kk]
template <class S>
int launch_rowblock_split(bool relu, const float* A, int64_t lda, const float* W, int64_t ldw,
                          int w_rows, int w_cols, bool transpose_w, float* C, int64_t ldc, int64_t n,
                          int red_dim, int out_dim, const float* R, int64_t ldr, hipStream_t s)
{
    const int nct = (int)ceil_div(out_dim, S::BN);
    const int64_t grid = ceil_div(n, S::BM) * nct;
    if (grid <= 0) return MIXGCN_OK;
    if (grid > 0x7FFFFFFF) return fail(MIXGCN_EINVAL, "update: too many row tiles");
    const int out_rows = nct * S::BN, out_cols = red_dim;
    const size_t plane = (size_t)out_rows * out_cols;
    void* scratch = nullptr;
    MIXGCN_TRY(get_scratch(2, kPlanes * plane * sizeof(uint16_t), &scratch));
    uint16_t* planes = (uint16_t*)scratch;
    hipLaunchKernelGGL(split3_weights_kernel, dim3((unsigned)ceil_div((int64_t)plane, kBlock)),
                       dim3(kBlock), 0, s, W, ldw, w_rows, w_cols, transpose_w ? 1 : 0, planes,
                       out_rows, out_cols, S::BN);
#define MIXGCN_ROWBLOCK(RELU, MASK)                                                               \
    hipLaunchKernelGGL((rowblock_split_kernel<S, RELU, MASK>), dim3((unsigned)grid), dim3(kBlock), \
                       0, s, A, lda, planes, C, ldc, n, red_dim, out_dim, R, ldr, nct)
    if (R) MIXGCN_ROWBLOCK(false, true);
    else if (relu) MIXGCN_ROWBLOCK(true, false);
    else MIXGCN_ROWBLOCK(false, false);
#undef MIXGCN_ROWBLOCK
    return MIXGCN_OK;
}

}  // namespace

bool update_split_applies(int op, int64_t lda, int64_t ldb, int64_t ldr, int64_t n, int32_t k,
                          int32_t m)
{
    if (n <= 0) return false;
    if (lda >= (1 << 22) || ldr >= (1 << 22)) return false;  // 32-bit offsets inside a tile
    if (op == MIXGCN_OP_WGRAD && ldb >= (1 << 22)) return false;
    // outputs of at most 64 columns and reductions of fewer than four steps are bound by their
    // memory traffic on either path
    if (op == MIXGCN_OP_FWD || op == MIXGCN_OP_FWD_RELU) return m > 64 && k >= 64 && k % BKS == 0;
    if (op == MIXGCN_OP_DGRAD) return k > 64 && m >= 64 && m % BKS == 0;
    // the weight gradient: whole 128 x 128 tiles, and at least one whole step of rows (a remainder
    // of fewer than 16 rows goes to the fp32 MFMA kernel)
    if (op == MIXGCN_OP_WGRAD) return k % 128 == 0 && m % 128 == 0 && n >= BKS;
    return false;
}

// dW[k x m] = beta dW + A[n x k]^T (B (.) mask)[n x m] for whole 128 x 128 tiles and a row count of
// whole steps
static int launch_wgrad_split(const float* A, int64_t lda, const float* B, int64_t ldb, float* C,
                              int64_t ldc, int64_t n, int32_t k, int32_t m, const float* R,
                              int64_t ldr, float beta, hipStream_t s, Timer* timer)
{
    const int nit = k / 128, njt = m / 128, tiles = nit * njt;
    int64_t n_slabs = ceil_div(n, 1024);
    const int64_t cap = tiles >= 1024 ? 1 : 1024 / tiles;
    if (n_slabs > cap) n_slabs = cap;
    if (n_slabs < 1) n_slabs = 1;
    const int64_t rows_per_slab = ceil_div(ceil_div(n, n_slabs), BKS) * BKS;
    n_slabs = ceil_div(n, rows_per_slab);
    const int64_t cells = (int64_t)k * m;
    void* scratch = nullptr;
    MIXGCN_TRY(get_scratch(0, (size_t)n_slabs * cells * sizeof(float), &scratch));
    float* P = (float*)scratch;
    const unsigned grid = (unsigned)(n_slabs * tiles);
    if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateWgrad, s));
    if (R)
        hipLaunchKernelGGL((wgrad_split_kernel<true>), dim3(grid), dim3(kBlock), 0, s, A, lda, B, ldb, R,
                           ldr, P, k, m, rows_per_slab, n, nit, njt);
    else
        hipLaunchKernelGGL((wgrad_split_kernel<false>), dim3(grid), dim3(kBlock), 0, s, A, lda, B, ldb,
                           R, ldr, P, k, m, rows_per_slab, n, nit, njt);
    if (timer) MIXGCN_TRY(timer->end(s));
    return launch_wgrad_reduce(P, n_slabs, cells, m, C, ldc, beta, s);
}

int launch_update_split(int op, const float* A, int64_t lda, const float* W, int64_t ldw, float* C,
                        int64_t ldc, int64_t n, int32_t k, int32_t m, const float* R, int64_t ldr,
                        float beta, hipStream_t s, Timer* timer)
{
    if (op == MIXGCN_OP_WGRAD) {
        // here W is the upstream gradient [n x m]; n must be a multiple of 16
        MIXGCN_TRY(launch_wgrad_split(A, lda, W, ldw, C, ldc, n, k, m, R, ldr, beta, s, timer));
        MIXGCN_HIP_TRY(hipGetLastError());
        return MIXGCN_OK;
    }
    if (op == MIXGCN_OP_FWD || op == MIXGCN_OP_FWD_RELU) {
        // C[n x m] = A[n x k] W, W stored k x m: operand rows = output columns -> transposed split
        const bool relu = op == MIXGCN_OP_FWD_RELU;
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateFwd, s));
        MIXGCN_TRY((launch_rowblock_split<Shape128x128>(relu, A, lda, W, ldw, k, m, true, C, ldc, n, k,
                                                       m, nullptr, 0, s)));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else if (op == MIXGCN_OP_DGRAD) {
        // C[n x k] = (A (.) mask)[n x m] W^T, W stored k x m: operand rows = rows of W
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateDgrad, s));
        MIXGCN_TRY((launch_rowblock_split<Shape128x128>(false, A, lda, W, ldw, k, m, false, C, ldc, n,
                                                       m, k, R, ldr, s)));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else {
        return fail(MIXGCN_EINVAL, "update: this product has no split path");
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace mixgcn
