// Node update H' = sigma(Z W) (paper Algorithm 2, update phase) and the two dense products of
// its backward pass, dZ = dP W^T and dW = Z^T dP, on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32).  Row-block kernels: the node dimension is the long one, the feature
// dimensions are at most a few hundred, so a workgroup owns 128 node rows (forward / dgrad) or
// a slab of node rows (wgrad, split over the reduction and combined in fp64 by a second kernel).
#include <type_traits>

#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;          // reduction depth staged per step
// Workgroups per CU that the register allocation of each kernel is held to (measured best of
// 2, 3, 4 on the 128 x 128 shapes): the masked row-block kernel keeps more values live.
constexpr int kRowblockMinBlocks = 3, kRowblockMaskedMinBlocks = 2, kWgradMinBlocks = 4;
constexpr int kLdsPad = 4;      // row stride of the staged tiles = tile width + 4 floats

// Tile shape: WM x WN waves (4 in total), each owning TM x TN accumulator tiles of 32 x 32.
template <int WM_, int WN_, int TM_, int TN_>
struct Shape {
    static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
    static constexpr int BM = WM * TM * 32;  // extent along the A-operand free dimension
    static constexpr int BN = WN * TN * 32;  // extent along the B-operand free dimension
    static_assert(WM * WN == 4, "four waves per block");
};
using Shape128x128 = Shape<2, 2, 2, 2>;
using Shape128x32 = Shape<4, 1, 1, 1>;

// acc += As[kk][a-rows] (x) Bs[kk][b-cols] over the BK staged reduction steps.  The operand
// registers of step k2 + 2 are read from LDS before the MFMAs of step k2 are issued.
// MFMA 32x32x2 operand layout: lane l supplies A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32].
template <class S>
__device__ inline void mma_step(const float* As, const float* Bs, int wm, int wn, int lane,
                                floatx16 (&acc)[S::TM][S::TN])
{
    constexpr int LDA = S::BM + kLdsPad, LDB = S::BN + kLdsPad;
    const int li = lane & 31, lk = lane >> 5;
    const float* ap = As + lk * LDA + wm * S::TM * 32 + li;
    const float* bp = Bs + lk * LDB + wn * S::TN * 32 + li;
    float a[2][S::TM], b[2][S::TN];
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm) a[0][tm] = ap[tm * 32];
#pragma unroll
    for (int tn = 0; tn < S::TN; ++tn) b[0][tn] = bp[tn * 32];
#pragma unroll
    for (int k2 = 0; k2 < BK; k2 += 2) {
        const int cur = (k2 >> 1) & 1, nxt = cur ^ 1;
        if (k2 + 2 < BK) {
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm) a[nxt][tm] = ap[(k2 + 2) * LDA + tm * 32];
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn) b[nxt][tn] = bp[(k2 + 2) * LDB + tn * 32];
        }
#pragma unroll
        for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][tm], b[cur][tn],
                                                                   acc[tm][tn], 0, 0, 0);
        // keep the order written here: the LDS reads of step k2 + 2 go out before the MFMAs of
        // step k2, so their latency hides behind the matrix pipe instead of in front of it
        __builtin_amdgcn_sched_group_barrier(0x100, S::TM + S::TN, 0);  // DS reads
        __builtin_amdgcn_sched_group_barrier(0x008, S::TM * S::TN, 0);  // MFMAs
    }
}

// One 16-byte piece of an operand tile on its way from global memory to LDS.  issue() only
// starts the loads (addresses are clamped into the matrix, so they are unconditional and
// nothing waits on them); value() applies the zero fill outside [0, rows) x [0, cols) and the
// optional ReLU-derivative mask x * 1[R > 0] when the piece is written to LDS one step later.
// Feature tensors are fp32 (float) or bf16 (uint16_t, widened to fp32 on the way to LDS and
// rounded to nearest even on the way out); weights are always fp32.
template <typename T>
struct Raw4;
template <>
struct Raw4<float> {
    float4 q;
    __device__ inline float4 widen() const { return q; }
};
template <>
struct Raw4<uint16_t> {
    uint2 q;
    __device__ inline float4 widen() const
    {
        return make_float4(__uint_as_float(q.x << 16), __uint_as_float(q.x & 0xFFFF0000u),
                           __uint_as_float(q.y << 16), __uint_as_float(q.y & 0xFFFF0000u));
    }
};

__device__ inline uint16_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ inline void store_elem(float* p, float x) { *p = x; }
__device__ inline void store_elem(uint16_t* p, float x) { *p = bf16_rne(x); }

template <bool MASK, typename T>
struct Piece {
    Raw4<T> v;
    Raw4<T> m;
    int nvalid;  // leading components inside the matrix (0..4)

    __device__ inline void issue(const T* __restrict__ M, int64_t ld, int64_t r, int c,
                                 int64_t rows, int cols, const T* __restrict__ R, int64_t ldr)
    {
        const bool ok = r < rows && c < cols;
        nvalid = ok ? (cols - c < 4 ? cols - c : 4) : 0;
        const int64_t rr = r < rows ? r : rows - 1;
        const int cc = c < cols ? c : 0;
        v = *reinterpret_cast<const Raw4<T>*>(M + rr * ld + cc);
        if (MASK) m = *reinterpret_cast<const Raw4<T>*>(R + rr * ldr + cc);
    }
    // CHECKED = false: the caller knows the piece lies wholly inside the matrix
    template <bool CHECKED = true>
    __device__ inline float4 value() const
    {
        float4 o = v.widen();
        if (MASK) {
            const float4 mm = m.widen();
            o.x = mm.x > 0.f ? o.x : 0.f;
            o.y = mm.y > 0.f ? o.y : 0.f;
            o.z = mm.z > 0.f ? o.z : 0.f;
            o.w = mm.w > 0.f ? o.w : 0.f;
        }
        if (CHECKED && nvalid < 4) {
            if (nvalid < 1) o.x = 0.f;
            if (nvalid < 2) o.y = 0.f;
            if (nvalid < 3) o.z = 0.f;
            o.w = 0.f;
        }
        return o;
    }
};

// ---- fast path: tiles that lie wholly inside their matrices, fp32 -------------------------------
// A vector instruction costs the SIMD four cycles during which its matrix core idles (measured:
// MFMA and vector work of a SIMD do not overlap on this part), so the inner loop of a tile with
// nothing to clip is written to need almost none: every global address is a scalar base (stepped
// with scalar arithmetic) plus a per-thread 32-bit offset that never changes, and every LDS
// address is a per-thread base plus an immediate.  LDS accesses go through volatile pointers so
// that the compiler keeps them as single instructions with 16-bit immediates: fused into
// two-address forms (8-bit offsets) they would need a vector add per pair to rebase.
typedef __attribute__((address_space(3))) float lds_float;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) floatx4 lds_floatx4;

// One operand tile of a step: E free indices x BK reduction indices, staged to LDS as [k][e].
//   TRANSPOSED: memory is [e][k]; an item is 4 consecutive k of one e (4 single-word writes)
//   DIRECT:     memory is [k][e]; an item is 4 consecutive e of one k (one 16-byte write)
// Item `tid` of pass p lies a whole number of rows (of memory) after item `tid` of pass 0, so one
// 32-bit offset per thread serves every pass: the pass only moves the uniform base.
template <int E, bool TRANSPOSED, bool MASK>
struct FastTile {
    static constexpr int LD = E + kLdsPad;
    static constexpr int ITEMS = TRANSPOSED ? E * (BK / 4) : BK * (E / 4);
    static constexpr int PASSES = (ITEMS + kBlock - 1) / kBlock;
    // rows of memory between passes, and floats of LDS between passes
    static constexpr int PASS_ROWS = TRANSPOSED ? kBlock / (BK / 4) : kBlock / (E / 4);
    static constexpr int PASS_LDS = TRANSPOSED ? PASS_ROWS : PASS_ROWS * LD;
    static_assert(PASSES == 1 || ITEMS % kBlock == 0, "whole passes");
    uint32_t goff, moff;  // byte offset of the thread's item in the operand / the mask reference
    int lpos;             // float index of the item in the LDS tile
    bool on;              // the thread has an item (tiles smaller than one pass)
    float4 v[PASSES], m[PASSES];

    __device__ inline void init(int tid, uint32_t pitch, uint32_t pitch_r)
    {
        on = (ITEMS % kBlock == 0) || tid < ITEMS;
        const int it = on ? tid : 0;
        if (TRANSPOSED) {
            const int e = it / (BK / 4), kq = 4 * (it % (BK / 4));
            goff = (uint32_t)e * pitch + 4u * kq;
            moff = (uint32_t)e * pitch_r + 4u * kq;
            lpos = kq * LD + e;
        } else {
            const int kk = it / (E / 4), e = 4 * (it % (E / 4));
            goff = (uint32_t)kk * pitch + 4u * e;
            moff = (uint32_t)kk * pitch_r + 4u * e;
            lpos = kk * LD + e;
        }
    }
    // base, base_r: uniform addresses of the step's tile; pitch in bytes
    __device__ inline void load(const char* base, const char* base_r, size_t pitch, size_t pitch_r)
    {
        if (on) {
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                v[p] = *reinterpret_cast<const float4*>(base + p * PASS_ROWS * pitch + goff);
                if (MASK)
                    m[p] = *reinterpret_cast<const float4*>(base_r + p * PASS_ROWS * pitch_r + moff);
            }
        }
    }
    __device__ static inline float keep(float x, float r) { return MASK ? (r > 0.f ? x : 0.f) : x; }
    __device__ inline void store(float* tile) const
    {
        if (on) {
#pragma unroll
            for (int p = 0; p < PASSES; ++p) {
                const float x0 = keep(v[p].x, m[p].x), x1 = keep(v[p].y, m[p].y);
                const float x2 = keep(v[p].z, m[p].z), x3 = keep(v[p].w, m[p].w);
                if (TRANSPOSED) {
                    volatile lds_float* o = (volatile lds_float*)(tile + lpos + p * PASS_LDS);
                    o[0 * LD] = x0;
                    o[1 * LD] = x1;
                    o[2 * LD] = x2;
                    o[3 * LD] = x3;
                } else {
                    const floatx4 q = {x0, x1, x2, x3};
                    *(lds_floatx4*)(tile + lpos + p * PASS_LDS) = q;
                }
            }
        }
    }
};

// mma_step with single-word LDS reads at immediate offsets.
template <class S>
__device__ inline void mma_step_fast(const float* As, const float* Bs, int wm, int wn, int lane,
                                     floatx16 (&acc)[S::TM][S::TN])
{
    constexpr int LDA = S::BM + kLdsPad, LDB = S::BN + kLdsPad;
    const int li = lane & 31, lk = lane >> 5;
    const volatile lds_float* ap = (const volatile lds_float*)(As + lk * LDA + wm * S::TM * 32 + li);
    const volatile lds_float* bp = (const volatile lds_float*)(Bs + lk * LDB + wn * S::TN * 32 + li);
    float a[2][S::TM], b[2][S::TN];
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm) a[0][tm] = ap[tm * 32];
#pragma unroll
    for (int tn = 0; tn < S::TN; ++tn) b[0][tn] = bp[tn * 32];
#pragma unroll
    for (int k2 = 0; k2 < BK; k2 += 2) {
        const int cur = (k2 >> 1) & 1, nxt = cur ^ 1;
        if (k2 + 2 < BK) {
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm) a[nxt][tm] = ap[(k2 + 2) * LDA + tm * 32];
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn) b[nxt][tn] = bp[(k2 + 2) * LDB + tn * 32];
        }
#pragma unroll
        for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn)
                acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[cur][tm], b[cur][tn],
                                                                   acc[tm][tn], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, S::TM + S::TN, 0);  // DS reads of step k2 + 2
        __builtin_amdgcn_sched_group_barrier(0x008, S::TM * S::TN, 0);  // MFMAs of step k2
    }
}

// The reduction loop of the fast path: nk full steps, LDS double buffered with compile-time
// buffer indices (two steps per trip) so that buffer offsets fold into the immediates.
template <class S, class TA, class TB, class LoadFn>
__device__ inline void fast_reduction(float (&As)[2][BK * (S::BM + kLdsPad)],
                                      float (&Bs)[2][BK * (S::BN + kLdsPad)], TA& ta, TB& tb,
                                      LoadFn load, int64_t nk, int wm, int wn, int lane,
                                      floatx16 (&acc)[S::TM][S::TN])
{
    load((int64_t)0);
    ta.store(As[0]);
    tb.store(Bs[0]);
    __syncthreads();
    int64_t s = 0;
    while (s + 2 < nk) {
        load(s + 1);
        mma_step_fast<S>(As[0], Bs[0], wm, wn, lane, acc);
        ta.store(As[1]);
        tb.store(Bs[1]);
        __syncthreads();
        load(s + 2);
        mma_step_fast<S>(As[1], Bs[1], wm, wn, lane, acc);
        ta.store(As[0]);
        tb.store(Bs[0]);
        __syncthreads();
        s += 2;
    }
    if (s + 1 < nk) {
        load(s + 1);
        mma_step_fast<S>(As[0], Bs[0], wm, wn, lane, acc);
        ta.store(As[1]);
        tb.store(Bs[1]);
        __syncthreads();
        mma_step_fast<S>(As[1], Bs[1], wm, wn, lane, acc);
    } else {
        mma_step_fast<S>(As[0], Bs[0], wm, wn, lane, acc);
    }
}

// Workgroups are dealt round-robin to the 8 XCDs.  This maps the hardware block index to a
// logical one such that consecutive logical indices run on the same XCD, so tiles that share
// an operand (the column tiles of one row block) find it in that XCD's L2.
__device__ inline unsigned xcd_local_index(unsigned bid, unsigned grid)
{
    const unsigned q = grid / 8, rem = grid % 8, x = bid % 8;
    return x * q + (x < rem ? x : rem) + bid / 8;
}

// ---- row-block kernel: C[n x MD] = op(A)[n x KD] * Bop[KD x MD] -------------------------------
//   B_TRANS = false: Bop[kk][j] = B[kk * ldb + j]   (forward:  Z W)
//   B_TRANS = true : Bop[kk][j] = B[j * ldb + kk]   (dgrad:   dP W^T with W stored k x m)
//   MASK: A is multiplied by 1[R > 0] on the way in (dgrad of a ReLU layer).
// A is staged transposed (reduction-major) so that the MFMA operand reads are unit-stride.
// LDS tiles are double buffered: one barrier per reduction step.
template <class S, bool B_TRANS, bool RELU, bool MASK, typename T>
__global__ __launch_bounds__(kBlock, MASK ? kRowblockMaskedMinBlocks : kRowblockMinBlocks) void
rowblock_gemm_kernel(
    const T* __restrict__ A, int64_t lda, const float* __restrict__ B, int64_t ldb,
    T* __restrict__ C, int64_t ldc, int64_t n, int KD, int MD, const T* __restrict__ R,
    int64_t ldr, int n_col_tiles)
{
    constexpr int LDA = S::BM + kLdsPad, LDB = S::BN + kLdsPad;
    __shared__ float As[2][BK * LDA];
    __shared__ float Bs[2][BK * LDB];
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

    // staging maps: "strided" = 4 consecutive reduction indices of one row/col per thread
    constexpr int A_PASSES = S::BM / 64;                       // 64 rows per pass
    constexpr int BT_PASSES = S::BN / 64 > 0 ? S::BN / 64 : 1; // B_TRANS: 64 cols per pass
    constexpr int BN_F4 = S::BN / 4;                           // float4 per staged B row
    constexpr int B_ROWS_PER_PASS = kBlock / BN_F4;
    constexpr int B_PASSES = (BK + B_ROWS_PER_PASS - 1) / B_ROWS_PER_PASS;
    Piece<MASK, T> ra[A_PASSES];
    Piece<false, float> rb[B_TRANS ? BT_PASSES : B_PASSES];

    auto issue_tiles = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p)
            ra[p].issue(A, lda, row0 + p * 64 + tid / 4, k0 + 4 * (tid & 3), n, KD, R, ldr);
        if (B_TRANS) {
#pragma unroll
            for (int p = 0; p < BT_PASSES; ++p) {
                const int j = p * 64 + tid / 4;
                rb[p].issue(B, ldb, col0 + (j < S::BN ? j : 0), k0 + 4 * (tid & 3), MD, KD, nullptr, 0);
            }
        } else {
#pragma unroll
            for (int p = 0; p < B_PASSES; ++p) {
                const int kk = p * B_ROWS_PER_PASS + tid / BN_F4;
                rb[p].issue(B, ldb, k0 + (kk < BK ? kk : 0), col0 + 4 * (tid % BN_F4), KD, MD, nullptr, 0);
            }
        }
    };
    // CHECKED = false when every piece of the two tiles lies inside its matrix (uniform): the
    // zero fill then costs no vector ALU work next to the MFMAs
    auto store_tiles_as = [&](float* as, float* bs, auto checked) {
        constexpr bool CHECKED = decltype(checked)::value;
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int i = p * 64 + tid / 4, kq = 4 * (tid & 3);
            const float4 v = ra[p].template value<CHECKED>();
            as[(kq + 0) * LDA + i] = v.x;
            as[(kq + 1) * LDA + i] = v.y;
            as[(kq + 2) * LDA + i] = v.z;
            as[(kq + 3) * LDA + i] = v.w;
        }
        if (B_TRANS) {
#pragma unroll
            for (int p = 0; p < BT_PASSES; ++p) {
                const int j = p * 64 + tid / 4, kq = 4 * (tid & 3);
                if (j < S::BN) {
                    const float4 v = rb[p].template value<CHECKED>();
                    bs[(kq + 0) * LDB + j] = v.x;
                    bs[(kq + 1) * LDB + j] = v.y;
                    bs[(kq + 2) * LDB + j] = v.z;
                    bs[(kq + 3) * LDB + j] = v.w;
                }
            }
        } else {
#pragma unroll
            for (int p = 0; p < B_PASSES; ++p) {
                const int kk = p * B_ROWS_PER_PASS + tid / BN_F4;
                if (kk < BK)
                    *reinterpret_cast<float4*>(&bs[kk * LDB + 4 * (tid % BN_F4)]) =
                        rb[p].template value<CHECKED>();
            }
        }
    };
    const bool tile_inside = row0 + S::BM <= n && col0 + S::BN <= MD;
    auto store_tiles = [&](float* as, float* bs, int k0) {
        if (tile_inside && k0 + BK <= KD) store_tiles_as(as, bs, std::false_type{});
        else store_tiles_as(as, bs, std::true_type{});
    };

    const int nk = (KD + BK - 1) / BK;
    // every piece inside its matrix, whole reduction steps, 32-bit offsets within a tile
    const bool fast = std::is_same<T, float>::value && tile_inside && KD % BK == 0 &&
                      lda < (1 << 22) && ldb < (1 << 22) && ldr < (1 << 22);
    if (fast) {
        FastTile<S::BM, true, MASK> ta;
        FastTile<S::BN, B_TRANS, false> tb;
        ta.init(tid, (uint32_t)lda * 4u, (uint32_t)ldr * 4u);
        tb.init(tid, (uint32_t)ldb * 4u, 0u);
        const char* a0 = reinterpret_cast<const char*>(A + row0 * lda);
        const char* r0 = MASK ? reinterpret_cast<const char*>(R + row0 * ldr) : nullptr;
        const char* b0 = reinterpret_cast<const char*>(B_TRANS ? B + (int64_t)col0 * ldb : B + col0);
        const size_t b_step = B_TRANS ? (size_t)BK * 4 : (size_t)BK * 4 * (size_t)ldb;
        auto load = [&](int64_t st) {
            ta.load(a0 + (size_t)st * (BK * 4), r0 + (size_t)st * (BK * 4), (size_t)lda * 4,
                    (size_t)ldr * 4);
            tb.load(b0 + (size_t)st * b_step, nullptr, (size_t)ldb * 4, 0);
        };
        fast_reduction<S>(As, Bs, ta, tb, load, (int64_t)nk, wm, wn, lane, acc);
    } else {
        issue_tiles(0);
        store_tiles(As[0], Bs[0], 0);
        __syncthreads();
        for (int i = 0; i < nk; ++i) {
            const int cur = i & 1;
            if (i + 1 < nk) issue_tiles((i + 1) * BK);
            mma_step<S>(As[cur], Bs[cur], wm, wn, lane, acc);
            if (i + 1 < nk) store_tiles(As[cur ^ 1], Bs[cur ^ 1], (i + 1) * BK);
            __syncthreads();
        }
    }

    // D layout of the 32x32 MFMA: lane l, register v -> row 8*(v/4) + 4*(l/32) + v%4, col l%32
    const int li = lane & 31, lk = lane >> 5;
    if (tile_inside) {
        // no bounds to test: a scalar base per 32 x 32 tile and register, one 32-bit lane offset
        const int wmu = __builtin_amdgcn_readfirstlane(wm), wnu = __builtin_amdgcn_readfirstlane(wn);
        const uint32_t lane_off = (uint32_t)(4 * lk) * (uint32_t)ldc + (uint32_t)li;
#pragma unroll
        for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn) {
                T* tile = C + (row0 + (wmu * S::TM + tm) * 32) * ldc + col0 + (wnu * S::TN + tn) * 32;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float x = acc[tm][tn][v];
                    if (RELU) x = fmaxf(x, 0.f);
                    store_elem(tile + (int64_t)(8 * (v / 4) + (v % 4)) * ldc + lane_off, x);
                }
            }
        return;
    }
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn) {
            const int c = col0 + (wn * S::TN + tn) * 32 + li;
            if (c >= MD) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = row0 + (wm * S::TM + tm) * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (r < n) {
                    float x = acc[tm][tn][v];
                    if (RELU) x = x > 0.f ? x : 0.f;
                    store_elem(&C[r * ldc + c], x);
                }
            }
        }
}

// ---- slab kernel: P[slab][KD x MD] = A[rows of slab][KD]^T * (B (.) 1[R > 0])[rows][MD] --------
// Both operands are staged exactly as they lie in memory (node-major), which already is the
// reduction-major layout the MFMA operand reads want.
template <class S, bool MASK, typename T>
__global__ __launch_bounds__(kBlock, kWgradMinBlocks) void wgrad_slab_kernel(
    const T* __restrict__ A, int64_t lda, const T* __restrict__ B, int64_t ldb,
    const T* __restrict__ R, int64_t ldr, float* __restrict__ P, int64_t n, int KD, int MD,
    int64_t rows_per_slab, int n_i_tiles, int n_j_tiles)
{
    constexpr int LDA = S::BM + kLdsPad, LDB = S::BN + kLdsPad;
    __shared__ float As[2][BK * LDA];
    __shared__ float Bs[2][BK * LDB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / S::WN, wn = wave % S::WN;
    const int tiles = n_i_tiles * n_j_tiles;
    const unsigned lid = xcd_local_index(blockIdx.x, gridDim.x);
    const int64_t slab = lid / tiles;
    const int t = (int)(lid % tiles);
    const int i0 = (t / n_j_tiles) * S::BM, j0 = (t % n_j_tiles) * S::BN;
    const int64_t r_begin = slab * rows_per_slab;
    const int64_t r_end = (r_begin + rows_per_slab) < n ? (r_begin + rows_per_slab) : n;

    floatx16 acc[S::TM][S::TN];
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

    constexpr int AM_F4 = S::BM / 4, BN_F4 = S::BN / 4;
    constexpr int A_RPP = kBlock / AM_F4, B_RPP = kBlock / BN_F4;
    constexpr int A_PASSES = (BK + A_RPP - 1) / A_RPP, B_PASSES = (BK + B_RPP - 1) / B_RPP;
    Piece<false, T> ra[A_PASSES];
    Piece<MASK, T> rb[B_PASSES];

    auto issue_tiles = [&](int64_t r0) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int kk = p * A_RPP + tid / AM_F4;
            ra[p].issue(A, lda, r0 + (kk < BK ? kk : 0), i0 + 4 * (tid % AM_F4), r_end, KD, nullptr, 0);
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int kk = p * B_RPP + tid / BN_F4;
            rb[p].issue(B, ldb, r0 + (kk < BK ? kk : 0), j0 + 4 * (tid % BN_F4), r_end, MD, R, ldr);
        }
    };
    auto store_tiles_as = [&](float* as, float* bs, auto checked) {
        constexpr bool CHECKED = decltype(checked)::value;
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int kk = p * A_RPP + tid / AM_F4;
            if (kk < BK)
                *reinterpret_cast<float4*>(&as[kk * LDA + 4 * (tid % AM_F4)]) =
                    ra[p].template value<CHECKED>();
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int kk = p * B_RPP + tid / BN_F4;
            if (kk < BK)
                *reinterpret_cast<float4*>(&bs[kk * LDB + 4 * (tid % BN_F4)]) =
                    rb[p].template value<CHECKED>();
        }
    };
    const bool tile_inside = i0 + S::BM <= KD && j0 + S::BN <= MD;
    auto store_tiles = [&](float* as, float* bs, int64_t r0) {
        if (tile_inside && r0 + BK <= r_end) store_tiles_as(as, bs, std::false_type{});
        else store_tiles_as(as, bs, std::true_type{});
    };

    const bool fast = std::is_same<T, float>::value && tile_inside && r_begin < r_end &&
                      (r_end - r_begin) % BK == 0 && lda < (1 << 22) && ldb < (1 << 22) &&
                      ldr < (1 << 22);
    if (fast) {
        FastTile<S::BM, false, false> ta;
        FastTile<S::BN, false, MASK> tb;
        ta.init(tid, (uint32_t)lda * 4u, 0u);
        tb.init(tid, (uint32_t)ldb * 4u, (uint32_t)ldr * 4u);
        const char* a0 = reinterpret_cast<const char*>(A + r_begin * lda + i0);
        const char* b0 = reinterpret_cast<const char*>(B + r_begin * ldb + j0);
        const char* m0 = MASK ? reinterpret_cast<const char*>(R + r_begin * ldr + j0) : nullptr;
        auto load = [&](int64_t st) {
            ta.load(a0 + (size_t)st * BK * 4 * (size_t)lda, nullptr, (size_t)lda * 4, 0);
            tb.load(b0 + (size_t)st * BK * 4 * (size_t)ldb, m0 + (size_t)st * BK * 4 * (size_t)ldr,
                    (size_t)ldb * 4, (size_t)ldr * 4);
        };
        fast_reduction<S>(As, Bs, ta, tb, load, (r_end - r_begin) / BK, wm, wn, lane, acc);
    } else if (r_begin < r_end) {
        const int64_t nk = (r_end - r_begin + BK - 1) / BK;
        issue_tiles(r_begin);
        store_tiles(As[0], Bs[0], r_begin);
        __syncthreads();
        for (int64_t i = 0; i < nk; ++i) {
            const int cur = (int)(i & 1);
            if (i + 1 < nk) issue_tiles(r_begin + (i + 1) * BK);
            mma_step<S>(As[cur], Bs[cur], wm, wn, lane, acc);
            if (i + 1 < nk) store_tiles(As[cur ^ 1], Bs[cur ^ 1], r_begin + (i + 1) * BK);
            __syncthreads();
        }
    }
    float* out = P + (size_t)slab * KD * MD;
    const int li = lane & 31, lk = lane >> 5;
    if (tile_inside) {
        const int wmu = __builtin_amdgcn_readfirstlane(wm), wnu = __builtin_amdgcn_readfirstlane(wn);
        const uint32_t lane_off = (uint32_t)(4 * lk) * (uint32_t)MD + (uint32_t)li;
#pragma unroll
        for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn) {
                float* tile = out + (size_t)(i0 + (wmu * S::TM + tm) * 32) * MD + j0 +
                              (wnu * S::TN + tn) * 32;
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    tile[(size_t)(8 * (v / 4) + (v % 4)) * MD + lane_off] = acc[tm][tn][v];
            }
        return;
    }
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn) {
            const int j = j0 + (wn * S::TN + tn) * 32 + li;
            if (j >= MD) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + (wm * S::TM + tm) * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (i < KD) out[(size_t)i * MD + j] = acc[tm][tn][v];
            }
        }
}

// dW = beta * dW + sum over slabs.  A block owns 64 consecutive cells; its four waves each add
// every fourth slab (in slab order, fp64) and the four sums are combined in a fixed order, so
// the result is deterministic.
__global__ __launch_bounds__(kBlock) void wgrad_reduce_kernel(const float* __restrict__ P,
                                                              int64_t n_slabs, int64_t cells,
                                                              int MD, float* __restrict__ dW,
                                                              int64_t ldw, float beta)
{
    __shared__ double part[kBlock / kWave][kWave];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * kWave + lane;
    double s = 0.0;
    if (i < cells) {
        // eight loads in flight, added in the order of the plain loop
        constexpr int kStep = kBlock / kWave;
        int64_t b = w;
        for (; b + 7 * kStep < n_slabs; b += 8 * kStep) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = P[(size_t)(b + u * kStep) * cells + i];
#pragma unroll
            for (int u = 0; u < 8; ++u) s += (double)v[u];
        }
        for (; b < n_slabs; b += kStep) s += (double)P[(size_t)b * cells + i];
    }
    part[w][lane] = s;
    __syncthreads();
    if (w == 0 && i < cells) {
        const double t = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        float* o = dW + (i / MD) * ldw + (i % MD);
        *o = (float)(beta != 0.f ? (double)beta * (double)*o + t : t);
    }
}

// G <- G (.) 1[R > 0], four elements per thread (bf16: zeroing keeps the bits exact).
template <typename T>
__global__ __launch_bounds__(kBlock) void relu_mask_kernel(T* __restrict__ G, int64_t ldg,
                                                           const T* __restrict__ R, int64_t ldr,
                                                           int64_t n, int m4)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * m4) return;
    const int64_t r = i / m4;
    const int c = (int)(i % m4) * 4;
    T* gp = G + r * ldg + c;
    const float4 h = reinterpret_cast<const Raw4<T>*>(R + r * ldr + c)->widen();
    if (!(h.x > 0.f)) gp[0] = (T)0;
    if (!(h.y > 0.f)) gp[1] = (T)0;
    if (!(h.z > 0.f)) gp[2] = (T)0;
    if (!(h.w > 0.f)) gp[3] = (T)0;
}

template <class S, bool B_TRANS, typename T>
int launch_rowblock(bool relu, const T* A, int64_t lda, const float* B, int64_t ldb, T* C,
                    int64_t ldc, int64_t n, int KD, int MD, const T* R, int64_t ldr,
                    hipStream_t s)
{
    const int nct = (int)ceil_div(MD, S::BN);
    const int64_t grid = ceil_div(n, S::BM) * nct;
    if (grid <= 0) return MIXGCN_OK;
    if (grid > 0x7FFFFFFF) return fail(MIXGCN_EINVAL, "update: too many row tiles");
#define MIXGCN_ROWBLOCK(RELU, MASK)                                                              \
    hipLaunchKernelGGL((rowblock_gemm_kernel<S, B_TRANS, RELU, MASK, T>), dim3((unsigned)grid),   \
                       dim3(kBlock), 0, s, A, lda, B, ldb, C, ldc, n, KD, MD, R, ldr, nct)
    if (R) MIXGCN_ROWBLOCK(false, true);
    else if (relu) MIXGCN_ROWBLOCK(true, false);
    else MIXGCN_ROWBLOCK(false, false);
#undef MIXGCN_ROWBLOCK
    return MIXGCN_OK;
}

}  // namespace

int launch_relu_mask(int dtype, void* G, int64_t ldg, const void* R, int64_t ldr, int64_t n,
                     int32_t m, hipStream_t s)
{
    const int m4 = (m + 3) / 4;  // rows are padded to 16 bytes, so the last vector is in bounds
    const int64_t total = n * m4;
    if (total == 0) return MIXGCN_OK;
    const dim3 grid((unsigned)ceil_div(total, kBlock));
    if (dtype == MIXGCN_F32)
        hipLaunchKernelGGL(relu_mask_kernel<float>, grid, dim3(kBlock), 0, s, (float*)G, ldg,
                           (const float*)R, ldr, n, m4);
    else
        hipLaunchKernelGGL(relu_mask_kernel<uint16_t>, grid, dim3(kBlock), 0, s, (uint16_t*)G, ldg,
                           (const uint16_t*)R, ldr, n, m4);
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

int launch_wgrad_reduce(const float* P, int64_t n_slabs, int64_t cells, int32_t m, float* dW,
                        int64_t ldw, float beta, hipStream_t s)
{
    if (cells <= 0) return MIXGCN_OK;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)ceil_div(cells, kWave)), dim3(kBlock),
                       0, s, P, n_slabs, cells, m, dW, ldw, beta);
    return MIXGCN_OK;
}

namespace {

template <typename T>
int update_typed(int op, const T* A, int64_t lda, const void* B_, int64_t ldb, void* C_,
                 int64_t ldc, int64_t n, int32_t k, int32_t m, const T* R, int64_t ldr, float beta,
                 hipStream_t s, Timer* timer)
{
    if (op == MIXGCN_OP_FWD || op == MIXGCN_OP_FWD_RELU) {
        const bool relu = op == MIXGCN_OP_FWD_RELU;
        const float* B = (const float*)B_;
        T* C = (T*)C_;
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateFwd, s));
        if (m > 64)
            MIXGCN_TRY((launch_rowblock<Shape128x128, false, T>(relu, A, lda, B, ldb, C, ldc, n, k, m,
                                                               nullptr, 0, s)));
        else
            MIXGCN_TRY((launch_rowblock<Shape128x32, false, T>(relu, A, lda, B, ldb, C, ldc, n, k, m,
                                                              nullptr, 0, s)));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else if (op == MIXGCN_OP_DGRAD) {
        // C[n x k] = (A (.) mask)[n x m] * W^T, W = B stored k x m: reduction over m
        const float* B = (const float*)B_;
        T* C = (T*)C_;
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateDgrad, s));
        if (k > 64)
            MIXGCN_TRY((launch_rowblock<Shape128x128, true, T>(false, A, lda, B, ldb, C, ldc, n, m, k,
                                                              R, ldr, s)));
        else
            MIXGCN_TRY((launch_rowblock<Shape128x32, true, T>(false, A, lda, B, ldb, C, ldc, n, m, k,
                                                             R, ldr, s)));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else if (op == MIXGCN_OP_WGRAD) {
        // C[k x m] = beta C + A[n x k]^T (B (.) mask)[n x m]
        const T* B = (const T*)B_;
        float* C = (float*)C_;
        const bool wide = m > 64;
        const int bm = 128, bn = wide ? 128 : 32;
        const int nit = (int)ceil_div(k, bm), njt = (int)ceil_div(m, bn);
        const int tiles = nit * njt;
        int64_t n_slabs = ceil_div(n, 1024);
        const int64_t cap = tiles >= 1024 ? 1 : 1024 / tiles;
        if (n_slabs > cap) n_slabs = cap;
        if (n_slabs < 1) n_slabs = 1;
        int64_t rows_per_slab = ceil_div(ceil_div(n, n_slabs), BK) * BK;
        if (rows_per_slab < BK) rows_per_slab = BK;
        n_slabs = n > 0 ? ceil_div(n, rows_per_slab) : 1;
        const int64_t cells = (int64_t)k * m;
        void* scratch = nullptr;
        MIXGCN_TRY(get_scratch(0, (size_t)n_slabs * cells * sizeof(float), &scratch));
        float* P = (float*)scratch;
        const unsigned grid = (unsigned)(n_slabs * tiles);
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateWgrad, s));
#define MIXGCN_WGRAD(SHAPE, MASK)                                                                \
    hipLaunchKernelGGL((wgrad_slab_kernel<SHAPE, MASK, T>), dim3(grid), dim3(kBlock), 0, s, A, lda, \
                       B, ldb, R, ldr, P, n, k, m, rows_per_slab, nit, njt)
        if (wide) {
            if (R) MIXGCN_WGRAD(Shape128x128, true);
            else MIXGCN_WGRAD(Shape128x128, false);
        } else {
            if (R) MIXGCN_WGRAD(Shape128x32, true);
            else MIXGCN_WGRAD(Shape128x32, false);
        }
#undef MIXGCN_WGRAD
        if (timer) MIXGCN_TRY(timer->end(s));
        MIXGCN_TRY(launch_wgrad_reduce(P, n_slabs, cells, m, C, ldc, beta, s));
    } else {
        return fail(MIXGCN_EINVAL, "update: unknown op");
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace

int launch_update(int op, int dtype, const void* A, int64_t lda, const void* B, int64_t ldb,
                  void* C, int64_t ldc, int64_t n, int32_t k, int32_t m, const void* R,
                  int64_t ldr, float beta, hipStream_t s, Timer* timer)
{
    if (dtype == MIXGCN_F32 && g_update_arith == MIXGCN_ARITH_BF16X3 &&
        update_split_applies(op, lda, ldb, ldr, n, k, m)) {
        const float* a = (const float*)A;
        const float* b = (const float*)B;
        const float* r = (const float*)R;
        if (op != MIXGCN_OP_WGRAD)
            return launch_update_split(op, a, lda, b, ldb, (float*)C, ldc, n, k, m, r, ldr, beta, s,
                                       timer);
        // whole steps of 16 node rows on the bf16 matrix cores, the last few rows on the fp32 ones
        const int64_t n16 = n - n % 16;
        MIXGCN_TRY(launch_update_split(op, a, lda, b, ldb, (float*)C, ldc, n16, k, m, r, ldr, beta, s,
                                       timer));
        if (n16 == n) return MIXGCN_OK;
        return update_typed<float>(op, a + n16 * lda, lda, b + n16 * ldb, ldb, C, ldc, n - n16, k, m,
                                   r ? r + n16 * ldr : nullptr, ldr, 1.f, s, nullptr);
    }
    if (dtype == MIXGCN_F32)
        return update_typed<float>(op, (const float*)A, lda, B, ldb, C, ldc, n, k, m,
                                   (const float*)R, ldr, beta, s, timer);
    return launch_update_bf16(op, (const uint16_t*)A, lda, B, ldb, C, ldc, n, k, m,
                              (const uint16_t*)R, ldr, beta, s, timer);
}

}  // namespace mixgcn
