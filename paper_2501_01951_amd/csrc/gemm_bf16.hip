// Node update and its backward products for bf16-stored features (paper Algorithm 2, update
// phase) on the bf16 matrix cores: v_mfma_f32_32x32x16_bf16, fp32 accumulation.
//
// Activations and gradients are bf16 in memory and enter the MFMA as they are.  Weights are
// fp32: every call first splits W = hi + lo into two bf16 terms (|W - hi - lo| < 2^-16 |W|) in
// the layout the B operand wants (output index major, reduction index contiguous, zero padded
// to whole tiles, and tile by tile in the order the kernel walks them, so that a step's weights
// are one dense block), so a product with W is two MFMAs and keeps fp32-class weights.  The weight
// gradient multiplies two bf16 tensors and needs no split.
//
// MFMA 32x32x16 operand layout: lane l supplies A[i = l % 32][k = 8 (l / 32) + 0..7] and
// B[k = 8 (l / 32) + 0..7][j = l % 32] as eight consecutive bf16; D as for the fp32 32x32 MFMA.
// Tiles are therefore staged row-major with the reduction index contiguous and read with one
// 16-byte LDS load per operand.
#include "device_utils.h"
#include "internal.h"

namespace mixgcn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BKB = 32;       // reduction depth staged per step (bf16 elements)
constexpr int LDT = BKB + 8;  // LDS row stride: 80 bytes, so 16-byte reads of 16 rows hit all banks

template <int WM_, int WN_, int TM_, int TN_>
struct Shape {
    static constexpr int WM = WM_, WN = WN_, TM = TM_, TN = TN_;
    static constexpr int BM = WM * TM * 32;
    static constexpr int BN = WN * TN * 32;
    static_assert(WM * WN == 4, "four waves per block");
};
using Shape128x128 = Shape<2, 2, 2, 2>;
using Shape128x32 = Shape<4, 1, 1, 1>;

__device__ inline uint16_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ inline unsigned xcd_local_index(unsigned bid, unsigned grid)
{
    const unsigned q = grid / 8, rem = grid % 8, x = bid % 8;
    return x * q + (x < rem ? x : rem) + bid / 8;
}

// Operand element (j, kk) = transpose ? W[kk][j] : W[j][kk], zero outside W, as bf16 hi and lo
// parts, in the order the row-block kernel walks them: [column tile j / bn][step kk / BKB]
// [j % bn][kk % BKB], so that the weights of one step of one tile are bn * 64 contiguous bytes.
__device__ __host__ inline size_t split_weight_index(int j, int kk, int bn, int n_steps)
{
    return (((size_t)(j / bn) * n_steps + kk / BKB) * bn + j % bn) * BKB + kk % BKB;
}
__global__ __launch_bounds__(kBlock) void split_weights_kernel(
    const float* __restrict__ W, int64_t ldw, int rows_w, int cols_w, int transpose,
    uint16_t* __restrict__ hi, uint16_t* __restrict__ lo, int out_rows, int out_cols, int bn)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= out_rows * out_cols) return;
    const int j = idx / out_cols, kk = idx % out_cols;
    const int r = transpose ? kk : j, c = transpose ? j : kk;
    const float x = (r < rows_w && c < cols_w) ? W[(int64_t)r * ldw + c] : 0.f;
    const uint16_t h = bf16_rne(x);
    const float rest = x - __uint_as_float((uint32_t)h << 16);
    const size_t o = split_weight_index(j, kk, bn, out_cols / BKB);
    hi[o] = h;
    lo[o] = (rest == rest && fabsf(rest) <= 3.0e38f) ? bf16_rne(rest) : (uint16_t)0;
}

// Eight bf16 of a feature tile on their way from global memory to LDS: issue() starts the
// loads from an address clamped into the matrix, value() zeroes what lies outside it and, with
// MASK, what the ReLU-derivative mask 1[R > 0] removes.
template <bool MASK>
struct Piece8 {
    uint4 v, m;
    int nvalid;  // leading elements inside the matrix (0..8)

    __device__ inline void issue(const uint16_t* __restrict__ M, int64_t ld, int64_t r, int c,
                                 int64_t rows, int cols, const uint16_t* __restrict__ R,
                                 int64_t ldr)
    {
        const bool ok = r < rows && c < cols;
        nvalid = ok ? (cols - c < 8 ? cols - c : 8) : 0;
        const int64_t rr = r < rows ? r : rows - 1;
        const int cc = c < cols ? c : 0;
        v = *reinterpret_cast<const uint4*>(M + rr * ld + cc);
        if (MASK) m = *reinterpret_cast<const uint4*>(R + rr * ldr + cc);
        else m = make_uint4(0u, 0u, 0u, 0u);
    }
    __device__ static inline uint32_t keep_word(uint32_t x, uint32_t r, int left)
    {
        uint32_t keep = 0;
        if (left > 0) keep |= 0x0000FFFFu;
        if (left > 1) keep |= 0xFFFF0000u;
        if (MASK) {
            if (!(__uint_as_float(r << 16) > 0.f)) keep &= 0xFFFF0000u;
            if (!(__uint_as_float(r & 0xFFFF0000u) > 0.f)) keep &= 0x0000FFFFu;
        }
        return x & keep;
    }
    __device__ inline uint4 value() const
    {
        uint4 o;
        o.x = keep_word(v.x, m.x, nvalid);
        o.y = keep_word(v.y, m.y, nvalid - 2);
        o.z = keep_word(v.z, m.z, nvalid - 4);
        o.w = keep_word(v.w, m.w, nvalid - 6);
        return o;
    }
};

__device__ inline bf16x8 lds_operand(const uint16_t* p)
{
    return *reinterpret_cast<const bf16x8*>(p);
}

// ---- fast path of the row-block kernel ----------------------------------------------------------
// Vector instructions do not overlap with MFMAs on a SIMD of this part (each costs 4 cycles, an
// eighth of a 32x32x16 bf16 MFMA), and the generic staging path above spends more cycles on
// address arithmetic and zero-fill masks than the MFMAs take.  A tile whose rows all exist, with
// a reduction depth of whole steps, needs none of that: both operands are 16-byte copies from a
// scalar base plus a fixed per-thread offset to a fixed LDS position (the split weights are
// padded to whole tiles with zeros).  What is left per step is the ReLU mask, three packed 16-bit
// integer instructions and an AND per 32-bit word.
typedef short short2v __attribute__((ext_vector_type(2)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) uintx4 lds_uintx4;
__device__ inline void lds_store16(uint16_t* p, const uint4& v)
{
    const uintx4 q = {v.x, v.y, v.z, v.w};
    *(lds_uintx4*)p = q;
}

// x with the halves zeroed whose reference half (bf16 bits) is not > 0: as 16-bit integers,
// max(r, 0) is positive exactly for positive finite values (and +inf), its negation then has
// the sign bit set, which an arithmetic shift spreads over the half.
__device__ inline uint32_t keep_positive(uint32_t x, uint32_t r)
{
    short2v rr;
    __builtin_memcpy(&rr, &r, 4);
    const short2v zero = {0, 0};
    const short2v keep = (-__builtin_elementwise_max(rr, zero)) >> 15;
    uint32_t k;
    __builtin_memcpy(&k, &keep, 4);
    return x & k;
}

// two fp32 -> two bf16 (round to nearest even, the conversion instruction of this part), first
// argument in the low half
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) uintx2 lds_uintx2;
__device__ inline uint32_t pack_bf16_pair(float a, float b)
{
    const floatx2 v = {a, b};
    const bf16x2 h = __builtin_convertvector(v, bf16x2);
    uint32_t u;
    __builtin_memcpy(&u, &h, 4);
    return u;
}

// Tile row of a thread's 16-byte pieces: rows are dealt so that the 16 lanes of one LDS write
// cycle (four rows of 64 bytes) take rows q, q + 4, q + 8, q + 12 of a group of 16, which at 20
// banks per row start 16 banks apart (0, 16, 32, 48 of 64) and do not collide.
__device__ inline int staged_row(int tid)
{
    const int x = tid >> 2;
    return (x & ~15) | ((x & 3) << 2) | ((x >> 2) & 3);
}

template <class S, bool MASK>
struct FastStage {
    static constexpr int A_PASSES = S::BM / 64;
    static constexpr int B_PASSES = (S::BN + 63) / 64;
    uint32_t aoff, roff, boff;  // bytes from the step's scalar bases
    int lpos;                   // halfword index in a staged tile
    bool b_on[B_PASSES];
    uint4 a[A_PASSES], r[A_PASSES], bh[B_PASSES], bl[B_PASSES];

    static constexpr uint32_t kPitchB = BKB * 2;  // a weight tile of one step is dense
    __device__ inline void init(int tid, uint32_t pitch_a, uint32_t pitch_r)
    {
        const int prow = staged_row(tid), pk = 8 * (tid & 3);
        aoff = (uint32_t)prow * pitch_a + 2u * pk;
        roff = (uint32_t)prow * pitch_r + 2u * pk;
        // threads beyond a narrow weight tile load a row of it again and store nothing
        boff = (uint32_t)(prow % S::BN) * kPitchB + 2u * pk;
        lpos = prow * LDT + pk;
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) b_on[p] = p * 64 + prow < S::BN;
    }
    __device__ inline void load(const char* a0, const char* r0, const char* bh0, const char* bl0,
                                size_t pitch_a, size_t pitch_r)
    {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            a[p] = *reinterpret_cast<const uint4*>(a0 + p * 64 * pitch_a + aoff);
            if (MASK) r[p] = *reinterpret_cast<const uint4*>(r0 + p * 64 * pitch_r + roff);
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            bh[p] = *reinterpret_cast<const uint4*>(bh0 + p * 64 * kPitchB + boff);
            bl[p] = *reinterpret_cast<const uint4*>(bl0 + p * 64 * kPitchB + boff);
        }
    }
    // TAIL: the last step of a reduction depth that is not a whole number of steps; `km` clears
    // the elements past the depth (what the row holds there is not part of the operand)
    template <bool TAIL = false>
    __device__ inline void store(uint16_t* as, uint16_t* bhs, uint16_t* bls,
                                 const uint4& km = uint4()) const
    {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            uint4 v = a[p];
            if (MASK) {
                v.x = keep_positive(v.x, r[p].x);
                v.y = keep_positive(v.y, r[p].y);
                v.z = keep_positive(v.z, r[p].z);
                v.w = keep_positive(v.w, r[p].w);
            }
            if (TAIL) {
                v.x &= km.x;
                v.y &= km.y;
                v.z &= km.z;
                v.w &= km.w;
            }
            lds_store16(as + lpos + p * 64 * LDT, v);
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p)
            if (b_on[p]) {
                lds_store16(bhs + lpos + p * 64 * LDT, bh[p]);
                lds_store16(bls + lpos + p * 64 * LDT, bl[p]);
            }
    }
};

// ---- row-block kernel: C[n x MD] = (A (.) 1[R > 0])[n x KD] * Bop[KD x MD] ---------------------
// Bop is given split, in the order of split_weights_kernel (bn = BN): j < n_col_tiles * BN,
// kk < ldb (a multiple of BKB), zero outside the weights.
// Occupancy decides these kernels: they are bound by memory traffic, and what hides a
// workgroup's barrier and load waits is another workgroup on the same compute unit.  The wide
// tile therefore keeps ONE set of operand tiles in LDS (two barriers per step) and one set of
// staging registers, which fits three workgroups per compute unit (34 KB of LDS, 160 registers);
// with double-buffered tiles and two register sets only two fit, and every shape of config 5 ran
// 5-24 % slower.  The narrow tile is small enough for four workgroups with double buffering.
template <class S, bool RELU, bool MASK>
__global__ __launch_bounds__(kBlock)
    __attribute__((amdgpu_waves_per_eu(S::BN >= 128 ? 3 : 4, S::BN >= 128 ? 3 : 4))) void rowblock_bf16_kernel(
    const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ Bh,
    const uint16_t* __restrict__ Bl, int ldb, uint16_t* __restrict__ C, int64_t ldc, int64_t n,
    int KD, int MD, const uint16_t* __restrict__ R, int64_t ldr, int n_col_tiles)
{
    // one buffer: the operand tiles (one set for the wide tile, two for the narrow one), and
    // after the last step the output tile
    constexpr bool kDouble = S::BN < 128;
    constexpr int kTileA = S::BM * LDT, kTileB = S::BN * LDT;
    constexpr int LDC = S::BN + 4;  // output tile rows: 66 or 18 banks, 8-byte aligned
    constexpr int kSets = kDouble ? 2 : 1;
    constexpr int kOperands = kSets * (kTileA + 2 * kTileB);
    constexpr int kSmem = S::BM * LDC > kOperands ? S::BM * LDC : kOperands;
    __shared__ __attribute__((aligned(16))) uint16_t smem[kSmem];
    uint16_t *As[2], *Bhs[2], *Bls[2];
    As[0] = smem;
    As[1] = kDouble ? smem + kTileA : As[0];
    Bhs[0] = smem + kSets * kTileA;
    Bhs[1] = kDouble ? Bhs[0] + kTileB : Bhs[0];
    Bls[0] = smem + kSets * kTileA + kSets * kTileB;
    Bls[1] = kDouble ? Bls[0] + kTileB : Bls[0];
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

    // a tile row holds BKB bf16 = 4 pieces of 16 bytes; a pass of the block covers 64 tile rows
    constexpr int A_PASSES = S::BM / 64;
    constexpr int B_PASSES = (S::BN + 63) / 64;
    Piece8<MASK> ra[A_PASSES];
    uint4 rbh[B_PASSES], rbl[B_PASSES];
    const int prow = staged_row(tid), pk = 8 * (tid & 3);

    auto issue_tiles = [&](int k0) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p)
            ra[p].issue(A, lda, row0 + p * 64 + prow, k0 + pk, n, KD, R, ldr);
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int j = p * 64 + prow;
            const size_t off = split_weight_index(col0 + (j < S::BN ? j : 0), k0 + pk, S::BN, ldb / BKB);
            rbh[p] = *reinterpret_cast<const uint4*>(Bh + off);
            rbl[p] = *reinterpret_cast<const uint4*>(Bl + off);
        }
    };
    auto store_tiles = [&](uint16_t* as, uint16_t* bh, uint16_t* bl) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p)
            *reinterpret_cast<uint4*>(&as[(p * 64 + prow) * LDT + pk]) = ra[p].value();
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int j = p * 64 + prow;
            if (j < S::BN) {
                *reinterpret_cast<uint4*>(&bh[j * LDT + pk]) = rbh[p];
                *reinterpret_cast<uint4*>(&bl[j * LDT + pk]) = rbl[p];
            }
        }
    };
    const int li = lane & 31, lk = lane >> 5;
    auto mma_step = [&](const uint16_t* as, const uint16_t* bh, const uint16_t* bl) {
#pragma unroll
        for (int kc = 0; kc < BKB; kc += 16) {
            bf16x8 a[S::TM], h[S::TN], l[S::TN];
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
                a[tm] = lds_operand(&as[((wm * S::TM + tm) * 32 + li) * LDT + kc + 8 * lk]);
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn) {
                h[tn] = lds_operand(&bh[((wn * S::TN + tn) * 32 + li) * LDT + kc + 8 * lk]);
                l[tn] = lds_operand(&bl[((wn * S::TN + tn) * 32 + li) * LDT + kc + 8 * lk]);
            }
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < S::TN; ++tn) {
                    // weights as the first operand: the accumulators hold the tile transposed,
                    // a lane then owns one node row and four consecutive columns per register quad
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(l[tn], a[tm],
                                                                          acc[tm][tn], 0, 0, 0);
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(h[tn], a[tm],
                                                                          acc[tm][tn], 0, 0, 0);
                }
        }
    };

    const int nk = (KD + BKB - 1) / BKB;
    // every row of the tile exists, 32-bit offsets inside a tile, and the reduction depth is a
    // whole number of steps or the rows are long enough to read the last step whole (what lies
    // past the depth is cleared on the way to LDS)
    const bool ragged = KD % BKB != 0;
    const bool fast = row0 + S::BM <= n && lda < (1 << 22) && ldr < (1 << 22) &&
                      (!ragged || ((int64_t)nk * BKB <= lda && (!MASK || (int64_t)nk * BKB <= ldr)));
    if (fast) {
        uint4 km;
        {
            const int left = KD - (nk - 1) * BKB - pk;  // elements of this thread's piece inside
            const auto word = [&](int w) {
                return (left > 2 * w ? 0x0000FFFFu : 0u) | (left > 2 * w + 1 ? 0xFFFF0000u : 0u);
            };
            km = make_uint4(word(0), word(1), word(2), word(3));
        }
        // writes the staged step to LDS; the last step of a ragged depth goes through the mask
        auto put = [&](const FastStage<S, MASK>& st, int step, uint16_t* as, uint16_t* bhs,
                       uint16_t* bls) {
            if (ragged && step == nk - 1) st.template store<true>(as, bhs, bls, km);
            else st.template store<false>(as, bhs, bls);
        };
        // Loads beyond the last step repeat it (never stored), so that no load is conditional.
        FastStage<S, MASK> st0;
        st0.init(tid, (uint32_t)lda * 2u, (uint32_t)ldr * 2u);
        const char* a0 = reinterpret_cast<const char*>(A + row0 * lda);
        const char* r0 = MASK ? reinterpret_cast<const char*>(R + row0 * ldr) : nullptr;
        const size_t tile0 = split_weight_index(col0, 0, S::BN, ldb / BKB);
        const char* bh0 = reinterpret_cast<const char*>(Bh + tile0);
        const char* bl0 = reinterpret_cast<const char*>(Bl + tile0);
        auto load = [&](FastStage<S, MASK>& st, int step) {
            const size_t sc = (size_t)(step < nk ? step : nk - 1);
            const size_t o = sc * (BKB * 2), ob = sc * (S::BN * BKB * 2);
            st.load(a0 + o, r0 + o, bh0 + ob, bl0 + ob, (size_t)lda * 2, (size_t)ldr * 2);
        };
        if constexpr (!kDouble) {
            // one set of tiles: the loads of the next step are in flight during the products
            load(st0, 0);
            for (int i = 0; i < nk; ++i) {
                put(st0, i, As[0], Bhs[0], Bls[0]);
                load(st0, i + 1);
                __syncthreads();
                mma_step(As[0], Bhs[0], Bls[0]);
                __syncthreads();  // before the next step's tiles overwrite these
            }
        } else {
            // two sets of tiles, one barrier per step, loads one step ahead
            load(st0, 0);
            put(st0, 0, As[0], Bhs[0], Bls[0]);
            __syncthreads();
            int i = 0;
            for (; i + 2 < nk; i += 2) {
                load(st0, i + 1);
                mma_step(As[0], Bhs[0], Bls[0]);
                put(st0, i + 1, As[1], Bhs[1], Bls[1]);
                __syncthreads();
                load(st0, i + 2);
                mma_step(As[1], Bhs[1], Bls[1]);
                put(st0, i + 2, As[0], Bhs[0], Bls[0]);
                __syncthreads();
            }
            if (nk - i == 2) {
                load(st0, i + 1);
                mma_step(As[0], Bhs[0], Bls[0]);
                put(st0, i + 1, As[1], Bhs[1], Bls[1]);
                __syncthreads();
                mma_step(As[1], Bhs[1], Bls[1]);
            } else {
                mma_step(As[0], Bhs[0], Bls[0]);
            }
        }
    } else {
        issue_tiles(0);
        if constexpr (!kDouble) {
            for (int i = 0; i < nk; ++i) {
                store_tiles(As[0], Bhs[0], Bls[0]);
                if (i + 1 < nk) issue_tiles((i + 1) * BKB);
                __syncthreads();
                mma_step(As[0], Bhs[0], Bls[0]);
                __syncthreads();
            }
        } else {
            store_tiles(As[0], Bhs[0], Bls[0]);
            __syncthreads();
            for (int i = 0; i < nk; ++i) {
                const int cur = i & 1;
                if (i + 1 < nk) issue_tiles((i + 1) * BKB);
                mma_step(As[cur], Bhs[cur], Bls[cur]);
                if (i + 1 < nk) store_tiles(As[cur ^ 1], Bhs[cur ^ 1], Bls[cur ^ 1]);
                __syncthreads();
            }
        }
    }

    // Accumulator layout (transposed product): lane l, register v -> node row l % 32, column
    // 8 (v / 4) + 4 (l / 32) + v % 4 of the 32 x 32 tile.
    // Converted in pairs by the hardware, collected in LDS and written as 8-byte pieces of whole
    // rows (a lane's own elements lie in 32 different rows: written directly they would be
    // 2-byte stores scattered over as many lines).
    __syncthreads();  // every wave is done with the operand tiles
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // ReLU on the fp32 sums, one maximum per element (on the packed pairs it took six
                // instructions per word, a third of this kernel's vector work)
                float e0 = acc[tm][tn][4 * g], e1 = acc[tm][tn][4 * g + 1];
                float e2 = acc[tm][tn][4 * g + 2], e3 = acc[tm][tn][4 * g + 3];
                if (RELU) {
                    e0 = fmaxf(e0, 0.f);
                    e1 = fmaxf(e1, 0.f);
                    e2 = fmaxf(e2, 0.f);
                    e3 = fmaxf(e3, 0.f);
                }
                const uint32_t w0 = pack_bf16_pair(e0, e1);
                const uint32_t w1 = pack_bf16_pair(e2, e3);
                const uintx2 v = {w0, w1};
                *(lds_uintx2*)(smem + ((wm * S::TM + tm) * 32 + li) * LDC + (wn * S::TN + tn) * 32 +
                               8 * g + 4 * lk) = v;
            }
    __syncthreads();
    constexpr int CPR = S::BN / 4;     // 8-byte pieces per row
    constexpr int RPP = kBlock / CPR;  // rows per pass of the block
    const int crow = tid / CPR, cpiece = tid % CPR;
    const int c = col0 + 4 * cpiece;
    const int c_valid = c < MD ? (MD - c < 4 ? MD - c : 4) : 0;  // columns of the piece inside C
    if (c_valid == 0) return;
    uint16_t* cbase = C + row0 * ldc + c;
    const int64_t rows_left = n - row0;
#pragma unroll
    for (int p = 0; p < S::BM / RPP; ++p) {
        const int r = p * RPP + crow;
        if (r >= rows_left) break;
        const uintx2 v = *(const lds_uintx2*)(smem + r * LDC + 4 * cpiece);
        uint16_t* dst = cbase + (int64_t)r * ldc;
        if (c_valid == 4) {
            *reinterpret_cast<uint2*>(dst) = make_uint2(v.x, v.y);
        } else {
            dst[0] = (uint16_t)v.x;
            if (c_valid > 1) dst[1] = (uint16_t)(v.x >> 16);
            if (c_valid > 2) dst[2] = (uint16_t)v.y;
        }
    }
}

// ---- slab kernel: P[slab][KD x MD] = A[rows of slab][KD]^T * (B (.) 1[R > 0])[rows][MD] --------
// The reduction runs over node rows, which is the slow index of both operands in memory, so a
// tile is transposed on its way into LDS: a thread takes the same eight columns of two
// consecutive rows and writes eight 32-bit words, each holding one column's pair of rows.
template <class S, bool MASK>
__global__ __launch_bounds__(kBlock) void wgrad_bf16_kernel(
    const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ B, int64_t ldb,
    const uint16_t* __restrict__ R, int64_t ldr, float* __restrict__ P, int64_t n, int KD, int MD,
    int64_t rows_per_slab, int n_i_tiles, int n_j_tiles)
{
    __shared__ __attribute__((aligned(16))) uint16_t As[2][S::BM * LDT];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][S::BN * LDT];
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

    // 16 row pairs x (tile width / 8) column groups per step; one block pass covers 16 groups
    constexpr int A_PASSES = S::BM / 128 > 0 ? S::BM / 128 : 1;
    constexpr int B_PASSES = S::BN / 128 > 0 ? S::BN / 128 : 1;
    const int rp = tid / 16, cg = tid % 16;
    Piece8<false> a0[A_PASSES], a1[A_PASSES];
    Piece8<MASK> b0[B_PASSES], b1[B_PASSES];

    auto issue_tiles = [&](int64_t r0) {
        const int64_t ra = r0 + 2 * rp;
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int c = 8 * (p * 16 + cg);
            const int cc = c < S::BM ? c : 0;
            a0[p].issue(A, lda, ra, i0 + cc, r_end, KD, nullptr, 0);
            a1[p].issue(A, lda, ra + 1, i0 + cc, r_end, KD, nullptr, 0);
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int c = 8 * (p * 16 + cg);
            const int cc = c < S::BN ? c : 0;
            b0[p].issue(B, ldb, ra, j0 + cc, r_end, MD, R, ldr);
            b1[p].issue(B, ldb, ra + 1, j0 + cc, r_end, MD, R, ldr);
        }
    };
    // words of the two rows -> LDS[(column)][row pair]
    auto scatter = [&](uint16_t* tile, int c, const uint4& x, const uint4& y) {
        uint32_t* t32 = reinterpret_cast<uint32_t*>(tile);
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            t32[(c + 2 * w) * (LDT / 2) + rp] = (xs[w] & 0xFFFFu) | (ys[w] << 16);
            t32[(c + 2 * w + 1) * (LDT / 2) + rp] = (xs[w] >> 16) | (ys[w] & 0xFFFF0000u);
        }
    };
    auto store_tiles = [&](uint16_t* as, uint16_t* bs) {
#pragma unroll
        for (int p = 0; p < A_PASSES; ++p) {
            const int c = 8 * (p * 16 + cg);
            if (c < S::BM) scatter(as, c, a0[p].value(), a1[p].value());
        }
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            const int c = 8 * (p * 16 + cg);
            if (c < S::BN) scatter(bs, c, b0[p].value(), b1[p].value());
        }
    };
    const int li = lane & 31, lk = lane >> 5;
    auto mma_step = [&](const uint16_t* as, const uint16_t* bs) {
#pragma unroll
        for (int kc = 0; kc < BKB; kc += 16) {
            bf16x8 a[S::TM], b[S::TN];
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
                a[tm] = lds_operand(&as[((wm * S::TM + tm) * 32 + li) * LDT + kc + 8 * lk]);
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn)
                b[tn] = lds_operand(&bs[((wn * S::TN + tn) * 32 + li) * LDT + kc + 8 * lk]);
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < S::TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn],
                                                                          acc[tm][tn], 0, 0, 0);
        }
    };

    if (r_begin < r_end) {
        const int64_t nk = (r_end - r_begin + BKB - 1) / BKB;
        issue_tiles(r_begin);
        store_tiles(As[0], Bs[0]);
        __syncthreads();
        for (int64_t i = 0; i < nk; ++i) {
            const int cur = (int)(i & 1);
            if (i + 1 < nk) issue_tiles(r_begin + (i + 1) * BKB);
            mma_step(As[cur], Bs[cur]);
            if (i + 1 < nk) store_tiles(As[cur ^ 1], Bs[cur ^ 1]);
            __syncthreads();
        }
    }
    float* out = P + (size_t)slab * KD * MD;
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

// ---- the same product without the scattered LDS writes -------------------------------------------
// (In the kernel above the transposing 4-byte writes keep the LDS busy 80 % of the time, seven
// eighths of it with bank conflicts.)  Here the tiles are staged as they lie, row-major
// [node row][feature] with 16-byte copies, and the LDS read transposes: ds_read_b64_tr_b16 hands
// lane i of a group of 16 lanes element i % 4 of the 8 bytes addressed by lanes i / 4, i / 4 + 4,
// i / 4 + 8 and i / 4 + 12, so with lane s of the group pointing at row s / 4, features
// 4 (s % 4) .. + 3, every lane receives its own feature at four consecutive rows, and two such
// reads are one MFMA operand.  Two groups are served per cycle from 64 banks (four rows of 64
// bytes): a row pitch of 64 bytes modulo 256 keeps them apart.  Rows come in whole steps of 32
// (the caller gives the last n % 32 rows to the kernel above); features beyond the matrices are
// zeroed with per-thread masks that do not change from step to step.
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) shortx4 lds_shortx4;

template <int PITCH>
__device__ inline bf16x8 read_transposed(const uint16_t* p)
{
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)p);
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_shortx4*)(p + 4 * PITCH));
    const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    bf16x8 o;
    __builtin_memcpy(&o, &v, 16);
    return o;
}

template <class S, bool MASK>
__global__ __launch_bounds__(kBlock) void wgrad_bf16_tr_kernel(
    const uint16_t* __restrict__ A, int64_t lda, const uint16_t* __restrict__ B, int64_t ldb,
    const uint16_t* __restrict__ R, int64_t ldr, float* __restrict__ P, int64_t n, int KD, int MD,
    int64_t rows_per_slab, int n_i_tiles, int n_j_tiles)
{
    static_assert(S::BM == 128 && (S::BN == 128 || S::BN == 32), "tile shapes of the staging");
    constexpr int PA = 128 + 32;                         // halfwords per staged row of A
    constexpr int PB = S::BN == 128 ? 128 + 32 : 32;     // ... of B
    constexpr int B_PPR = S::BN / 8;                     // 16-byte pieces per row of B
    constexpr int B_RPP = kBlock / B_PPR;                // rows per pass of the block
    constexpr int B_PASSES = B_RPP >= BKB ? 1 : BKB / B_RPP;
    __shared__ __attribute__((aligned(16))) uint16_t As[2][BKB * PA];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BKB * PB];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / S::WN, wn = wave % S::WN;
    const int tiles = n_i_tiles * n_j_tiles;
    const unsigned lid = xcd_local_index(blockIdx.x, gridDim.x);
    const int64_t slab = lid / tiles;
    const int t = (int)(lid % tiles);
    const int i0 = (t / n_j_tiles) * S::BM, j0 = (t % n_j_tiles) * S::BN;
    const int64_t r_begin = slab * rows_per_slab;
    const int64_t r_end = (r_begin + rows_per_slab) < n ? (r_begin + rows_per_slab) : n;
    const int nk = (int)((r_end - r_begin) / BKB);  // whole steps: the caller sees to it

    floatx16 acc[S::TM][S::TN];
#pragma unroll
    for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < S::TN; ++tn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[tm][tn][v] = 0.f;

    // staging: A rows tid / 16 and tid / 16 + 16, features 8 (tid % 16) .. + 7; B alike with its
    // own pieces per row.  A piece beyond the matrix is loaded from column 0 and masked to zero.
    auto keep_words = [](int nvalid, uint32_t* kw) {
#pragma unroll
        for (int w = 0; w < 4; ++w)
            kw[w] = (nvalid > 2 * w ? 0x0000FFFFu : 0u) | (nvalid > 2 * w + 1 ? 0xFFFF0000u : 0u);
    };
    const int arow = tid >> 4, acol = i0 + 8 * (tid & 15);
    const int a_valid = acol < KD ? (KD - acol < 8 ? KD - acol : 8) : 0;
    uint32_t a_keep[4];
    keep_words(a_valid, a_keep);
    const uint32_t a_off = ((uint32_t)arow * (uint32_t)lda + (uint32_t)(a_valid ? acol : 0)) * 2u;
    const int a_pos = arow * PA + 8 * (tid & 15);
    const int brow = tid / B_PPR, bcol = j0 + 8 * (tid % B_PPR);
    const bool b_on = brow < BKB;
    const int b_valid = bcol < MD ? (MD - bcol < 8 ? MD - bcol : 8) : 0;
    uint32_t b_keep[4];
    keep_words(b_valid, b_keep);
    const int brow_c = b_on ? brow : 0;  // idle threads of a narrow tile load row 0 again
    const uint32_t b_off = ((uint32_t)brow_c * (uint32_t)ldb + (uint32_t)(b_valid ? bcol : 0)) * 2u;
    const uint32_t r_off = MASK ? ((uint32_t)brow_c * (uint32_t)ldr + (uint32_t)(b_valid ? bcol : 0)) * 2u : 0u;
    const int b_pos = brow_c * PB + 8 * (tid % B_PPR);
    const bool inside = i0 + S::BM <= KD && j0 + S::BN <= MD;

    const char* a0 = reinterpret_cast<const char*>(A + r_begin * lda);
    const char* b0 = reinterpret_cast<const char*>(B + r_begin * ldb);
    const char* m0 = MASK ? reinterpret_cast<const char*>(R + r_begin * ldr) : nullptr;
    const size_t step_a = (size_t)BKB * 2 * (size_t)lda, step_b = (size_t)BKB * 2 * (size_t)ldb,
                 step_r = (size_t)BKB * 2 * (size_t)ldr;

    struct Regs {
        uint4 a[2], b[B_PASSES], r[B_PASSES];
    };
    // a step beyond the last one loads the last one again (never stored): no branch around loads
    auto load = [&](Regs& g, int step) {
        const size_t sc = (size_t)(step < nk ? step : nk - 1);
#pragma unroll
        for (int p = 0; p < 2; ++p)
            g.a[p] = *reinterpret_cast<const uint4*>(a0 + sc * step_a + (size_t)p * 16 * 2 * (size_t)lda + a_off);
#pragma unroll
        for (int p = 0; p < B_PASSES; ++p) {
            g.b[p] = *reinterpret_cast<const uint4*>(b0 + sc * step_b + (size_t)p * B_RPP * 2 * (size_t)ldb + b_off);
            if (MASK)
                g.r[p] = *reinterpret_cast<const uint4*>(m0 + sc * step_r + (size_t)p * B_RPP * 2 * (size_t)ldr + r_off);
        }
    };
    auto store = [&](const Regs& g, uint16_t* as, uint16_t* bs) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            uint4 v = g.a[p];
            if (!inside) {
                v.x &= a_keep[0];
                v.y &= a_keep[1];
                v.z &= a_keep[2];
                v.w &= a_keep[3];
            }
            lds_store16(as + a_pos + p * 16 * PA, v);
        }
        if (b_on) {
#pragma unroll
            for (int p = 0; p < B_PASSES; ++p) {
                uint4 v = g.b[p];
                if (MASK) {
                    v.x = keep_positive(v.x, g.r[p].x);
                    v.y = keep_positive(v.y, g.r[p].y);
                    v.z = keep_positive(v.z, g.r[p].z);
                    v.w = keep_positive(v.w, g.r[p].w);
                }
                if (!inside) {
                    v.x &= b_keep[0];
                    v.y &= b_keep[1];
                    v.z &= b_keep[2];
                    v.w &= b_keep[3];
                }
                lds_store16(bs + b_pos + p * B_RPP * PB, v);
            }
        }
    };
    // operand reads: lane -> 16-lane group (feature block, reduction half), place in the group
    const int grp = lane >> 4, gs = lane & 15;
    const int rrow = 8 * (grp >> 1) + (gs >> 2), rcol = 16 * (grp & 1) + 4 * (gs & 3);
    auto step_mma = [&](const uint16_t* as, const uint16_t* bs) {
#pragma unroll
        for (int kc = 0; kc < BKB; kc += 16) {
            bf16x8 a[S::TM], b[S::TN];
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
                a[tm] = read_transposed<PA>(as + (kc + rrow) * PA + (wm * S::TM + tm) * 32 + rcol);
#pragma unroll
            for (int tn = 0; tn < S::TN; ++tn)
                b[tn] = read_transposed<PB>(bs + (kc + rrow) * PB + (wn * S::TN + tn) * 32 + rcol);
#pragma unroll
            for (int tm = 0; tm < S::TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < S::TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[tm], b[tn], acc[tm][tn],
                                                                          0, 0, 0);
        }
    };

    if (nk > 0) {
        // LDS double buffered one step ahead, global loads two steps ahead in two register sets
        Regs g0, g1;
        load(g0, 0);
        load(g1, 1);
        store(g0, As[0], Bs[0]);
        load(g0, 2);
        __syncthreads();
        int i = 0;
        for (; i + 2 < nk; i += 2) {
            step_mma(As[0], Bs[0]);
            store(g1, As[1], Bs[1]);
            load(g1, i + 3);
            __syncthreads();
            step_mma(As[1], Bs[1]);
            store(g0, As[0], Bs[0]);
            load(g0, i + 4);
            __syncthreads();
        }
        step_mma(As[0], Bs[0]);
        if (nk - i == 2) {
            store(g1, As[1], Bs[1]);
            __syncthreads();
            step_mma(As[1], Bs[1]);
        }
    }

    const int li = lane & 31, lk = lane >> 5;
    float* out = P + (size_t)slab * KD * MD;
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

// C[n x out_dim] = (A (.) mask)[n x red_dim] * Wop, Wop[kk][j] = transpose_w ? W[kk][j] : W[j][kk]
template <class S>
int launch_rowblock_bf16(bool relu, const uint16_t* A, int64_t lda, const float* W, int64_t ldw,
                         int w_rows, int w_cols, bool transpose_w, uint16_t* C, int64_t ldc,
                         int64_t n, int red_dim, int out_dim, const uint16_t* R, int64_t ldr,
                         hipStream_t s)
{
    const int nct = (int)ceil_div(out_dim, S::BN);
    const int64_t grid = ceil_div(n, S::BM) * nct;
    if (grid <= 0) return MIXGCN_OK;
    if (grid > 0x7FFFFFFF) return fail(MIXGCN_EINVAL, "update: too many row tiles");
    const int out_rows = nct * S::BN, out_cols = (int)ceil_div(red_dim, BKB) * BKB;
    void* scratch = nullptr;
    MIXGCN_TRY(get_scratch(2, (size_t)2 * out_rows * out_cols * sizeof(uint16_t), &scratch));
    uint16_t* hi = (uint16_t*)scratch;
    uint16_t* lo = hi + (size_t)out_rows * out_cols;
    hipLaunchKernelGGL(split_weights_kernel, dim3((unsigned)ceil_div(out_rows * out_cols, kBlock)),
                       dim3(kBlock), 0, s, W, ldw, w_rows, w_cols, transpose_w ? 1 : 0, hi, lo,
                       out_rows, out_cols, S::BN);
#define MIXGCN_ROWBLOCK(RELU, MASK)                                                              \
    hipLaunchKernelGGL((rowblock_bf16_kernel<S, RELU, MASK>), dim3((unsigned)grid), dim3(kBlock), \
                       0, s, A, lda, hi, lo, out_cols, C, ldc, n, red_dim, out_dim, R, ldr, nct)
    if (R) MIXGCN_ROWBLOCK(false, true);
    else if (relu) MIXGCN_ROWBLOCK(true, false);
    else MIXGCN_ROWBLOCK(false, false);
#undef MIXGCN_ROWBLOCK
    return MIXGCN_OK;
}

}  // namespace

int launch_update_bf16(int op, const uint16_t* A, int64_t lda, const void* B_, int64_t ldb,
                       void* C_, int64_t ldc, int64_t n, int32_t k, int32_t m, const uint16_t* R,
                       int64_t ldr, float beta, hipStream_t s, Timer* timer)
{
    if (op == MIXGCN_OP_FWD || op == MIXGCN_OP_FWD_RELU) {
        // C[n x m] = A[n x k] W, W stored k x m: operand rows = output columns -> transposed split
        const bool relu = op == MIXGCN_OP_FWD_RELU;
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateFwd, s));
        if (m > 64)
            MIXGCN_TRY((launch_rowblock_bf16<Shape128x128>(relu, A, lda, (const float*)B_, ldb, k, m,
                                                          true, (uint16_t*)C_, ldc, n, k, m,
                                                          nullptr, 0, s)));
        else
            MIXGCN_TRY((launch_rowblock_bf16<Shape128x32>(relu, A, lda, (const float*)B_, ldb, k, m,
                                                         true, (uint16_t*)C_, ldc, n, k, m, nullptr,
                                                         0, s)));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else if (op == MIXGCN_OP_DGRAD) {
        // C[n x k] = (A (.) mask)[n x m] W^T, W stored k x m: operand rows = rows of W
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateDgrad, s));
        if (k > 64)
            MIXGCN_TRY((launch_rowblock_bf16<Shape128x128>(false, A, lda, (const float*)B_, ldb, k, m,
                                                          false, (uint16_t*)C_, ldc, n, m, k, R,
                                                          ldr, s)));
        else
            MIXGCN_TRY((launch_rowblock_bf16<Shape128x32>(false, A, lda, (const float*)B_, ldb, k, m,
                                                         false, (uint16_t*)C_, ldc, n, m, k, R, ldr,
                                                         s)));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else if (op == MIXGCN_OP_WGRAD) {
        // C[k x m] = beta C + A[n x k]^T (B (.) mask)[n x m]: whole steps of 32 rows with the
        // transposing LDS reads, the last n % 32 rows with the scattering kernel, added on top
        const uint16_t* B = (const uint16_t*)B_;
        float* C = (float*)C_;
        const bool wide = m > 64;
        const int bm = 128, bn = wide ? 128 : 32;
        const int nit = (int)ceil_div(k, bm), njt = (int)ceil_div(m, bn);
        const int tiles = nit * njt;
        const int64_t cells = (int64_t)k * m;
        const bool pitches_ok = lda < (1 << 25) && ldb < (1 << 25) && ldr < (1 << 25);
        const int64_t n_main = pitches_ok ? n - n % BKB : 0;
        if (timer) MIXGCN_TRY(timer->begin(kTimeUpdateWgrad, s));
        auto part = [&](bool transposing_reads, int64_t row0, int64_t rows, float beta_part) -> int {
            int64_t n_slabs = ceil_div(rows, 2048);
            const int64_t cap = tiles >= 1024 ? 1 : 1024 / tiles;
            if (n_slabs > cap) n_slabs = cap;
            if (n_slabs < 1) n_slabs = 1;
            int64_t rows_per_slab = ceil_div(ceil_div(rows, n_slabs), BKB) * BKB;
            if (rows_per_slab < BKB) rows_per_slab = BKB;
            n_slabs = rows > 0 ? ceil_div(rows, rows_per_slab) : 1;
            void* scratch = nullptr;
            MIXGCN_TRY(get_scratch(0, (size_t)n_slabs * cells * sizeof(float), &scratch));
            float* P = (float*)scratch;
            const unsigned grid = (unsigned)(n_slabs * tiles);
            const uint16_t* a = A + row0 * lda;
            const uint16_t* b = B + row0 * ldb;
            const uint16_t* r = R ? R + row0 * ldr : nullptr;
#define MIXGCN_WGRAD(KERNEL, SHAPE, MASK)                                                        \
    hipLaunchKernelGGL((KERNEL<SHAPE, MASK>), dim3(grid), dim3(kBlock), 0, s, a, lda, b, ldb, r,  \
                       ldr, P, rows, k, m, rows_per_slab, nit, njt)
#define MIXGCN_WGRAD_SHAPES(KERNEL)                                                              \
    do {                                                                                         \
        if (wide) {                                                                              \
            if (r) MIXGCN_WGRAD(KERNEL, Shape128x128, true);                                     \
            else MIXGCN_WGRAD(KERNEL, Shape128x128, false);                                      \
        } else {                                                                                 \
            if (r) MIXGCN_WGRAD(KERNEL, Shape128x32, true);                                      \
            else MIXGCN_WGRAD(KERNEL, Shape128x32, false);                                       \
        }                                                                                        \
    } while (0)
            if (transposing_reads) MIXGCN_WGRAD_SHAPES(wgrad_bf16_tr_kernel);
            else MIXGCN_WGRAD_SHAPES(wgrad_bf16_kernel);
#undef MIXGCN_WGRAD_SHAPES
#undef MIXGCN_WGRAD
            return launch_wgrad_reduce(P, n_slabs, cells, m, C, ldc, beta_part, s);
        };
        if (n_main > 0) MIXGCN_TRY(part(true, 0, n_main, beta));
        if (n_main < n || n == 0) MIXGCN_TRY(part(false, n_main, n - n_main, n_main > 0 ? 1.f : beta));
        if (timer) MIXGCN_TRY(timer->end(s));
    } else {
        return fail(MIXGCN_EINVAL, "update: unknown op");
    }
    MIXGCN_HIP_TRY(hipGetLastError());
    return MIXGCN_OK;
}

}  // namespace mixgcn
