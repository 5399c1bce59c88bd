/*
 * Seeded synthetic inputs for the GCN hot path: edge lists (Erdos-Renyi G(n,p), R-MAT,
 * Zipf-source power law) and dense tensors (uniform, normal, Glorot-uniform, labels).
 *
 * This file holds no GCN arithmetic.  It only produces inputs, and it is the one piece of
 * code that both the CPU oracle's tests and the HIP library's tests/bench may share.
 *
 * Every value is a pure function of (seed, stream, index): a counter-based generator built
 * on the SplitMix64 finalizer.  The output therefore does not depend on the thread count or
 * on the order in which elements are produced.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* key for one (seed, stream) pair; draws are mix64(key + idx * odd) */
static inline uint64_t stream_key(uint64_t seed, uint64_t stream)
{
    return mix64(mix64(seed) ^ (stream * 0xD6E8FEB86659FD93ull));
}

static inline uint64_t draw(uint64_t key, uint64_t idx)
{
    return mix64(key + idx * 0x9E3779B97F4A7C15ull);
}

/* ---- id scramble: a bijection on [0, 2^scale) ------------------------------------------- */
static inline uint64_t scramble_id(uint64_t x, int scale, uint64_t key)
{
    const uint64_t mask = (scale >= 64) ? ~0ull : ((1ull << scale) - 1);
    const int sh = scale / 2 + 1;
    uint64_t m1 = (key | 1ull), m2 = ((key >> 17) | 1ull);
    x = (x * m1 + (key >> 7)) & mask;
    x ^= x >> sh;
    x = (x * m2) & mask;
    x ^= x >> sh;
    x = (x * 0x9E3779B97F4A7C15ull + 0x7F4A7C15ull) & mask;
    return x;
}

/*
 * R-MAT edge generator.  Edge i descends `scale` levels of the 2x2 recursive partition with
 * quadrant probabilities (a, b, c, 1-a-b-c); no per-level noise.  If n_limit < 2^scale an
 * edge whose (scrambled) endpoints are not both < n_limit is redrawn with the next attempt
 * counter.  scramble != 0 applies a fixed bijective relabelling of the ids so that the hubs
 * are not clustered at the low ids.
 */
void gg_rmat_edges(uint64_t seed, int scale, uint64_t n_edges, double a, double b, double c,
                   int scramble, uint64_t n_limit, uint32_t* src, uint32_t* dst)
{
    const uint64_t key = stream_key(seed, 0x524D4154ull /* "RMAT" */);
    const uint64_t skey = stream_key(seed, 0x5343524Dull /* "SCRM" */);
    const uint32_t ta = (uint32_t)(a * 4294967296.0);
    const uint32_t tb = (uint32_t)((a + b) * 4294967296.0);
    const uint32_t tc = (uint32_t)((a + b + c) * 4294967296.0);
    const uint64_t n_full = 1ull << scale;
    if (n_limit == 0 || n_limit > n_full) n_limit = n_full;
    const int words = (scale + 1) / 2; /* two 32-bit draws per 64-bit word */

#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n_edges; ++i) {
        uint64_t u, v;
        for (uint64_t attempt = 0;; ++attempt) {
            const uint64_t ekey = mix64(key ^ mix64((uint64_t)i + (attempt << 48)));
            u = 0;
            v = 0;
            for (int w = 0; w < words; ++w) {
                uint64_t r = draw(ekey, (uint64_t)w);
                for (int half = 0; half < 2; ++half) {
                    int level = 2 * w + half;
                    if (level >= scale) break;
                    uint32_t x = (uint32_t)(r >> (32 * half));
                    unsigned ubit, vbit;
                    if (x < ta) { ubit = 0; vbit = 0; }
                    else if (x < tb) { ubit = 0; vbit = 1; }
                    else if (x < tc) { ubit = 1; vbit = 0; }
                    else { ubit = 1; vbit = 1; }
                    u = (u << 1) | ubit;
                    v = (v << 1) | vbit;
                }
            }
            if (scramble) {
                u = scramble_id(u, scale, skey);
                v = scramble_id(v, scale, skey);
            }
            if (u < n_limit && v < n_limit) break;
        }
        src[i] = (uint32_t)u;
        dst[i] = (uint32_t)v;
    }
}

/*
 * Erdos-Renyi G(n, p): one Bernoulli(p) draw per unordered pair {i, j}, i < j, taken from
 * the hash of (seed, i, j).  Pairs are emitted in lexicographic order.  Returns the number
 * of edges; writes at most `cap` of them (call with cap = 0 to count).
 */
uint64_t gg_er_edges(uint64_t seed, uint32_t n, double p, uint32_t* src, uint32_t* dst,
                     uint64_t cap)
{
    const uint64_t key = stream_key(seed, 0x4552ull /* "ER" */);
    const uint64_t thr = (p >= 1.0) ? ~0ull : (uint64_t)(p * 18446744073709551616.0);
    uint64_t cnt = 0;
    for (uint32_t i = 0; i < n; ++i)
        for (uint32_t j = i + 1; j < n; ++j) {
            uint64_t r = draw(key, (uint64_t)i * n + j);
            if (r < thr || p >= 1.0) {
                if (cnt < cap) { src[cnt] = i; dst[cnt] = j; }
                ++cnt;
            }
        }
    return cnt;
}

/*
 * Power-law edge list.  Node out-degrees follow a discrete power law with tail exponent alpha
 * (P(deg = k) ~ k^-alpha): the node of rank r (r = 1 is the largest) is drawn as the source of an
 * edge with probability proportional to (r + r0)^(-1/(alpha-1)), the rank-size form of that law,
 * where r0 shifts the head so that the expected largest out-degree is about max_degree.  Ranks
 * are drawn by inverting the continuous CDF in closed form (no table) and mapped to node ids by
 * a fixed multiplicative bijection modulo n; destinations are uniform over [0, n).
 */
void gg_zipf_edges(uint64_t seed, uint32_t n, uint64_t n_edges, double alpha, double max_degree,
                   uint32_t* src, uint32_t* dst)
{
    const uint64_t key = stream_key(seed, 0x5A495046ull /* "ZIPF" */);
    const double beta = 1.0 / (alpha - 1.0); /* rank-size exponent, < 1 for alpha > 2 */
    const double ob = 1.0 - beta;
    /* find r0: expected degree of the top rank = n_edges * r0^-beta / integral <= max_degree */
    double r0 = 1.0;
    for (int it = 0; it < 60; ++it) {
        double total = (pow((double)n + r0, ob) - pow(r0, ob)) / ob;
        double top = (double)n_edges * pow(r0, -beta) / total;
        if (top <= max_degree) break;
        r0 *= 1.25;
    }
    const double lo = pow(r0, ob), hi = pow((double)n + r0, ob);
    uint64_t mult = 0x9E3779B1ull % n;
    if (mult == 0) mult = 1;
    for (;;) { /* multiplier coprime with n: a bijection of the ranks onto the node ids */
        uint64_t x = mult, y = n;
        while (y) { uint64_t t = x % y; x = y; y = t; }
        if (x == 1) break;
        ++mult;
    }
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n_edges; ++i) {
        uint64_t r = draw(key, (uint64_t)i);
        double uu = ((double)(r >> 11) + 0.5) * (1.0 / 9007199254740992.0);
        double rank = pow(lo + uu * (hi - lo), 1.0 / ob) - r0;
        uint64_t rk = rank <= 0.0 ? 0 : (uint64_t)rank;
        if (rk >= n) rk = n - 1;
        uint64_t r2 = draw(key ^ 0xA5A5A5A5A5A5A5A5ull, (uint64_t)i);
        src[i] = (uint32_t)((rk * mult) % n);
        dst[i] = (uint32_t)(((r2 >> 32) * (uint64_t)n) >> 32);
    }
}

/* ---- dense tensors: rows x cols values laid out with leading dimension ld (pad = 0) ------ */

void gg_fill_uniform(uint64_t seed, uint64_t stream, int64_t rows, int64_t cols, int64_t ld,
                     double lo, double hi, float* out)
{
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float* o = out + r * ld;
        for (int64_t c = 0; c < cols; ++c) {
            uint64_t x = draw(key, (uint64_t)(r * cols + c));
            double u = ((double)(x >> 11) + 0.5) * (1.0 / 9007199254740992.0);
            o[c] = (float)(lo + (hi - lo) * u);
        }
        for (int64_t c = cols; c < ld; ++c) o[c] = 0.0f;
    }
}

/* standard normal by Box-Muller; element e uses the pair-draw floor(e/2) */
void gg_fill_normal(uint64_t seed, uint64_t stream, int64_t rows, int64_t cols, int64_t ld,
                    float* out)
{
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float* o = out + r * ld;
        for (int64_t c = 0; c < cols; ++c) {
            uint64_t e = (uint64_t)(r * cols + c);
            uint64_t x = draw(key, e >> 1);
            double u1 = ((double)(x >> 32) + 1.0) * (1.0 / 4294967296.0); /* (0, 1] */
            double u2 = (double)(x & 0xFFFFFFFFull) * (1.0 / 4294967296.0);
            double rad = sqrt(-2.0 * log(u1));
            double ang = 6.283185307179586476925286766559 * u2;
            o[c] = (float)((e & 1) ? rad * sin(ang) : rad * cos(ang));
        }
        for (int64_t c = cols; c < ld; ++c) o[c] = 0.0f;
    }
}

/* Glorot-uniform: U[-a, a], a = sqrt(6 / (fan_in + fan_out)); W is fan_in x fan_out */
void gg_fill_glorot(uint64_t seed, uint64_t stream, int64_t fan_in, int64_t fan_out, int64_t ld,
                    float* out)
{
    double a = sqrt(6.0 / (double)(fan_in + fan_out));
    gg_fill_uniform(seed, stream, fan_in, fan_out, ld, -a, a, out);
}

void gg_fill_labels(uint64_t seed, uint64_t stream, int64_t n, int32_t n_classes, int32_t* out)
{
    const uint64_t key = stream_key(seed, stream);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        uint64_t x = draw(key, (uint64_t)i);
        out[i] = (int32_t)(((x >> 32) * (uint64_t)n_classes) >> 32);
    }
}
