/*
 * tg_oracle.c -- CPU oracle for the TernGrad hot path (arXiv 1705.07878).
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT: see tg_oracle.h.  Plain C, one element
 * at a time, fp64 two-pass statistics, no blocking or fusion.  The only
 * concession to run time is an optional OpenMP "parallel for" over elements,
 * legal because every element's random field depends on its index alone.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC tg_oracle.c -lm
 * (-ffp-contract=off: the Bernoulli draw is defined by separately rounded fp32
 * operations.)
 */
#include "tg_oracle.h"

#include <float.h>
#include <math.h>
#include <stddef.h>

#if defined(FLT_EVAL_METHOD) && FLT_EVAL_METHOD != 0
#error "float expressions must be evaluated in fp32 (FLT_EVAL_METHOD == 0)"
#endif

#ifdef _OPENMP
#include <omp.h>
#endif

static int g_threads = 1;

int tgo_set_threads(int n_threads) {
    if (n_threads >= 1) g_threads = n_threads;
#ifndef _OPENMP
    g_threads = 1;
#endif
    return g_threads;
}

/* ---- Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11).  Multipliers and Weyl key increments are the
 * published ones. ---- */
static const uint32_t PHILOX_M0 = 0xD2511F53u;
static const uint32_t PHILOX_M1 = 0xCD9E8D57u;
static const uint32_t PHILOX_W0 = 0x9E3779B9u; /* golden ratio */
static const uint32_t PHILOX_W1 = 0xBB67AE85u; /* sqrt(3) - 1   */

void tgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += PHILOX_W0; k1 += PHILOX_W1; }
        uint64_t p0 = (uint64_t)PHILOX_M0 * c0;
        uint64_t p1 = (uint64_t)PHILOX_M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

uint32_t tgo_random_field(uint64_t seed, uint32_t step, uint32_t worker, uint64_t e) {
    uint64_t q = e >> 3;
    uint32_t ctr[4] = { (uint32_t)q, (uint32_t)(q >> 32), worker, step };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    tgo_philox4x32_10(ctr, key, out);
    unsigned h = (unsigned)(e & 7u);
    return (out[h >> 1] >> (16u * (h & 1u))) & 0xFFFFu;
}

/* Eq. 3: P(b = 1) = |g| / s, realised as u * s < |g| with u = (2r+1) / 2^17. */
int tgo_bernoulli(uint32_t r, float s, float a) {
    const float s17 = s * 0x1p-17f;                 /* one fp32 rounding */
    const float thr = (float)(2u * r + 1u) * s17;   /* one fp32 rounding */
    return thr < a;
}

/* layer that holds flat index e: the l with off[l] <= e < off[l+1] */
static int64_t layer_of(int64_t e, int64_t n_layers, const int64_t* off) {
    int64_t l = 0;
    while (l + 1 < n_layers && e >= off[l + 1]) ++l;
    return l;
}

void tgo_clip_stats(const float* g, int64_t n_layers, const int64_t* off, float c,
                    float* tau, float* s_local) {
    const int noclip = !(c > 0.0f) || isinf(c);
    for (int64_t l = 0; l < n_layers; ++l) {
        const int64_t lo = off[l], hi = off[l + 1], cnt = hi - lo;
        double sigma = 0.0;
        float m = 0.0f;
        if (cnt > 0) {
            double sum = 0.0;
            #pragma omp parallel for reduction(+:sum) num_threads(g_threads) schedule(static)
            for (int64_t e = lo; e < hi; ++e) sum += (double)g[e];
            const double mu = sum / (double)cnt;
            double ss = 0.0;
            #pragma omp parallel for reduction(+:ss) num_threads(g_threads) schedule(static)
            for (int64_t e = lo; e < hi; ++e) {
                const double d = (double)g[e] - mu;
                ss += d * d;
            }
            sigma = sqrt(ss / (double)cnt);           /* population std (Eq. 5's sigma) */
            #pragma omp parallel for reduction(max:m) num_threads(g_threads) schedule(static)
            for (int64_t e = lo; e < hi; ++e) {
                const float ab = fabsf(g[e]);
                if (ab > m) m = ab;
            }
        }
        const float t = noclip ? INFINITY : (float)((double)c * sigma);
        tau[l] = t;
        s_local[l] = (m < t) ? m : t;                 /* Eq. 2 on the clipped layer */
    }
}

void tgo_share_scalers(const float* s_local, int n_workers, int64_t n_layers, float* s_shared) {
    for (int64_t l = 0; l < n_layers; ++l) {
        float m = s_local[l];
        for (int w = 1; w < n_workers; ++w) {
            const float v = s_local[(int64_t)w * n_layers + l];
            if (v > m) m = v;
        }
        s_shared[l] = m;                              /* Eq. 4 */
    }
}

/* Eq. 5, Eq. 3, Eq. 1 (without s) for one element: the ternary value t in {-1, 0, +1} */
static int ternary_value(const float* g, int64_t e, int64_t n_layers, const int64_t* off,
                         const float* tau, const float* s_shared,
                         uint64_t seed, uint32_t step, uint32_t worker) {
    const int64_t l = layer_of(e, n_layers, off);
    const float ge = g[e];
    const float a = fminf(fabsf(ge), tau[l]);                         /* Eq. 5 */
    const uint32_t r = tgo_random_field(seed, step, worker, (uint64_t)e);
    const int b = tgo_bernoulli(r, s_shared[l], a);                   /* Eq. 3 */
    return b ? (signbit(ge) ? -1 : 1) : 0;                            /* Eq. 1 without s */
}

void tgo_ternarize_pack(const float* g, int64_t n_layers, const int64_t* off,
                        const float* tau, const float* s_shared,
                        uint64_t seed, uint32_t step, uint32_t worker, uint8_t* codes) {
    const int64_t n = off[n_layers];
    const int64_t n_bytes = (n + 3) / 4;
    /* one byte = four consecutive elements; bytes are independent */
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t byte = 0; byte < n_bytes; ++byte) {
        unsigned packed = 0;
        for (int j = 0; j < 4; ++j) {
            const int64_t e = 4 * byte + j;
            if (e >= n) break;                        /* pad codes stay 00 */
            const int t = ternary_value(g, e, n_layers, off, tau, s_shared, seed, step, worker);
            packed |= ((unsigned)t & 3u) << (2 * j);
        }
        codes[byte] = (uint8_t)packed;
    }
}

int tgo_code_at(const uint8_t* codes, int64_t e) {
    const unsigned f = (codes[e >> 2] >> (2 * (e & 3))) & 3u;
    return (f & 2u) ? (int)f - 4 : (int)f;            /* two's complement, 2 bits */
}

void tgo_unpack_average(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                        const int64_t* off, const float* s_shared, float* avg) {
    const int64_t n = off[n_layers];
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        const int64_t l = layer_of(e, n_layers, off);
        long k = 0;
        for (int w = 0; w < n_workers; ++w) k += tgo_code_at(codes[w], e);
        avg[e] = (float)((double)k * (double)s_shared[l] / (double)n_workers);
    }
}

/* Algorithm 1, server line, when every worker keeps its own scaler (no scaler sharing, the case the
 * text before Eq. 4 describes): avg_e = (1/N) * sum_i s_l^(i) * t_i(e). */
void tgo_unpack_average_scalers(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                                const int64_t* off, const float* s_workers, float* avg) {
    const int64_t n = off[n_layers];
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        const int64_t l = layer_of(e, n_layers, off);
        double sum = 0.0;
        for (int w = 0; w < n_workers; ++w)
            sum += (double)s_workers[(int64_t)w * n_layers + l] * (double)tgo_code_at(codes[w], e);
        avg[e] = (float)(sum / (double)n_workers);
    }
}

void tgo_unpack_update(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                       const int64_t* off, const float* s_shared, float eta, float* weights) {
    const int64_t n = off[n_layers];
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        const int64_t l = layer_of(e, n_layers, off);
        long k = 0;
        for (int w = 0; w < n_workers; ++w) k += tgo_code_at(codes[w], e);
        const double avg = (double)k * (double)s_shared[l] / (double)n_workers;
        weights[e] = (float)((double)weights[e] - (double)eta * avg);
    }
}

void tgo_average_float(const float* const* grads, int n_workers, int64_t n, float* avg) {
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        double sum = 0.0;
        for (int w = 0; w < n_workers; ++w) sum += (double)grads[w][e];
        avg[e] = (float)(sum / (double)n_workers);
    }
}

int tgo_sum_bits(int n_workers) {
    /* smallest width whose 2^bits values hold the 2N+1 levels -N .. N (Section 3.1) */
    int bits = 1;
    while ((1L << bits) < 2L * n_workers + 1) ++bits;
    return bits;
}

void tgo_sum_pack(const uint8_t* const* codes, int n_workers, int64_t n, int bits, uint8_t* ksum) {
    const int64_t n_bytes = (n * bits + 7) / 8;
    for (int64_t i = 0; i < n_bytes; ++i) ksum[i] = 0;
    for (int64_t e = 0; e < n; ++e) {
        long k = 0;
        for (int w = 0; w < n_workers; ++w) k += tgo_code_at(codes[w], e);
        /* the buffer is one little-endian bit stream: bit j of field e is stream bit e*bits + j */
        for (int j = 0; j < bits; ++j) {
            const int64_t pos = e * bits + j;
            if ((k >> j) & 1L) ksum[pos >> 3] |= (uint8_t)(1u << (pos & 7));
        }
    }
}

void tgo_decode_sum(const uint8_t* ksum, int bits, int n_workers, int64_t n_layers,
                    const int64_t* off, const float* s_shared, float* avg) {
    const int64_t n = off[n_layers];
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        const int64_t l = layer_of(e, n_layers, off);
        int f = 0;
        for (int j = 0; j < bits; ++j) {
            const int64_t pos = e * bits + j;
            f |= ((ksum[pos >> 3] >> (pos & 7)) & 1) << j;
        }
        const int k = (f & (1 << (bits - 1))) ? f - (1 << bits) : f;     /* two's complement, `bits` wide */
        avg[e] = (float)((double)k * (double)s_shared[l] / (double)n_workers);
    }
}

void tgo_unpack_update_momentum(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                                const int64_t* off, const float* s_shared, float eta, float mu,
                                float* velocity, float* weights) {
    const int64_t n = off[n_layers];
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        const int64_t l = layer_of(e, n_layers, off);
        long k = 0;
        for (int w = 0; w < n_workers; ++w) k += tgo_code_at(codes[w], e);
        const double avg = (double)k * (double)s_shared[l] / (double)n_workers;
        const double v = (double)mu * (double)velocity[e] + avg;
        velocity[e] = (float)v;
        weights[e] = (float)((double)weights[e] - (double)eta * v);
    }
}

void tgo_ternarize_pack_base3(const float* g, int64_t n_layers, const int64_t* off,
                              const float* tau, const float* s_shared,
                              uint64_t seed, uint32_t step, uint32_t worker, uint8_t* codes3) {
    const int64_t n = off[n_layers];
    const int64_t n_bytes = (n + 4) / 5;
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t byte = 0; byte < n_bytes; ++byte) {
        unsigned packed = 0, weight = 1;
        for (int j = 0; j < 5; ++j, weight *= 3) {
            const int64_t e = 5 * byte + j;
            if (e >= n) break;                        /* pad digits stay 0 */
            const int t = ternary_value(g, e, n_layers, off, tau, s_shared, seed, step, worker);
            packed += weight * (unsigned)((t + 3) % 3);
        }
        codes3[byte] = (uint8_t)packed;
    }
}

int tgo_trit_at(const uint8_t* codes3, int64_t e) {
    unsigned v = codes3[e / 5] % 243u;
    for (int j = 0; j < (int)(e % 5); ++j) v /= 3;
    const int d = (int)(v % 3);
    return d == 2 ? -1 : d;
}

void tgo_unpack_average_base3(const uint8_t* const* codes3, int n_workers, int64_t n_layers,
                              const int64_t* off, const float* s_shared, float* avg) {
    const int64_t n = off[n_layers];
    #pragma omp parallel for num_threads(g_threads) schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        const int64_t l = layer_of(e, n_layers, off);
        long k = 0;
        for (int w = 0; w < n_workers; ++w) k += tgo_trit_at(codes3[w], e);
        avg[e] = (float)((double)k * (double)s_shared[l] / (double)n_workers);
    }
}
