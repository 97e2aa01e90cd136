/*
 * tg_oracle.h -- CPU oracle for the TernGrad hot path (arXiv 1705.07878).
 *
 * TEST INFRASTRUCTURE, NOT THE PRODUCT.  This is a plain, slow, obviously
 * correct host implementation of what the hot path computes, written from the
 * paper's definitions (Section 3.1 Eq. 1-4, Section 3.3 Eq. 5, Algorithm 1).
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg
 * may call it.  It shares no source, header, table or helper with the HIP
 * library and neither side includes the other.
 *
 * All pointers are HOST pointers.  All reductions are fp64, two-pass.
 *
 * Notation (paper): g = gradient vector of one layer of one worker, s = scaler
 * (Eq. 2 / Eq. 4), b = Bernoulli vector (Eq. 3), c*sigma = clip threshold
 * (Eq. 5), N = W = number of workers.  "Layer" = one tensor: weights and
 * biases are separate layers (Section 3.3, layer-wise ternarizing).
 * Layers are given as a flat concatenation with an offset table
 * off[0..L], off[0] = 0, off[L] = n, non-decreasing.
 *
 * Parity pins (see tests/test_oracle_*.py):
 *   - Philox4x32-10 block function: pinned against an independent public
 *     implementation compiled at test time.
 *   - Bernoulli decision: exhaustive enumeration of the 65,536 random fields.
 *   - population-vs-sample standard deviation: PARITY UNPINNED (the paper only
 *     says "standard deviation"; population, mean-subtracted is the reading).
 */
#ifndef TG_ORACLE_H
#define TG_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Number of OpenMP threads the element-wise loops may use (default 1).
 * Results do not depend on it: the generator is counter based. Returns the
 * value now in force. */
int tgo_set_threads(int n_threads);

/* Philox4x32 with 10 rounds (Salmon et al., SC'11): one 128-bit counter block
 * under a 64-bit key -> four 32-bit words. */
void tgo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The 16-bit random field r in [0, 65535] assigned to flat element index e of
 * `worker` at `step` under `seed`:
 *   block q = e >> 3 ; counter = (lo32(q), hi32(q), worker, step) ;
 *   key = (lo32(seed), hi32(seed)) ; h = e & 7 ;
 *   r = (out[h >> 1] >> (16 * (h & 1))) & 0xFFFF.
 * The uniform variate is u = (r + 1/2) / 2^16 = (2r + 1) / 2^17. */
uint32_t tgo_random_field(uint64_t seed, uint32_t step, uint32_t worker, uint64_t e);

/* Eq. 3: the Bernoulli draw b = [u * s < a], taken in fp32 as
 *   s17 = fl32(s * 2^-17) ; thr = fl32((float)(2r + 1) * s17) ; b = (thr < a).
 * a = |clipped gradient|.  No division: s = 0 gives b = (0 < a). */
int tgo_bernoulli(uint32_t r, float s, float a);

/* Eq. 5 + Eq. 2, one worker.  Per layer l (fp64, two passes):
 *   mu = mean(g_l) ; sigma = sqrt(mean((g_l - mu)^2)) ; tau_l = (float)(c * sigma)
 *   s_local_l = min(max|g_l|, tau_l)   (= max |clip(g_l)|)
 * c <= 0 or c = +inf means "no clipping": tau_l = +inf, s_local_l = max|g_l|.
 * An empty layer gets sigma = 0 and max = 0.
 * g: [n] ; tau, s_local: [L]. */
void tgo_clip_stats(const float* g, int64_t n_layers, const int64_t* off, float c,
                    float* tau, float* s_local);

/* Eq. 4: s_shared[l] = max_w s_local[w*L + l]. */
void tgo_share_scalers(const float* s_local, int n_workers, int64_t n_layers, float* s_shared);

/* Eq. 1 + Eq. 3 + Eq. 5 + 2-bit code, one worker.  For flat index e in layer l:
 *   a = min(|g_e|, tau_l) ; r = tgo_random_field(seed, step, worker, e)
 *   b = tgo_bernoulli(r, s_shared_l, a) ; t = b ? (signbit(g_e) ? -1 : +1) : 0
 * code = t & 3 (00 = 0, 01 = +1, 11 = -1), stored LSB first, four per byte:
 * byte e >> 2 holds code << 2*(e & 3).  Writes exactly ceil(n/4) bytes; pad
 * codes in the last byte are 00.  tau: this worker's [L]; s_shared: [L]. */
void tgo_ternarize_pack(const float* g, int64_t n_layers, const int64_t* off,
                        const float* tau, const float* s_shared,
                        uint64_t seed, uint32_t step, uint32_t worker, uint8_t* codes);

/* The ternary value t in {-2,-1,0,+1} held by element e of a code buffer: the
 * 2-bit field read as a two's-complement number (10 = -2 is never produced by
 * tgo_ternarize_pack and is decoded literally). */
int tgo_code_at(const uint8_t* codes, int64_t e);

/* Algorithm 1, server line, with the shared scaler:
 *   k_e = sum_w t_w(e) (exact integer) ; avg_e = (float)((double)k_e * s_shared_l / W).
 * codes: W host pointers to ceil(n/4)-byte buffers; avg: [n]. */
void tgo_unpack_average(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                        const int64_t* off, const float* s_shared, float* avg);

/* Algorithm 1, worker line "update parameters", applied directly to the pulled codes:
 *   w_e <- (float)( (double)w_e - (double)eta * k_e * s_shared_l / W ),
 * i.e. w - eta * avg with avg as in tgo_unpack_average but never rounded to fp32.
 * weights: [n], updated in place. */
void tgo_unpack_update(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                       const int64_t* off, const float* s_shared, float eta, float* weights);

/* Algorithm 1, server line, WITHOUT scaler sharing (every worker ternarized with its own scaler
 * s^(i), the situation the text before Eq. 4 starts from):
 *   avg_e = (float)( (sum_i (double)s_workers[i][l] * t_i(e)) / N ),
 * summed in worker order (each product is exact).  s_workers: [W][L] row-major.  With equal rows
 * the result is that of tgo_unpack_average, bit for bit (k*s is exact in fp64 for N <= 64). */
void tgo_unpack_average_scalers(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                                const int64_t* off, const float* s_workers, float* avg);

/* Denser encoding toward the information bound 32/log2(3) = 20.18x of Section 3.1: five ternary
 * values per byte (1.6 bits each, 20x).  Digit d = t mod 3 (0 -> 0, +1 -> 1, -1 -> 2); byte j holds
 * elements 5j .. 5j+4 as d0 + 3*d1 + 9*d2 + 27*d3 + 81*d4 (0..242).  Same clip, same random field
 * and same Bernoulli draw as tgo_ternarize_pack: the ternary values are identical, only the
 * container differs.  Writes ceil(n/5) bytes; pad digits are 0. */
void tgo_ternarize_pack_base3(const float* g, int64_t n_layers, const int64_t* off,
                              const float* tau, const float* s_shared,
                              uint64_t seed, uint32_t step, uint32_t worker, uint8_t* codes3);

/* ternary value of element e of a base-3 buffer (a byte above 242 yields digits of byte mod 243) */
int tgo_trit_at(const uint8_t* codes3, int64_t e);

/* tgo_unpack_average over base-3 buffers. */
void tgo_unpack_average_base3(const uint8_t* const* codes3, int n_workers, int64_t n_layers,
                              const int64_t* off, const float* s_shared, float* avg);

/* Layers kept in floating point (Section 4.2: the last classification layer is not
 * ternarized): the plain average avg_e = (float)( (sum_w (double)g_w[e]) / W ), summed in
 * worker order.  grads: W host pointers to n floats; avg: [n]. */
void tgo_average_float(const float* const* grads, int n_workers, int64_t n, float* avg);

/* The same update with momentum, the optimizer most of the paper's experiments use (Section 4):
 *   v_e <- (float)( mu * v_e + avg_e ) ;  w_e <- (float)( w_e - eta * v_e(new, unrounded) ),
 * avg_e = k_e * s_shared_l / W, everything in fp64, each output rounded once. */
void tgo_unpack_update_momentum(const uint8_t* const* codes, int n_workers, int64_t n_layers,
                                const int64_t* off, const float* s_shared, float eta, float mu,
                                float* velocity, float* weights);

/* Server-to-worker pull with parameter localization + scaler sharing (Section 3.1): the
 * averaged gradient has at most 2N+1 levels k * s/N, so the server sends the integer
 * k_e = sum_w t_w(e) in a `bits`-wide two's-complement field instead of a 32-bit float;
 * tgo_sum_bits(N) = ceil(log2(2N+1)) is the narrowest width that holds -N .. N (3, 4, 5 bits for
 * N = 2, 4, 8).  The buffer is one little-endian bit stream: bit j of field e is bit (e*bits + j) & 7
 * of byte (e*bits + j) >> 3 (bits = 4: element e in nibble e & 1 of byte e >> 1; bits = 8: byte e).
 * Writes ceil(n * bits / 8) bytes; pad bits are 0.  Only the low `bits` bits of k are kept.
 * 2 <= bits <= 8. */
int tgo_sum_bits(int n_workers);
void tgo_sum_pack(const uint8_t* const* codes, int n_workers, int64_t n, int bits, uint8_t* ksum);

/* The worker's side of that pull: avg_e = (float)((double)k_e * s_shared_l / W), k_e the
 * sign-extended field.  Same result as tgo_unpack_average on the codes the sums came from. */
void tgo_decode_sum(const uint8_t* ksum, int bits, int n_workers, int64_t n_layers,
                    const int64_t* off, const float* s_shared, float* avg);

#ifdef __cplusplus
}
#endif
#endif
