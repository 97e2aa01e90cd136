/*
 * terngrad.h -- C ABI of libterngrad.so: the data-parallel hot path of TernGrad
 * (layer-wise stochastic gradient ternarization, arXiv 1705.07878) on MI355X.
 *
 * One training step, worker i of N (Algorithm 1), maps onto four calls:
 *
 *   tg_clip_stats      Eq. 5 + Eq. 2   clip threshold c*sigma and local scaler, per layer
 *   tg_share_scalers   Eq. 4           shared scaler = max over workers, per layer
 *   tg_ternarize_pack  Eq. 1, 3, 5     clip -> Bernoulli(|g|/s) -> sign -> 2-bit code
 *   tg_unpack_average  Alg. 1, server  decode N code buffers, sum, rescale by s/N
 *
 * "Layer" means one tensor: the gradients of weights and of biases are
 * ternarized separately (Section 3.3, layer-wise ternarizing).  A worker's
 * gradient is the flat fp32 concatenation of its L layers; off[0..L] holds the
 * element offsets (off[0] = 0, off[L] = n, non-decreasing; empty layers allowed).
 * Finer buckets than a layer (Section 3.3) are expressed by a finer table.
 *
 * Conventions
 *   - Every function returns a tg_status; nothing throws, prints or sets errno.
 *   - "dev" pointers are device (HBM) pointers, "host" pointers are host memory.
 *     The caller owns every gradient, scaler, code and output buffer.  A plan
 *     owns only its own tables and reduction workspace.
 *   - Gradient and average pointers must be 16-byte aligned, code pointers
 *     4-byte aligned.
 *   - Compute calls are asynchronous on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream), never synchronise and never allocate.
 *   - The N workers of one machine are batched: arrays of N device pointers are
 *     passed from the host and one launch covers all of them.  A real
 *     one-worker-per-GPU deployment calls with n_workers = 1 and
 *     worker_base = its rank.
 *   - Inputs must be finite; the result for NaN/Inf gradients is unspecified
 *     (never a fault).
 *   - Threads and streams: a plan is immutable after creation except for the
 *     reduction workspace that tg_clip_stats writes.  Calls on one plan may be
 *     issued from any thread and on any stream, but two tg_clip_stats calls on
 *     the same plan must not overlap on the device (order them on one stream or
 *     with events, or use one plan per stream); all other calls only read the
 *     plan.  A plan belongs to the device that was current at tg_plan_create and
 *     must be used with streams of that device.  tg_plan_destroy does not wait
 *     for work in flight: synchronise first.
 *
 * Definitions the paper leaves open (and this library fixes)
 *   - sigma is the population standard deviation of the layer, mean subtracted.
 *   - Clipping precedes ternarizing on every worker (Section 3.3), so the
 *     scaler is the max-abs of the CLIPPED layer: s_local = min(max|g|, c*sigma).
 *   - Random numbers: Philox4x32-10, key = (lo32, hi32) of seed, counter =
 *     (lo32(q), hi32(q), worker, step) with q = e >> 3 for flat element index e;
 *     element e uses the 16-bit field (e & 7) of the 128-bit output, low half
 *     of word 0 first:  r = (out[(e&7)>>1] >> 16*(e&1)) & 0xFFFF,
 *     u = (2r + 1) / 2^17.
 *   - Eq. 3 is taken without division, in fp32:
 *       s17 = fl(s * 2^-17) ; b = [ fl((float)(2r+1) * s17) < min(|g|, c*sigma) ].
 *   - 2-bit codes: 00 = 0, 01 = +1, 11 = -1 (two's complement), four per byte,
 *     least significant pair first, flat over the layers; pad codes are 00.
 *     10 is never produced and decodes as -2.
 */
#ifndef TERNGRAD_H
#define TERNGRAD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tg_plan tg_plan;

typedef enum {
    TG_OK = 0,
    TG_ERR_INVALID_ARG = -1,      /* null pointer, bad size, offsets not monotone, ... */
    TG_ERR_ALIGNMENT = -2,        /* a device pointer is not aligned as required      */
    TG_ERR_TOO_MANY_WORKERS = -3, /* n_workers > plan's max_workers or TG_MAX_WORKERS  */
    TG_ERR_HIP = -4,              /* a HIP call failed: see tg_last_hip_error()        */
    TG_ERR_ALLOC = -5,            /* host or device allocation failed                  */
    TG_ERR_TOO_LARGE = -6         /* the job exceeds TG_STATIC_SCRATCH_BYTES           */
} tg_status;

/* The paper trains with up to N = 64 workers (Section 4.1, LeNet). */
#define TG_MAX_WORKERS 64
/* Largest model a plan accepts: 2^35 elements (128 GiB of fp32 per worker), 2^22 layers. */
#define TG_MAX_ELEMENTS ((int64_t)1 << 35)
#define TG_MAX_LAYERS ((int64_t)1 << 22)

/* ---- plan: the offset table of one model, uploaded once ------------------- */

/* Builds the tables for a model with `n_layers` tensors whose element offsets
 * are offsets[0..n_layers] (host), uploads them to the current device and
 * reserves the reduction workspace of tg_clip_stats for up to `max_workers`
 * workers per call.  Requires n_layers >= 1, offsets[0] = 0, offsets
 * non-decreasing, 1 <= offsets[n_layers] <= TG_MAX_ELEMENTS, n_layers <= TG_MAX_LAYERS,
 * 1 <= max_workers <= TG_MAX_WORKERS.
 * Errors: TG_ERR_INVALID_ARG, TG_ERR_TOO_MANY_WORKERS, TG_ERR_ALLOC, TG_ERR_HIP. */
tg_status tg_plan_create(int64_t n_layers, const int64_t* offsets, int max_workers, tg_plan** out);

/* Frees the plan's device and host memory.  NULL is accepted. */
tg_status tg_plan_destroy(tg_plan* plan);

int64_t tg_num_elements(const tg_plan* plan); /* n, or -1 for NULL */
int64_t tg_num_layers(const tg_plan* plan);   /* L, or -1 for NULL */
/* Size in bytes a code buffer must have: ceil(n/4) rounded up to a multiple of
 * 16.  The first ceil(n/4) bytes carry codes; the rest is written as 0. */
int64_t tg_packed_bytes(const tg_plan* plan);

const char* tg_strerror(int status);
/* The hipError_t of the most recent failing HIP call on this thread (0 = none). */
int tg_last_hip_error(void);

/* Host-only: the tables tg_plan_create derives from an offset table, exported
 * so that they can be checked without a GPU.
 *   tile_layer[t]  = layer holding element t * tile (tile = *tile_elems)
 *   tile_whole[t]  = 1 when no other layer begins inside [t * tile, min((t+1) * tile, n)), else 0
 *   seg[3*i..]     = (layer, begin, end) of the i-th reduction segment: a maximal
 *                    run of elements inside one layer and one statistics chunk
 *                    of *chunk_elems elements (8192 to 65536, chosen from
 *                    n * max_workers)
 * Pass NULL arrays (or too small capacities) to query the sizes only. */
tg_status tg_describe_tables(int64_t n_layers, const int64_t* offsets, int max_workers,
                             int64_t* tile_elems, int64_t* n_tiles, int32_t* tile_layer, uint8_t* tile_whole,
                             int64_t tile_cap,
                             int64_t* chunk_elems, int64_t* n_segments, int64_t* seg, int64_t seg_cap);

/* ---- the four calls of the hot path --------------------------------------- */

/* Eq. 5 and Eq. 2, for n_workers gradients in one launch.
 *   grads    host array of n_workers dev pointers, each to n fp32
 *   c        clip constant (the paper uses 2.5); c <= 0 or +inf = no clipping
 *            (the "TernGrad-noclip" row of Table 2): tau = +inf, s_local = max|g|
 *   tau      dev [n_workers][L] out: c * sigma of each layer of each worker
 *   s_local  dev [n_workers][L] out: min(max|g|, tau)
 * Sums of (g - K) and (g - K)^2 are accumulated in fp64 about the pivot K = first element of the
 * layer, in a fixed order: results are identical from run to run, exact for a constant layer, and
 * within 1e-7 relative of a two-pass fp64 computation whenever sigma >= 1e-3 |mean - K| (relative
 * error about 1e-14 (1 + (mean - K)^2 / sigma^2)).  An empty layer gets tau = 0 (or +inf without
 * clipping) and s_local = 0. */
tg_status tg_clip_stats(tg_plan* plan, int n_workers, const float* const* grads, float c,
                        float* tau, float* s_local, void* stream);

/* For callers that cannot allocate device memory or want no workspace tied to a plan: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  tg_clip_stats with its
 * per-segment partial sums in a fixed buffer of TG_STATIC_SCRATCH_BYTES that is part of the loaded
 * library (static device memory, one copy per GPU, held until the process ends) instead of the
 * plan's workspace.  Arguments and results are those of tg_clip_stats, bit for bit.  Between being
 * called and returning it calls no hipMalloc, hipFree or other allocating routine (the address of
 * the buffer on the plan's device was resolved in tg_plan_create).
 *   - n_workers may exceed the plan's max_workers (up to TG_MAX_WORKERS): the plan's workspace is unused.
 *   - The job must fit: tg_static_scratch_needed(plan, n_workers) <= TG_STATIC_SCRATCH_BYTES
 *     (20 bytes per reduction segment and worker; the flat 10^9-element, 8-worker job needs 9.8 MB),
 *     else TG_ERR_TOO_LARGE and nothing is launched.
 *   - Every call on a GPU, from any plan, thread or stream, shares that GPU's one buffer: calls that
 *     overlap on the device race.  Order them on one stream or with events.  The buffer keeps the
 *     last call's partial sums; nothing in it has to be cleared between calls.
 *   - The current device must be the plan's device. */
#define TG_STATIC_SCRATCH_BYTES (16 * 1024 * 1024)
int64_t tg_static_scratch_needed(const tg_plan* plan, int n_workers); /* bytes, or -1 for bad arguments */
tg_status tg_clip_stats_static(tg_plan* plan, int n_workers, const float* const* grads, float c,
                               float* tau, float* s_local, void* stream);

/* Eq. 4: s_shared[l] = max_w s_local[w][l].
 *   s_local  dev [n_workers][L] in ; s_shared dev [L] out.
 * Across GPUs this is the max-all-reduce of L floats per worker (the "2N
 * floating scalars" of Section 3.1); here the N rows sit in one buffer. */
tg_status tg_share_scalers(tg_plan* plan, int n_workers, const float* s_local,
                           float* s_shared, void* stream);

/* Eq. 1 + 3 + 5 and the 2-bit encoding, for n_workers gradients in one launch.
 *   grads        host array of n_workers dev pointers (n fp32 each)
 *   tau          dev [n_workers][L] in (each worker clips with its own sigma)
 *   s_shared     dev [L] in
 *   seed, step   RNG key and iteration counter t; worker w of this call draws
 *                with worker id worker_base + w
 *   codes        host array of n_workers dev pointers, each to tg_packed_bytes() bytes, out */
tg_status tg_ternarize_pack(tg_plan* plan, int n_workers, uint32_t worker_base,
                            const float* const* grads, const float* tau, const float* s_shared,
                            uint64_t seed, uint32_t step, uint8_t* const* codes, void* stream);

/* The same with the iteration counter t read from device memory at run time: a step recorded
 * once into a HIP graph (these calls allocate nothing and never synchronise, so they can be
 * captured) is replayed with a fresh random stream each time by advancing *step_dev between
 * replays, e.g. with tg_step_advance as the graph's last node.  For the callers whose step is
 * launch-bound (small models: five short launches).
 *   step_dev  dev pointer to one uint32, 4-byte aligned, read by the kernel */
tg_status tg_ternarize_pack_devstep(tg_plan* plan, int n_workers, uint32_t worker_base,
                                    const float* const* grads, const float* tau, const float* s_shared,
                                    uint64_t seed, const uint32_t* step_dev, uint8_t* const* codes, void* stream);

/* *step_dev += by, as a one-thread kernel on `stream` (no memset or memcpy node is involved). */
tg_status tg_step_advance(uint32_t* step_dev, uint32_t by, void* stream);

/* Algorithm 1, server line: avg[e] = (sum_w t_w[e]) * (s_shared[layer(e)] / n_workers),
 * the integer sum exact, one fp32 division per layer and one fp32 product per element.
 *   codes     host array of n_workers dev pointers to code buffers, in
 *   s_shared  dev [L] in
 *   avg       dev [n] fp32 out (at most 2N+1 distinct values per layer) */
tg_status tg_unpack_average(tg_plan* plan, int n_workers, const uint8_t* const* codes,
                            const float* s_shared, float* avg, void* stream);

/* ---- beyond the four calls: the next line of Algorithm 1 ------------------- */

/* Algorithm 1, worker lines "pull averaged gradients" + "update parameters" in one pass:
 *   weights[e] <- weights[e] - eta * (sum_w t_w[e]) * (s_shared[layer(e)] / n_workers)
 * with the average formed exactly as in tg_unpack_average and applied with one fused
 * multiply-add; it is never written to memory.  Under parameter localization (Section 3)
 * every worker runs this on its own copy of the parameters.
 *   codes, s_shared  as for tg_unpack_average
 *   eta              learning rate (finite)
 *   weights          dev [n] fp32, in/out, 16-byte aligned */
tg_status tg_unpack_update(tg_plan* plan, int n_workers, const uint8_t* const* codes,
                           const float* s_shared, float eta, float* weights, void* stream);

/* Algorithm 1, server line, WITHOUT scaler sharing: every worker ternarized with its own scaler
 * (call tg_ternarize_pack once per worker with that worker's row of s_local in place of s_shared),
 * which is the situation the text before Eq. 4 starts from:
 *   avg[e] = (1/N) * sum_i s_workers[i][layer(e)] * t_i(e)
 * summed per element in fp64 in worker order and rounded to fp32 once (within 1e-6 of the exact
 * mean relative to mean_i |s_i t_i|; exactly 0 where every t is 0).  With equal rows it agrees
 * with tg_unpack_average to that tolerance.  Up to 3^N levels per layer instead of 2N+1.
 *   s_workers  dev [n_workers][L] fp32, e.g. the s_local of tg_clip_stats
 *   avg        dev [n] fp32 out, 16-byte aligned */
tg_status tg_unpack_average_scalers(tg_plan* plan, int n_workers, const uint8_t* const* codes,
                                    const float* s_workers, float* avg, void* stream);

/* Tuning knob of tg_unpack_update and tg_unpack_update_momentum.  They have two kernels with
 * bit-identical results: a workgroup-cooperative one (four tiles of 1024 elements per workgroup,
 * faster while the weights fit the memory-side cache) and one with a wave per 256 elements (faster
 * from about 1 GiB of weights on); mode 0 (the default) picks by the size of the model, 1 forces the
 * first, 2 the second.  Applies to later calls on this plan.  TG_ERR_INVALID_ARG for other modes. */
tg_status tg_plan_set_update_kernel(tg_plan* plan, int mode);

/* The same with momentum (the optimizer of most experiments in Section 4):
 *   velocity[e] <- mu * velocity[e] + avg[e] ;  weights[e] <- weights[e] - eta * velocity[e]
 * (two fused multiply-adds; mu = 0 reproduces tg_unpack_update and leaves avg in velocity).
 *   velocity, weights  dev [n] fp32, in/out, 16-byte aligned, distinct buffers; eta, mu finite */
tg_status tg_unpack_update_momentum(tg_plan* plan, int n_workers, const uint8_t* const* codes,
                                    const float* s_shared, float eta, float mu, float* velocity,
                                    float* weights, void* stream);

/* Server-to-worker pull (Section 3.1): with parameter localization and a shared scaler the
 * averaged gradient has at most 2N+1 levels k * s/N, so it can travel as the integer
 * k = sum_w t_w in a narrow field instead of a 32-bit float (the paper's 32 / log2(1+2N)).
 * Fields are `bits`-wide two's complement, 2 <= bits <= 8, and the buffer is one little-endian bit
 * stream: bit j of field e is bit (e*bits + j) & 7 of byte (e*bits + j) >> 3 (bits = 4: element e
 * in nibble e & 1 of byte e >> 1; bits = 8: byte e).  A width holds the sums of n_workers workers
 * when n_workers < 2^(bits-1) (8 bits: every n_workers <= 64); tg_sum_bits(N) = ceil(log2(2N+1))
 * is the narrowest such width, the paper's figure: 3, 4, 5 bits for N = 2, 4, 8.  Widths 4 and 8
 * have their own (faster) kernels.
 * A buffer holds tg_sum_bytes(plan, bits) = ceil(n*bits/8) rounded up to 16 bytes, 16-byte
 * aligned; pad bits are written as 0.  Codes must be valid (no 10): only the low `bits`
 * bits of k are kept. */
int tg_sum_bits(int n_workers);                         /* -1 unless 1 <= n_workers <= TG_MAX_WORKERS */
int64_t tg_sum_bytes(const tg_plan* plan, int bits);   /* -1 for a NULL plan or bits outside 2..8 */

/* The server's side: decode the N code buffers, sum, write k.  ksum: dev, out. */
tg_status tg_unpack_sum_pack(tg_plan* plan, int n_workers, const uint8_t* const* codes, int bits,
                             uint8_t* ksum, void* stream);

/* The worker's side: avg[e] = k[e] * (s_shared[layer(e)] / n_workers), exactly the value
 * tg_unpack_average produces from the codes the sums came from.  n_workers is the N the sums
 * were formed over (it need not fit the plan's max_workers: no per-worker buffer is touched). */
tg_status tg_decode_sum(tg_plan* plan, int n_workers, const uint8_t* ksum, int bits,
                        const float* s_shared, float* avg, void* stream);

/* Denser container, toward the bound 32/log2(3) = 20.18x of Section 3.1: five ternary values per
 * byte (1.6 bits each, 20x smaller than fp32 instead of 16x).  Digit d = t mod 3 (0 -> 0, +1 -> 1,
 * -1 -> 2); byte j holds elements 5j..5j+4 as d0 + 3 d1 + 9 d2 + 27 d3 + 81 d4.  Clip, random
 * field and Bernoulli draw are those of tg_ternarize_pack: the ternary values are identical.
 * A buffer holds tg_packed_bytes_base3(plan) = ceil(n/5) rounded up to 16 bytes, 4-byte aligned;
 * pad digits and pad bytes are written as 0.  Arguments as for tg_ternarize_pack /
 * tg_unpack_average. */
int64_t tg_packed_bytes_base3(const tg_plan* plan);
tg_status tg_ternarize_pack_base3(tg_plan* plan, int n_workers, uint32_t worker_base,
                                  const float* const* grads, const float* tau, const float* s_shared,
                                  uint64_t seed, uint32_t step, uint8_t* const* codes3, void* stream);
tg_status tg_unpack_average_base3(tg_plan* plan, int n_workers, const uint8_t* const* codes3,
                                  const float* s_shared, float* avg, void* stream);

/* Layers kept in floating point.  Section 4.2 does not ternarize the last classification
 * layer; its gradients travel as fp32 and are averaged as such:
 *   avg[e] = (float)( (sum_w (double)grads[w][e]) / n_workers ),  e in [0, n)
 * (fp64 sum in worker order, one rounding).  Needs no plan: the caller builds the plan over the
 * ternarized layers only and hands the float layers' slice of each flat buffer to this call.  A float
 * layer in the middle of the buffer is handled the same way with two plans, one over the layers before
 * it and one over the layers after it, both called on the same buffers at their offsets; the slice must
 * then begin and end at a multiple of four elements (the alignment the plans' calls require); for other
 * layouts see tg_plan_set_layer_modes below.
 *   grads  host array of n_workers dev pointers, each to n fp32
 *   avg    dev [n] fp32 out
 * The pointers need only be float addresses, but all of them (avg included) must be congruent
 * modulo 16 bytes, as the same slice of equally laid out flat buffers is; else TG_ERR_ALIGNMENT. */
tg_status tg_average_float(int n_workers, int64_t n, const float* const* grads, float* avg, void* stream);

/* The same as a per-layer mode of ONE plan (Section 4.2 keeps the last classification layer in floating
 * point; here any layers, anywhere in the flat buffer, at any alignment).  layer_float: host array of L bytes, 1 = the layer is
 * kept in floating point, 0 = ternarized (the default for every layer); null resets all layers to 0;
 * other values TG_ERR_INVALID_ARG.  From then on, on this plan:
 *   - tg_clip_stats (and tg_clip_stats_static) writes tau = 0 and s_local = 0 for those layers, so that
 *     tg_share_scalers yields 0 and tg_ternarize_pack encodes every one of their elements as 00,
 *     whatever the gradients hold (NaN and Inf included): their codes carry nothing;
 *   - tg_unpack_average_mixed is tg_unpack_average followed, for the layers kept in floating point,
 *     by the mean of tg_average_float over their elements (same arithmetic, same tolerance); the
 *     ternarized layers come out exactly as from tg_unpack_average.  grads: host array of n_workers
 *     dev pointers to the workers' flat gradient buffers (what tg_clip_stats was given); may be null
 *     when no layer is kept in floating point.
 * Every other call treats such a layer as a layer with scaler 0: tg_unpack_average and the fused updates
 * leave the weights of those layers to the caller.  The passes still read the float layers' gradients
 * and write their (zero) codes: where the layout allows it (float layers at the end, boundaries at
 * multiples of four elements) a plan over the ternarized layers only plus tg_average_float moves fewer bytes.
 * The flags are copied to the device with a blocking copy: set them before the plan is in use, or
 * after the calls queued on it have finished. */
tg_status tg_plan_set_layer_modes(tg_plan* plan, const uint8_t* layer_float);
tg_status tg_unpack_average_mixed(tg_plan* plan, int n_workers, const uint8_t* const* codes,
                                  const float* const* grads, const float* s_shared, float* avg, void* stream);

#ifdef __cplusplus
}
#endif
#endif
