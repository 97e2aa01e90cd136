// Fused clip -> Bernoulli -> sign -> 2-bit pack (Eq. 1, 3, 5 and the 2-bit
// encoding of Section 3.1).  The unit of all tables is the tile of 1024 consecutive
// gradients (256 bytes of codes), four quarters of 256; a wave encodes NQ quarters:
// half a tile in the 2-bit kernel (measured 2 - 4 % faster than a whole tile per wave
// on every size: 5.26 against 5.35 ms on 8 x 10^9 elements, 0.672 against 0.701 ms
// on the VGG-A shapes; a quarter per wave is slower again), a whole tile in the
// base-3 kernel.
//   * NQ fully coalesced 128-bit loads per lane (lane l, load k reads
//     elements 256k + 4l .. 4l+3 of the wave's part), issued before anything that
//     depends on the layer tables, so table and data latencies overlap;
//   * one Philox4x32-10 block yields the 16-bit fields of 8 consecutive
//     elements, so lanes 2j and 2j+1 each compute one block per pair of quarters (for
//     elements 8j..8j+7 of two consecutive 256-element quarters) and swap halves over DPP;
//   * per element: fp32 threshold fma, clip-min, integer compare, two
//     funnel shifts that push the "non-zero" and "negative" bits into the byte;
//   * the NQ code bytes of a lane are transposed through 64 NQ bytes of LDS per
//     wave so that lanes store whole dwords and the wave 64 NQ contiguous bytes.
#pragma once

#include "tg_common.hpp"

namespace tg {

// u = (2r + 1) / 2^17 for the 16-bit random field r: the threshold u * s is formed as
// fma(r, 2 * s17, s17) with s17 = s * 2^-17.  (A 24-bit field, one Philox word per element and twice
// the Philox work, was measured: the encoder then becomes ALU-limited on the largest workload,
// 5.41 ms instead of 5.34 - 5.36 ms for 8 x 10^9 elements, one point of HBM fraction.)
constexpr float kFieldScale = 0x1p-17f;

struct TernArgs {
    const float* grads[kMaxWorkers];
    uint8_t* codes[kMaxWorkers];
    const float* tau;           // [W][L]
    const float* s_shared;      // [L]
    const int64_t* off;         // [L+1]
    const uint32_t* tile_info;  // per wave tile: layer of its first element | kTileWhole
    int64_t n;
    int64_t n_wave_tiles;       // wave tiles that cover packed_bytes * 4 elements
    int64_t packed_bytes;       // ceil(n/4) rounded up to 16
    int32_t n_layers;
    uint32_t key0, key1, step, worker_base;
    const uint32_t* step_dev;   // when not null the iteration counter is read from device memory
                                // (so that a captured graph can be replayed with a new step)
};

// 8 code bits of 4 elements.  rf[i]: the 16-bit random field of element i, already a float.
// threshold fl((2r+1) * s17) is formed as fma(r, 2*s17, s17): same real value,
// one rounding.  Both sides of the comparison are non-negative floats, so the
// order of their bit patterns as integers is their order as numbers.
__device__ __forceinline__ uint32_t encode4(const float4 v, const float rf[4],
                                            const float tau, const float s16, const float s17) {
    const float g[4] = {v.x, v.y, v.z, v.w};
    uint32_t acc = 0;
#pragma unroll
    for (int i = 3; i >= 0; --i) {
        const float thr = __builtin_fmaf(rf[i], s16, s17);
        const uint32_t gb = __float_as_uint(g[i]);
        const uint32_t ab = __float_as_uint(min_abs(g[i], tau));           // min(|g|, tau)
        const uint32_t d = __float_as_uint(thr) - ab;                       // bit 31 <=> thr < a
        acc = __builtin_amdgcn_alignbit(acc, d & gb, 31);                   // push "negative"
        acc = __builtin_amdgcn_alignbit(acc, d, 31);                        // push "non-zero"
    }
    return acc;   // code of g[i] at bits 2i..2i+1: 00 / 01 / 11
}

// The same for 4 elements that may lie in different layers: per-element tau and s17.
__device__ __forceinline__ uint32_t encode4v(const float4 v, const float rf[4],
                                             const float tau[4], const float s17[4]) {
    const float g[4] = {v.x, v.y, v.z, v.w};
    uint32_t acc = 0;
#pragma unroll
    for (int i = 3; i >= 0; --i) {
        const float thr = __builtin_fmaf(rf[i], s17[i] * 2.0f, s17[i]);
        const uint32_t gb = __float_as_uint(g[i]);
        const uint32_t ab = __float_as_uint(min_abs(g[i], tau[i]));
        const uint32_t d = __float_as_uint(thr) - ab;
        acc = __builtin_amdgcn_alignbit(acc, d & gb, 31);
        acc = __builtin_amdgcn_alignbit(acc, d, 31);
    }
    return acc;
}

// Code bytes of NQ quarters of one 1024-element tile, starting at quarter NQ * part: b[k] = 2-bit
// codes of the lane's elements 256 (NQ * part + k) + 4*lane .. +3, for worker index w (of this call)
// and tile wt.
template <int NQ = 4>
__device__ __forceinline__ void tile_code_bytes(const TernArgs& p, const int w, const int64_t wt,
                                                const int lane, uint32_t b[NQ], const int part = 0) {
    const int Q0 = NQ * part;          // first quarter of the tile this wave encodes
    const float* __restrict__ g = p.grads[w];
    const uint32_t worker = p.worker_base + (uint32_t)w;
    const int par = lane & 1;
    // read through the constant address space: a scalar load either way.  (A generic load here
    // would be a vector-memory operation ahead of the data loads, and the first use of the step,
    // in the first Philox round, would then wait for the data as well.)
    uint32_t step = p.step;
    if (p.step_dev) step = *reinterpret_cast<const __attribute__((address_space(4))) uint32_t*>((uintptr_t)p.step_dev);
    const int64_t e0 = wt * kWaveTile;

    // the data loads depend on nothing but the tile index: issue them before the
    // (dependent) table lookups so that the two latencies overlap.  The table holds one entry per
    // wave tile (also for the few padding tiles past the end), so the layer, the fast-path flag and
    // with them tau and s are two scalar loads deep, all in flight while the random bits are computed.
    const bool inside = e0 + kWaveTile <= p.n;
    float4 v[NQ];
    if (inside) {
        const float* gp = g + e0 + 256 * Q0 + 4 * lane;
#pragma unroll
        for (int k = 0; k < NQ; ++k) v[k] = load_stream(gp + 256 * k);
    } else {
        // ragged end of the buffer (or past it): missing elements read as 0, which encodes to 00
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const int64_t e = e0 + 256 * (Q0 + k) + 4 * lane;
            float t[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) t[i] = (e + i < p.n) ? g[e + i] : 0.0f;
            v[k] = make_float4(t[0], t[1], t[2], t[3]);
        }
    }

    const uint32_t info = p.tile_info[wt];
    const int l0 = (int)(info & ~kTileWhole);
    const bool whole = (info & kTileWhole) != 0;
    const float* __restrict__ tau_w = p.tau + (int64_t)w * p.n_layers;
    const float tau0 = tau_w[l0];
    const float s0 = p.s_shared[l0];

    // Philox blocks of this tile: q0 .. q0+127; lane computes q0 + 64P + 32*par + (lane>>1)
    float rf[NQ][4];               // random fields of the lane's elements, quarter k, as floats
    const uint64_t q = (uint64_t)(e0 >> 3) + (uint32_t)(32 * Q0 + 32 * par + (lane >> 1));
#pragma unroll
    for (int P = 0; P < NQ / 2; ++P) {
        const uint64_t qq = q + 64 * P;
        const U4 R = philox4x32_10((uint32_t)qq, (uint32_t)(qq >> 32), worker, step, p.key0, p.key1);
        // quarter 2P: elements 8j..8j+7 belong to the even lane's block; the even lane
        // uses its words 0,1, the odd lane the even lane's words 2,3.  Quarter 2P+1:
        // the odd lane's block; the even lane takes its words 0,1, the odd lane keeps 2,3.
        const uint32_t nx = swap_adjacent(R.x), ny = swap_adjacent(R.y);
        const uint32_t nz = swap_adjacent(R.z), nw = swap_adjacent(R.w);
        const uint32_t a0 = par ? nz : R.x, a1 = par ? nw : R.y;     // quarter 2P
        const uint32_t b0 = par ? R.z : nx, b1 = par ? R.w : ny;     // quarter 2P + 1
        // converted here, ahead of the branch on the kind of tile and of the wait for the data
        rf[2 * P][0] = (float)(a0 & 0xFFFFu), rf[2 * P][1] = (float)(a0 >> 16);
        rf[2 * P][2] = (float)(a1 & 0xFFFFu), rf[2 * P][3] = (float)(a1 >> 16);
        rf[2 * P + 1][0] = (float)(b0 & 0xFFFFu), rf[2 * P + 1][1] = (float)(b0 >> 16);
        rf[2 * P + 1][2] = (float)(b1 & 0xFFFFu), rf[2 * P + 1][3] = (float)(b1 >> 16);
    }

    // (a tile entirely past the end needs no special case: its elements read as 0 and its table
    // entry names the last layer, so it encodes to zeros; an early exit here would only keep the
    // table lookups from being scheduled alongside the Philox rounds)
    if (whole) {
        // ---- the tile lies inside layer l0 ----
        const float tau = tau0;
        const float s17 = s0 * kFieldScale;
        const float s16 = s17 * 2.0f;
#pragma unroll
        for (int k = 0; k < NQ; ++k) b[k] = encode4(v[k], rf[k], tau, s16, s17);
    } else {
        // ---- layers change inside the tile.  The layer of an element at tile position x is
        // l0 + #{ j > l0 : off[j] - e0 <= x }: a scalar pass over the (few) boundaries inside the
        // tile per quarter (the table is read through the scalar cache; keeping all 16 positions of
        // the lane live at once would cost the common path registers).
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const int x0 = 256 * (Q0 + k) + 4 * lane;
            int l[4] = {l0, l0, l0, l0};
            for (int j = l0 + 1; j < p.n_layers; ++j) {
                const int64_t rel = p.off[j] - e0;
                if (rel >= kWaveTile) break;
                const int r = (int)rel;
#pragma unroll
                for (int i = 0; i < 4; ++i) l[i] += (x0 + i >= r) ? 1 : 0;
            }
            if (__all(l[0] == l[3])) {
                // no lane's four elements straddle a boundary (buckets that are multiples of four
                // elements): one tau and one s per lane
                const float tau = l[0] == l0 ? tau0 : tau_w[l[0]];
                const float s17 = (l[0] == l0 ? s0 : p.s_shared[l[0]]) * kFieldScale;
                b[k] = encode4(v[k], rf[k], tau, s17 * 2.0f, s17);
            } else {
                float tau[4], s17[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    tau[i] = l[i] == l0 ? tau0 : tau_w[l[i]];
                    s17[i] = (l[i] == l0 ? s0 : p.s_shared[l[i]]) * kFieldScale;
                }
                b[k] = encode4v(v[k], rf[k], tau, s17);
            }
        }
    }
}

// Every XCD encodes runs of 32 consecutive workgroups (64 tiles, 256 KiB of gradient): a 64-byte line of
// the per-tile table then goes into one L2 instead of eight, and the AlexNet- and VGG-A-shaped jobs run
// 2 - 2.5 % faster (0.154 against 0.157 ms, 0.655 against 0.672 ms; 8 x 10^9 elements unchanged).  Runs of 8
// or 64 workgroups are 1 - 2 % slower than no remapping, 128 and 512 help one size and hurt another.
constexpr int kEncoderXcdRun = 32;

template <bool NT_CODES>
__global__ void __launch_bounds__(kBlock) ternarize_pack_kernel(const TernArgs p) {
    __shared__ uint32_t lds[kBlock / kWave][kWave / 2];   // 128 B per wave

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    // half a tile per wave: short-lived waves and a very large grid stream best here, and
    // without a loop every table lookup is a scalar load
    // XCD-aware order (see kEncoderXcdRun)
    const int64_t hw = xcd_run_index(blockIdx.x, kEncoderXcdRun) * (kBlock / kWave) + wave;     // half tile of this wave
    const int64_t wt = hw >> 1;
    const int part = (int)(hw & 1);
    if (wt >= p.n_wave_tiles) return;
    uint32_t b[2];
    tile_code_bytes<2>(p, blockIdx.y, wt, lane, b, part);

    // ---- transpose bytes (position 64k + lane) into dwords (position 4*lane, lanes 0..31) ----
    uint8_t* row = reinterpret_cast<uint8_t*>(lds[wave]);
#pragma unroll
    for (int k = 0; k < 2; ++k) row[64 * k + lane] = (uint8_t)b[k];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint32_t dw = lds[wave][lane & 31];
    const int64_t byte0 = (wt * kWaveTile >> 2) + 128 * part + 4 * lane;
    if (lane < 32 && byte0 < p.packed_bytes) store_through<NT_CODES>(reinterpret_cast<uint32_t*>(p.codes[blockIdx.y] + byte0), dw);
}

// ---- base-3 container: five ternary values per byte (1.6 bits, toward 32/log2(3)) ----
// A workgroup of five waves encodes five tiles = 5120 elements exactly as above, leaves their
// 1280 bytes of 2-bit codes in LDS, and 256 of its threads repack them: thread t turns 20
// consecutive elements (40 bits) into four bytes d0 + 3 d1 + 9 d2 + 27 d3 + 81 d4 with digit
// d = t mod 3 = code - (code >> 1).  1 KiB contiguous per workgroup.

__device__ __forceinline__ uint32_t base3_byte(const uint32_t digits10) {
    // five 2-bit digits (each 0..2) in bits 0..9
    const uint32_t d0 = digits10 & 3u, d1 = (digits10 >> 2) & 3u, d2 = (digits10 >> 4) & 3u;
    const uint32_t d3 = (digits10 >> 6) & 3u, d4 = (digits10 >> 8) & 3u;
    return d0 + 3u * d1 + 9u * d2 + 27u * d3 + 81u * d4;
}

template <bool NT_CODES>
__global__ void __launch_bounds__(kBase3Block) ternarize_pack_base3_kernel(const TernArgs p) {
    __shared__ uint32_t lds[kBase3Waves * kWave];       // 1280 B of 2-bit codes

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int64_t wt = (int64_t)blockIdx.x * kBase3Waves + wave;
    uint32_t b[4];
    tile_code_bytes(p, blockIdx.y, wt, lane, b);
    uint8_t* bytes = reinterpret_cast<uint8_t*>(lds);
#pragma unroll
    for (int k = 0; k < 4; ++k) bytes[256 * wave + 64 * k + lane] = (uint8_t)b[k];
    __syncthreads();

    const int t = threadIdx.x;
    if (t >= 256) return;
    // elements 20t .. 20t+19 of the workgroup = 2-bit bytes 5t .. 5t+4
    uint64_t x = 0;
#pragma unroll
    for (int j = 0; j < 5; ++j) x |= (uint64_t)bytes[5 * t + j] << (8 * j);
    x -= (x >> 1) & 0x5555555555ull;                     // code 00/01/11 -> digit 0/1/2 in every field
    uint32_t out = 0;
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) out |= base3_byte((uint32_t)(x >> (10 * qd)) & 0x3FFu) << (8 * qd);
    const int64_t byte0 = (int64_t)blockIdx.x * 1024 + 4 * t;
    if (byte0 < p.packed_bytes) store_through<NT_CODES>(reinterpret_cast<uint32_t*>(p.codes[blockIdx.y] + byte0), out);
}

}  // namespace tg
