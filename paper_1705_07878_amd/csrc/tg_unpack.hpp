// Fused unpack -> sum over workers -> rescale (Algorithm 1, server line, with
// the shared scaler of Eq. 4).  One wave turns W x 256 bytes of codes into 1024
// fp32 averages per step:
//   * lane L loads one dword (16 codes) of every worker: 256 contiguous bytes
//     per wave and worker;
//   * the ternary values are summed in packed form, never one element at a
//     time: code ^ 0b10 is t + 2 for the two's-complement code t, so one XOR
//     biases all 16 fields of a dword; even and odd fields are spread into 4-bit
//     counters, up to five workers are added per counter, then the counters are
//     widened to bytes.  Byte sums start at 128 - 2W, so a final XOR with 0x80
//     leaves k = sum_w t_w as a signed byte;
//   * the signed bytes (1 B per element) are transposed through LDS so that every
//     lane converts and stores whole float4s; the four waves of a workgroup write each
//     of its four tiles together, 4 KiB contiguous per store step.
#pragma once

#include "tg_common.hpp"

namespace tg {

struct UnpackArgs {
    const uint8_t* codes[kMaxWorkers];
    const float* s_shared;      // [L]
    const float* s_workers;     // [W][L]: every worker's own scaler, for the decoder without scaler sharing
    const int64_t* off;         // [L+1]
    const uint32_t* tile_info;  // per wave tile: layer of its first element | kTileWhole
    float* avg;                 // [n]: the average (out), or the weights (in/out) when updating
    float eta;                  // learning rate of the fused update
    float mu;                   // momentum of the fused update
    float* velocity;            // [n] momentum buffer (in/out), DST_MOMENTUM only
    const uint8_t* ksum_in;     // packed sums k (4- or 8-bit fields), when they are the source
    uint8_t* ksum_out;          // packed sums k, when they are the sink
    int64_t ksum_bytes;         // size of that buffer: ceil(n * bits / 8) rounded up to 16
    int64_t n;
    int64_t n_wave_tiles;       // ceil(n / 1024)
    int64_t packed_bytes;
    int32_t n_layers;
    int32_t n_workers;
};

struct Nib {
    uint32_t even, odd;         // 4-bit counters: nibble j of even/odd = element 2j / 2j+1
};

__device__ __forceinline__ void nib_add(Nib& a, const uint32_t x) {
    const uint32_t y = x ^ 0xAAAAAAAAu;                 // every 2-bit field: t -> t + 2
    a.even += y & 0x33333333u;
    a.odd += (y >> 2) & 0x33333333u;
}

// 8-bit counters, byte m of e_lo / o_lo / e_hi / o_hi = element 4m / 4m+1 / 4m+2 / 4m+3
struct Byt {
    uint32_t e_lo, o_lo, e_hi, o_hi;
};

__device__ __forceinline__ void widen_add(Byt& b, const Nib a) {
    b.e_lo += a.even & 0x0F0F0F0Fu;
    b.e_hi += (a.even >> 4) & 0x0F0F0F0Fu;
    b.o_lo += a.odd & 0x0F0F0F0Fu;
    b.o_hi += (a.odd >> 4) & 0x0F0F0F0Fu;
}

// 4x4 byte transpose: D[m] = bytes of elements 4m, 4m+1, 4m+2, 4m+3
__device__ __forceinline__ void gather_bytes(uint32_t D[4], const Byt b) {
    const uint32_t p01_lo = __builtin_amdgcn_perm(b.o_lo, b.e_lo, 0x05010400u);   // el 0 1 4 5
    const uint32_t p01_hi = __builtin_amdgcn_perm(b.o_lo, b.e_lo, 0x07030602u);   // el 8 9 12 13
    const uint32_t p23_lo = __builtin_amdgcn_perm(b.o_hi, b.e_hi, 0x05010400u);   // el 2 3 6 7
    const uint32_t p23_hi = __builtin_amdgcn_perm(b.o_hi, b.e_hi, 0x07030602u);   // el 10 11 14 15
    D[0] = __builtin_amdgcn_perm(p23_lo, p01_lo, 0x05040100u);
    D[1] = __builtin_amdgcn_perm(p23_lo, p01_lo, 0x07060302u);
    D[2] = __builtin_amdgcn_perm(p23_hi, p01_hi, 0x05040100u);
    D[3] = __builtin_amdgcn_perm(p23_hi, p01_hi, 0x07060302u);
}

// float4 of averages from 4 signed bytes
__device__ __forceinline__ float4 scale4(const uint32_t d, const float sc) {
    const int v = (int)d;
    float4 o;
    o.x = (float)(int)(int8_t)(v) * sc;
    o.y = (float)(int)(int8_t)(v >> 8) * sc;
    o.z = (float)(int)(int8_t)(v >> 16) * sc;
    o.w = (float)(v >> 24) * sc;
    return o;
}

// Cache policy of the float4 stores of the scaling sinks.  Non-temporal is what the library uses: on
// 10^9 elements x 8 workers the decoder takes 0.964 ms with nt, 1.00 ms with sc1 or sc0 sc1, 1.01 - 1.03 ms
// with plain stores; on the AlexNet- and VGG-A-shaped sizes 84 - 85 % of the HBM peak against 73 - 76 %.
// (The codes themselves are read with plain loads: non-temporal ones made the decoder 1 - 5 % slower
// inside the step, where the end of what the encoder just wrote is still cached.)
enum { ST_PLAIN = 0, ST_NT = 1 };

template <int POL>
__device__ __forceinline__ void store4(float* dst, const float4 v) {
    if (POL == ST_NT) store_stream(dst, v);
    else *reinterpret_cast<float4*>(dst) = v;
}

// Which tiles a workgroup owns: consecutive ones from `base` on.  (Spreading them 16 to 1024 tiles apart,
// so that the stores a wave issues one after the other lie far from each other, helps a bare write
// pattern but not the decoders: 0.985 - 1.06 ms against 0.964 ms on 10^9 elements.)
struct TileMap {
    int64_t base;
    __device__ __forceinline__ int64_t at(const int j) const { return base + j; }
};

// w - eta * avg, one rounding
__device__ __forceinline__ float4 apply4(const float4 w, const float4 a, const float eta) {
    return make_float4(__builtin_fmaf(-eta, a.x, w.x), __builtin_fmaf(-eta, a.y, w.y),
                       __builtin_fmaf(-eta, a.z, w.z), __builtin_fmaf(-eta, a.w, w.w));
}

// Where the per-element integer k comes from and where it goes.
//   source  SRC_CODES: k = sum_w t_w, from the W workers' 2-bit code buffers
//           SRC_K4 / SRC_K8: k read from a buffer of 4- / 8-bit two's-complement fields
//           SRC_KB: the same for any width BITS = 2..8 (one little-endian bit stream)
//   sink    DST_AVG:    avg[e] = k * (s/W)               (Algorithm 1, server line)
//           DST_UPDATE: w[e]  -= eta * k * (s/W)          (server line fused with the update line:
//                       the average is never written to or re-read from HBM)
//           DST_MOMENTUM: v[e] = mu * v[e] + k * (s/W) ; w[e] -= eta * v[e]   (momentum SGD,
//                       the optimizer of most of the paper's experiments)
//           DST_K4 / DST_K8: k itself in 4- / 8-bit fields (the server-to-worker pull of
//                       Section 3.1: at most 2N+1 levels instead of 32-bit floats)
//           DST_KB: the same for any width BITS = 2..8; ceil(log2(2N+1)) bits hold the 2N+1 levels
enum { SRC_CODES = 0, SRC_K4 = 1, SRC_K8 = 2, SRC_KB = 3 };
enum { DST_AVG = 0, DST_UPDATE = 1, DST_K4 = 2, DST_K8 = 3, DST_MOMENTUM = 4, DST_KB = 5 };

// 16 signed bytes (D[m] = elements 4m .. 4m+3) <-> 16 fields of BITS bits, field i at bit i * BITS
// of a 128-bit little-endian value (lo, hi)
template <int BITS>
__device__ __forceinline__ void fields_from_bytes(const uint32_t D[4], uint64_t& lo, uint64_t& hi) {
    constexpr uint64_t mask = (1ull << BITS) - 1;
    lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint64_t f = (uint64_t)(D[i >> 2] >> (8 * (i & 3))) & mask;
        const int pos = i * BITS;
        if (pos < 64) {
            lo |= f << pos;
            if (pos + BITS > 64) hi |= f >> (64 - pos);
        } else {
            hi |= f << (pos - 64);
        }
    }
}

template <int BITS>
__device__ __forceinline__ void bytes_from_fields(const uint64_t lo, const uint64_t hi, uint32_t D[4]) {
    constexpr uint32_t mask = (1u << BITS) - 1, sign = 1u << (BITS - 1);
    D[0] = D[1] = D[2] = D[3] = 0u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int pos = i * BITS;
        uint64_t f;
        if (pos >= 64) f = hi >> (pos - 64);
        else if (pos + BITS > 64) f = (lo >> pos) | (hi << (64 - pos));
        else f = lo >> pos;
        const uint32_t k = (((uint32_t)f & mask) ^ sign) - sign;         // sign extension from BITS bits
        D[i >> 2] |= (k & 0xFFu) << (8 * (i & 3));
    }
}

// sign-extend the low nibble of every byte: bit 3 set -> bits 4..7 set (0x08 * 30 = 0xF0)
__device__ __forceinline__ uint32_t sext_nibbles(const uint32_t y) {
    return y | ((y & 0x08080808u) * 30u);
}

// low nibbles of the 8 bytes of (d0, d1) -> 8 consecutive 4-bit fields
__device__ __forceinline__ uint32_t pack_nibbles(const uint32_t d0, const uint32_t d1) {
    const uint32_t y0 = d0 & 0x0F0F0F0Fu, y1 = d1 & 0x0F0F0F0Fu;
    const uint32_t t0 = y0 | (y0 >> 4), t1 = y1 | (y1 >> 4);     // bytes 0 and 2 hold two fields each
    return __builtin_amdgcn_perm(t1, t0, 0x06040200u);
}

constexpr int kTilesPerBlock = kBlock / kWave;   // 4 tiles of 1024 elements per workgroup

// the sum k of one tile's codes over the workers: D[m] = k of the lane's elements
// 16*lane + 4m .. 4m+3, one signed byte each; x(w) yields the lane's code dword of worker w
template <class LoadCodes>
__device__ __forceinline__ void sum_codes(const int W, uint32_t D[4], LoadCodes x) {
    const uint32_t bias = (uint32_t)(128 - 2 * W) * 0x01010101u;
    Byt acc = {bias, bias, bias, bias};
    for (int w0 = 0; w0 < W; w0 += 5) {
        // up to five workers per 4-bit counter: 5 * 3 = 15
        // all five loads are issued unconditionally (a clamped worker index keeps them valid) so that
        // they are in flight together; an absent worker's value is then replaced by t + 2 = 0.
        // (Requesting the next group before this one is summed was measured: no gain at W = 4,
        // 2 % slower at W = 8 on 10^9 elements.)
        uint32_t c[5];
#pragma unroll
        for (int j = 0; j < 5; ++j) c[j] = x(w0 + j < W ? w0 + j : W - 1);
#pragma unroll
        for (int j = 0; j < 5; ++j) c[j] = (w0 + j < W) ? c[j] : 0xAAAAAAAAu;
        Nib a = {0u, 0u};
#pragma unroll
        for (int j = 0; j < 5; ++j) nib_add(a, c[j]);
        widen_add(acc, a);
    }
    // counters hold 128 + k: flip bit 7 to get k as int8
    acc.e_lo ^= 0x80808080u; acc.o_lo ^= 0x80808080u; acc.e_hi ^= 0x80808080u; acc.o_hi ^= 0x80808080u;
    gather_bytes(D, acc);
}

// Scaling sinks, workgroup-cooperative: kb[t] holds the signed bytes of tile tile0 + t in element
// order (256 dwords); the NWAVES waves write the NTILES tiles quarter by quarter, wave j the
// quarters j, j + NWAVES, ..., so that every store step of the workgroup covers NWAVES KiB
// contiguous.  Measured 6 - 10 % faster than each wave storing its own tile.
template <int POL, int DST, int NWAVES, int NTILES>
struct Emit {
    static constexpr int kSteps = 4 * NTILES / NWAVES;
    static constexpr bool MOMENTUM = DST == DST_MOMENTUM;
    static constexpr bool UPDATE = DST == DST_UPDATE || MOMENTUM;
    float4 wv[kSteps], vv[MOMENTUM ? kSteps : 1];
    int l0s[kSteps];       // first layer of the tile written in step i
    float scs[kSteps];     // its scale s/W ...
    bool fast[kSteps];     // ... valid when the whole tile lies in that layer and inside the buffer

    // Everything that depends on nothing but the tile indices is fetched first, before the codes are
    // summed and long before the barrier: the weights (and velocities), and the layer and scale of the
    // tiles this wave will write.
    __device__ __forceinline__ void prefetch(const UnpackArgs& p, const TileMap tm, const int wave, const int lane) {
        const float fW = (float)p.n_workers;
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const int q = wave + i * NWAVES;
            const int64_t tile = tm.at(q >> 2);
            const int64_t te0 = tile * kWaveTile;
            if (UPDATE) {
                const int64_t e = te0 + 256 * (q & 3) + 4 * lane;
                if (e + 3 < p.n) {
                    wv[i] = load_stream(p.avg + e);
                    if (MOMENTUM) vv[i] = load_stream(p.velocity + e);
                }
            }
            l0s[i] = 0;
            scs[i] = 0.0f;
            fast[i] = false;
            if (tile < p.n_wave_tiles) {
                const uint32_t info = p.tile_info[tile];
                const int l0 = (int)(info & ~kTileWhole);
                const bool one_layer = (info & kTileWhole) != 0;
                l0s[i] = l0;
                if (one_layer && te0 + kWaveTile <= p.n) {
                    fast[i] = true;
                    scs[i] = p.s_shared[l0] / fW;
                }
            }
        }
    }

    // the four elements at e (all inside the buffer) from their signed bytes d and one scale
    __device__ __forceinline__ void emit4(const UnpackArgs& p, const int i, const int64_t e, const uint32_t d,
                                          const float sc) const {
        float4 o = scale4(d, sc);
        if (MOMENTUM) {
            const float4 v = vv[i];
            o = make_float4(__builtin_fmaf(p.mu, v.x, o.x), __builtin_fmaf(p.mu, v.y, o.y),
                            __builtin_fmaf(p.mu, v.z, o.z), __builtin_fmaf(p.mu, v.w, o.w));
            store4<POL>(p.velocity + e, o);
        }
        if (UPDATE) o = apply4(wv[i], o, p.eta);
        store4<POL>(p.avg + e, o);
    }

    // sums(t, i): dword i (the signed bytes of elements 4i .. 4i+3) of the workgroup's t-th tile
    template <class Sums>
    __device__ __forceinline__ void store(const UnpackArgs& p, Sums sums,
                                          const TileMap tm, const int wave, const int lane) const {
        const float fW = (float)p.n_workers;
#pragma unroll
        for (int i = 0; i < kSteps; ++i) {
            const int q = wave + i * NWAVES;
            const int t = q >> 2;
            const int64_t tile = tm.at(t);
            if (tile >= p.n_wave_tiles) continue;
            const int xq = 256 * (q & 3) + 4 * lane;           // position inside the tile
            const int64_t te0 = tile * kWaveTile;
            const int64_t e = te0 + xq;
            const uint32_t d = sums(t, 64 * (q & 3) + lane);
            const int l0 = l0s[i];
            if (fast[i]) {
                emit4(p, i, e, d, scs[i]);
            } else {
                // layers change inside the tile, or the tile is ragged: the layer of the element at
                // tile position x is l0 + #{ j > l0 : off[j] - te0 <= x } (one scalar pass over the
                // boundaries inside the tile)
                int l[4] = {l0, l0, l0, l0};
                for (int j = l0 + 1; j < p.n_layers; ++j) {
                    const int64_t rel = p.off[j] - te0;
                    if (rel >= kWaveTile) break;
                    const int r = (int)rel;
#pragma unroll
                    for (int k = 0; k < 4; ++k) l[k] += (xq + k >= r) ? 1 : 0;
                }
                if (__all(l[0] == l[3] && e + 3 < p.n)) {
                    // no lane's four elements straddle a boundary or the end (buckets that are
                    // multiples of four elements): one scale per lane
                    emit4(p, i, e, d, p.s_shared[l[0]] / fW);
                    continue;
                }
                // one scale per element
                const int di = (int)d;
                const int kk[4] = {(int)(int8_t)di, (int)(int8_t)(di >> 8), (int)(int8_t)(di >> 16), di >> 24};
                float o[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    o[k] = (float)kk[k] * (p.s_shared[l[k]] / fW);
                    if (MOMENTUM && e + k < p.n) {
                        o[k] = __builtin_fmaf(p.mu, p.velocity[e + k], o[k]);
                        p.velocity[e + k] = o[k];
                    }
                    if (UPDATE && e + k < p.n) o[k] = __builtin_fmaf(-p.eta, o[k], p.avg[e + k]);
                }
                if (e + 3 < p.n) {
                    store4<POL>(p.avg + e, make_float4(o[0], o[1], o[2], o[3]));
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (e + k < p.n) p.avg[e + k] = o[k];
                }
            }
        }
    }
};

// A workgroup owns 4 consecutive tiles.  Wave j sums the codes of its j-th tile (one short-lived pass,
// every table lookup a scalar load); the scaling sinks then write the tiles together (see Emit).
template <int POL, int SRC, int DST, int BITS = 0>
__global__ void __launch_bounds__(kBlock) unpack_average_kernel(const UnpackArgs p) {
    __shared__ uint32_t lds[kTilesPerBlock][kWaveTile / 4];   // 1 KiB per tile

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    const TileMap tm = {(int64_t)blockIdx.x * kTilesPerBlock};
    const int64_t wt = tm.at(wave);
    const bool valid = wt < p.n_wave_tiles;
    const int64_t e0 = wt * kWaveTile;

    Emit<POL, DST, kTilesPerBlock, kTilesPerBlock> emit;
    if (DST != DST_K4 && DST != DST_K8 && DST != DST_KB) emit.prefetch(p, tm, wave, lane);

    uint32_t D[4] = {0u, 0u, 0u, 0u};
    if (valid) {
        if (SRC == SRC_CODES) {
            const int64_t byte0 = (e0 >> 2) + 4 * lane;
            if (byte0 < p.packed_bytes)                    // false only in the ragged last tile
                sum_codes(p.n_workers, D, [&](int w) { return *reinterpret_cast<const uint32_t*>(p.codes[w] + byte0); });
        } else if (SRC == SRC_KB) {
            // the lane's 16 fields are the 2 * BITS bytes at byte 2 * BITS * lane of the tile's stream
            const int64_t byte0 = wt * (kWaveTile / 8 * BITS) + 2 * BITS * lane;
            uint64_t lo = 0, hi = 0;
#pragma unroll
            for (int j = 0; j < BITS; ++j) {
                const int64_t b = byte0 + 2 * j;
                const uint64_t h = b < p.ksum_bytes ? *reinterpret_cast<const uint16_t*>(p.ksum_in + b) : 0;
                if (j < 4) lo |= h << (16 * j);
                else hi |= h << (16 * (j - 4));
            }
            bytes_from_fields<BITS == 0 ? 1 : BITS>(lo, hi, D);
        } else if (SRC == SRC_K8) {
            const int64_t byte0 = e0 + 16 * lane;
            uint4 q = make_uint4(0u, 0u, 0u, 0u);
            if (byte0 < p.ksum_bytes) q = *reinterpret_cast<const uint4*>(p.ksum_in + byte0);
            D[0] = q.x, D[1] = q.y, D[2] = q.z, D[3] = q.w;
        } else {
            const int64_t byte0 = (e0 >> 1) + 8 * lane;
            uint2 q = make_uint2(0u, 0u);
            if (byte0 < p.ksum_bytes) q = *reinterpret_cast<const uint2*>(p.ksum_in + byte0);
            // nibble j of q.x / q.y = element j / 8 + j
            const uint32_t lo0 = q.x & 0x0F0F0F0Fu, hi0 = (q.x >> 4) & 0x0F0F0F0Fu;
            const uint32_t lo1 = q.y & 0x0F0F0F0Fu, hi1 = (q.y >> 4) & 0x0F0F0F0Fu;
            D[0] = sext_nibbles(__builtin_amdgcn_perm(hi0, lo0, 0x05010400u));
            D[1] = sext_nibbles(__builtin_amdgcn_perm(hi0, lo0, 0x07030602u));
            D[2] = sext_nibbles(__builtin_amdgcn_perm(hi1, lo1, 0x05010400u));
            D[3] = sext_nibbles(__builtin_amdgcn_perm(hi1, lo1, 0x07030602u));
        }
    }

    // ---- sinks that keep k: the lane's 16 fields are already consecutive in memory ----
    if (DST == DST_K8) {
        const int64_t byte0 = e0 + 16 * lane;
        if (valid && byte0 < p.ksum_bytes)
            *reinterpret_cast<uint4*>(p.ksum_out + byte0) = make_uint4(D[0], D[1], D[2], D[3]);
        return;
    }
    if (DST == DST_K4) {
        const int64_t byte0 = (e0 >> 1) + 8 * lane;
        if (valid && byte0 < p.ksum_bytes)
            *reinterpret_cast<uint2*>(p.ksum_out + byte0) = make_uint2(pack_nibbles(D[0], D[1]), pack_nibbles(D[2], D[3]));
        return;
    }

    if (DST == DST_KB) {
        // the lane's 2 * BITS bytes go to LDS as halfwords; the wave then stores the tile's 128 * BITS
        // bytes as whole dwords, contiguously
        if (!valid) return;
        uint64_t lo, hi;
        fields_from_bytes<BITS == 0 ? 1 : BITS>(D, lo, hi);
        uint16_t* row = reinterpret_cast<uint16_t*>(lds[wave]);
#pragma unroll
        for (int j = 0; j < BITS; ++j)
            row[BITS * lane + j] = (uint16_t)(j < 4 ? lo >> (16 * j) : hi >> (16 * (j - 4)));
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int64_t tile_byte0 = wt * (kWaveTile / 8 * BITS);
#pragma unroll
        for (int r = 0; r < (32 * BITS + kWave - 1) / kWave; ++r) {
            const int idx = lane + kWave * r;
            const int64_t b = tile_byte0 + 4 * idx;
            if (idx < 32 * BITS && b < p.ksum_bytes) *reinterpret_cast<uint32_t*>(p.ksum_out + b) = lds[wave][idx];
        }
        return;
    }

    // ---- sinks that scale: the bytes go through LDS (a 64 x 16 -> 256 x 4 transpose per tile) ----
    *reinterpret_cast<uint4*>(&lds[wave][4 * lane]) = make_uint4(D[0], D[1], D[2], D[3]);
    __syncthreads();
    emit.store(p, [&](int t, int i) { return lds[t][i]; }, tm, wave, lane);
}

// The sinks that also READ n floats (fused update, with or without momentum) are copies with a little
// arithmetic, and a copy streams best on this chip when every wave makes ONE 1 KiB access per stream
// and ends (measured on 4 GiB: 84 % of the HBM peak against 76 % with four accesses per wave, 78 % with two).  So here
// a wave owns a quarter tile: lane L the elements 4L .. 4L+3, one code BYTE per worker (a wave reads 64
// contiguous bytes per worker), summed in byte counters; no LDS, no barrier.  Flat 10^9 elements, 8
// workers: update 1.53 ms against 1.66 ms through the kernel above, with momentum 2.97 against 3.17 ms
// (a wave per half tile: 1.61 and 3.19 ms).  The code reads are four times as many instructions as
// in the kernel above, which is why the plain average (nothing but codes read) stays there: 1.42 ms
// this way against 0.98 ms.
template <int POL, int DST>
__global__ void __launch_bounds__(kBlock) unpack_quarter_kernel(const UnpackArgs p) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int64_t gq = (int64_t)blockIdx.x * (kBlock / kWave) + wave;      // quarter tile of this wave
    const int64_t tile = gq >> 2;
    const int qd = (int)(gq & 3);
    if (tile >= p.n_wave_tiles) return;
    const TileMap tm = {tile};
    Emit<POL, DST, 4, 1> emit;                  // one step: quarter qd of the tile
    emit.prefetch(p, tm, qd, lane);

    const int W = p.n_workers;
    const int64_t byte = (tile * kWaveTile >> 2) + 64 * qd + lane;
    const bool in_codes = byte < p.packed_bytes;           // false only in the ragged last tile
    uint32_t acc = (uint32_t)(128 - 2 * W) * 0x01010101u;
    for (int w0 = 0; w0 < W; w0 += 8) {
        // eight workers' bytes in flight (a clamped index keeps those of a short last group valid)
        uint32_t c[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) c[j] = p.codes[w0 + j < W ? w0 + j : W - 1][in_codes ? byte : 0];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // t + 2 of the byte's four fields (codes past the end of the buffer read as 00), each spread
            // into a byte of its own; an absent worker adds nothing
            uint32_t y = (in_codes ? c[j] : 0u) ^ 0xAAu;
            y = (y | (y << 6) | (y << 12) | (y << 18)) & 0x03030303u;
            acc += (w0 + j < W) ? y : 0u;
        }
    }
    const uint32_t d = acc ^ 0x80808080u;                  // counters hold 128 + k
    emit.store(p, [&](int, int) { return d; }, tm, qd, lane);
}

// ---- base-3 container (five ternary values per byte) as the source ----
// A workgroup of five waves owns five tiles = 5120 elements = 1024 bytes per worker.  Thread t of
// its first 256 threads owns the elements 20t .. 20t+19: it loads one dword (four bytes) per
// worker, translates every byte into five 2-bit codes through a 256-entry table in LDS (40 bits
// per dword) and sums them in the same packed counters as above, 16 + 4 elements.  The 20 signed
// bytes go to LDS in element order and the tiles are written cooperatively.
constexpr int kBase3Chunk = 5;   // workers per 4-bit counter

template <int POL, int DST>
__global__ void __launch_bounds__(kBase3Block) unpack_average_base3_kernel(const UnpackArgs p) {
    __shared__ uint16_t lut[256];
    __shared__ uint32_t kb[kBase3Waves][kWaveTile / 4];

    const int t = threadIdx.x;
    const int lane = t & (kWave - 1);
    const int wave = wave_uniform(t >> 6);
    const int W = p.n_workers;
    const int64_t tile0 = (int64_t)blockIdx.x * kBase3Waves;

    const TileMap tm = {tile0};
    Emit<POL, DST, kBase3Waves, kBase3Waves> emit;
    emit.prefetch(p, tm, wave, lane);

    // this thread's dword of every worker (threads 256..319 only take part in the stores)
    const int64_t byte0 = (int64_t)blockIdx.x * 1024 + 4 * (t & 255);
    const bool in_codes = byte0 < p.packed_bytes;
    auto load_chunk = [&](const int w0, uint32_t xs[kBase3Chunk]) {
#pragma unroll
        for (int j = 0; j < kBase3Chunk; ++j)          // unconditional, clamped: all loads in flight together
            xs[j] = *reinterpret_cast<const uint32_t*>(p.codes[w0 + j < W ? w0 + j : W - 1] + (in_codes ? byte0 : 0));
    };
    // the first workers' codes are requested before the table is built
    uint32_t xs[kBase3Chunk] = {};
    if (t < 256) load_chunk(0, xs);

    if (t < 256) {
        // digits of the byte (mod 243), digit 0 / 1 / 2 -> code 00 / 01 / 11
        uint32_t v = (uint32_t)t % 243u, c = 0;
#pragma unroll
        for (int m = 0; m < 5; ++m) {
            const uint32_t d = v % 3u;
            v /= 3u;
            c |= (d + (d >> 1)) << (2 * m);
        }
        lut[t] = (uint16_t)c;
    }
    __syncthreads();

    if (t < 256) {
        const uint32_t bias = (uint32_t)(128 - 2 * W) * 0x01010101u;
        Byt acc_lo = {bias, bias, bias, bias}, acc_hi = {bias, bias, bias, bias};
        for (int w0 = 0; w0 < W; w0 += kBase3Chunk) {
            uint32_t nx[kBase3Chunk] = {};
            if (w0 + kBase3Chunk < W) load_chunk(w0 + kBase3Chunk, nx);      // next chunk, while this one is decoded
            Nib a_lo = {0u, 0u}, a_hi = {0u, 0u};
#pragma unroll
            for (int j = 0; j < kBase3Chunk; ++j) {
                uint32_t lo = 0xAAAAAAAAu, hi = 0xAAAAAAAAu;           // an absent worker adds t + 2 = 0
                if (w0 + j < W) {
                    const uint32_t x = in_codes ? xs[j] : 0u;
                    const uint64_t c = (uint64_t)lut[x & 0xFFu] | ((uint64_t)lut[(x >> 8) & 0xFFu] << 10) |
                                       ((uint64_t)lut[(x >> 16) & 0xFFu] << 20) | ((uint64_t)lut[x >> 24] << 30);
                    lo = (uint32_t)c;                                   // codes of elements 0..15
                    hi = (uint32_t)(c >> 32) | 0xAAAAAA00u;            // codes of elements 16..19, rest neutral
                }
                nib_add(a_lo, lo);
                nib_add(a_hi, hi);
            }
            widen_add(acc_lo, a_lo);
            widen_add(acc_hi, a_hi);
#pragma unroll
            for (int j = 0; j < kBase3Chunk; ++j) xs[j] = nx[j];
        }
        acc_lo.e_lo ^= 0x80808080u; acc_lo.o_lo ^= 0x80808080u; acc_lo.e_hi ^= 0x80808080u; acc_lo.o_hi ^= 0x80808080u;
        acc_hi.e_lo ^= 0x80808080u; acc_hi.o_lo ^= 0x80808080u; acc_hi.e_hi ^= 0x80808080u; acc_hi.o_hi ^= 0x80808080u;
        uint32_t D[4], H[4];
        gather_bytes(D, acc_lo);
        gather_bytes(H, acc_hi);                                        // H[0] = elements 16..19
        uint32_t* dst = &kb[0][0] + 5 * t;                              // 20 bytes, element order
        dst[0] = D[0], dst[1] = D[1], dst[2] = D[2], dst[3] = D[3], dst[4] = H[0];
    }
    __syncthreads();
    emit.store(p, [&](int t, int i) { return kb[t][i]; }, tm, wave, lane);
}

// ---- the server line of Algorithm 1 without scaler sharing: avg = (1/N) sum_i s^(i) t_i ----
// The packed counters above need one scale per layer; with a scaler per worker the sum is taken per
// element in fp64 (each s * t is exact, the additions are in worker order), which makes this
// variant about as ALU- as memory-bound.  One wave per tile; lane L owns the 16 consecutive elements
// of its code dword, and the 16 results go through LDS so that the wave stores whole float4s,
// 1 KiB contiguous per store.
template <int POL>
__global__ void __launch_bounds__(kBlock) unpack_average_scalers_kernel(const UnpackArgs p) {
    __shared__ float lds[kTilesPerBlock][kWaveTile];     // 4 KiB per tile

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int64_t wt = (int64_t)blockIdx.x * kTilesPerBlock + wave;
    if (wt >= p.n_wave_tiles) return;
    const int64_t e0 = wt * kWaveTile;
    const int W = p.n_workers;
    const uint32_t info = p.tile_info[wt];
    const int l0 = (int)(info & ~kTileWhole);
    const bool whole = (info & kTileWhole) != 0;
    const int64_t byte0 = (e0 >> 2) + 4 * lane;
    const bool in_codes = byte0 < p.packed_bytes;          // false only in the ragged last tile
    const int64_t cbyte = in_codes ? byte0 : 0;

    double acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.0;

    if (whole) {
        for (int w0 = 0; w0 < W; w0 += 4) {
            // four workers' loads in flight; a clamped index keeps those of a short last group valid
            uint32_t x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
                x[j] = *reinterpret_cast<const uint32_t*>(p.codes[w0 + j < W ? w0 + j : W - 1] + cbyte);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (w0 + j >= W) break;
                const double sd = (double)p.s_workers[(int64_t)(w0 + j) * p.n_layers + l0];
                const int xi = in_codes ? (int)x[j] : 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int t = (int)((uint32_t)xi << (30 - 2 * i)) >> 30;  // 2-bit two's complement
                    acc[i] = __builtin_fma((double)t, sd, acc[i]);
                }
            }
        }
    } else {
        // layers change inside the tile: the layer of each of the lane's elements from one scalar pass
        // over the boundaries, then one scaler per element and worker
        int l[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) l[i] = l0;
        for (int j = l0 + 1; j < p.n_layers; ++j) {
            const int64_t rel = p.off[j] - e0;
            if (rel >= kWaveTile) break;
            const int r = (int)rel;
#pragma unroll
            for (int i = 0; i < 16; ++i) l[i] += (16 * lane + i >= r) ? 1 : 0;
        }
        for (int w = 0; w < W; ++w) {
            const int xi = in_codes ? (int)*reinterpret_cast<const uint32_t*>(p.codes[w] + cbyte) : 0;
            const float* __restrict__ sw = p.s_workers + (int64_t)w * p.n_layers;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int t = (int)((uint32_t)xi << (30 - 2 * i)) >> 30;
                acc[i] = __builtin_fma((double)t, (double)sw[l[i]], acc[i]);
            }
        }
    }

    // one rounding to fp32; the mean is taken as a product with 1/N in fp64
    const double inv = 1.0 / (double)W;
    float* row = lds[wave];
#pragma unroll
    for (int m = 0; m < 4; ++m)
        *reinterpret_cast<float4*>(row + 16 * lane + 4 * m) =
            make_float4((float)(acc[4 * m] * inv), (float)(acc[4 * m + 1] * inv),
                        (float)(acc[4 * m + 2] * inv), (float)(acc[4 * m + 3] * inv));
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int x = 4 * (lane + kWave * r);
        const float4 v = *reinterpret_cast<const float4*>(row + x);
        const int64_t e = e0 + x;
        if (e + 3 < p.n) {
            store4<POL>(p.avg + e, v);
        } else {
            const float o[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (e + k < p.n) p.avg[e + k] = o[k];
        }
    }
}

}  // namespace tg
