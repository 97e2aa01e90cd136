// Memory-system probes: the access patterns of the TernGrad kernels with the arithmetic taken out.
// They give the ceilings the real kernels are compared with (what this chip sustains for a plain
// streaming read, write, copy, and for a read accompanied by a thin write), on the same launch
// shape: one wave per tile of 1024 floats, four 128-bit accesses per lane.
#pragma once

#include "tg_common.hpp"

namespace tg {

enum { PROBE_READ = 0, PROBE_READ_NT = 1, PROBE_WRITE_NT = 2, PROBE_COPY_NT = 3, PROBE_READ_THIN_WRITE = 4 };

struct ProbeArgs {
    const float* src;     // [n_tiles * 1024]
    float* dst;           // [n_tiles * 1024]: write and copy; read probes touch dst[0] only (see below)
    uint32_t* thin;       // [n_tiles * 64]: one dword per lane, the shape of the 2-bit code stream
    int64_t n_tiles;
};

template <int KIND>
__global__ void __launch_bounds__(kBlock) probe_kernel(const ProbeArgs p) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int64_t wt = (int64_t)blockIdx.x * (kBlock / kWave) + wave;
    if (wt >= p.n_tiles) return;
    const int64_t e = wt * kWaveTile + 4 * lane;
    float4 v[4];
    if (KIND == PROBE_WRITE_NT) {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = make_float4(1.0f, 2.0f, 3.0f, (float)k);
    } else if (KIND == PROBE_READ) {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = *reinterpret_cast<const float4*>(p.src + e + 256 * k);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = load_stream(p.src + e + 256 * k);
    }
    if (KIND == PROBE_WRITE_NT || KIND == PROBE_COPY_NT) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float* d = p.dst + e + 256 * k;
            __builtin_nontemporal_store(v[k].x, d);
            __builtin_nontemporal_store(v[k].y, d + 1);
            __builtin_nontemporal_store(v[k].z, d + 2);
            __builtin_nontemporal_store(v[k].w, d + 3);
        }
        return;
    }
    // the loads must be consumed: fold them into one word
    uint32_t x = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        x ^= __float_as_uint(v[k].x) ^ __float_as_uint(v[k].y) ^ __float_as_uint(v[k].z) ^ __float_as_uint(v[k].w);
    if (KIND == PROBE_READ_THIN_WRITE) {
        store_through(p.thin + wt * kWave + lane, x);        // 256 contiguous bytes per wave, as the code stream
    } else if (x == 0x7FC12345u) {
        p.dst[0] = 1.0f;                                     // practically never: keeps the loads alive
    }
}

}  // namespace tg
