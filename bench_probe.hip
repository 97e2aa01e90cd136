// libbench_probe.so -- a measurement instrument of bench.py, no part of the TernGrad library.
// Memory-system probes: the access patterns of the TernGrad kernels with the arithmetic taken out,
// on the same launch shape (one wave per tile of 1024 floats, four 128-bit accesses per lane) and
// through the same load / store helpers as the kernels.  They give the ceilings the real kernels are
// compared with: what this chip sustains for a plain streaming read, write, copy, and for a read
// accompanied by a thin write.
//
//   int bench_probe(int kind, const float* src, float* dst, uint32_t* thin, int64_t n, void* stream)
//     kind  0 plain streaming read of src; 1 the same with non-temporal loads; 2 non-temporal write
//           of dst; 3 copy src -> dst (non-temporal both ways); 4 non-temporal read of src with one
//           dword written per 16 floats read (to thin): the traffic shape of tg_ternarize_pack, with the
//           encoder's cache policy for a code stream of that size;
//           5 the decoder's write pattern: workgroups of four waves own four tiles and write each
//           tile together, a wave's four stores 4 KiB apart (non-temporal)
//     src   dev [n] fp32 (kinds 0, 1, 3, 4), dst dev [n] fp32 (written by kinds 2, 3, 5; kinds 0, 1, 4
//           may write dst[0]), thin dev [n/16] uint32 (kind 4); n a multiple of 4096; 16-byte aligned
//     returns 0, or -1 (bad argument), -2 (alignment), -4 (launch failed)
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "paper_1705_07878_amd/csrc/tg_common.hpp"

namespace {

using namespace tg;

enum { PROBE_READ = 0, PROBE_READ_NT = 1, PROBE_WRITE_NT = 2, PROBE_COPY_NT = 3, PROBE_READ_THIN_WRITE = 4,
       PROBE_WRITE_NT_COOP = 5 };

struct ProbeArgs {
    const float* src;     // [n_tiles * 1024]
    float* dst;           // [n_tiles * 1024]: write and copy; read probes touch dst[0] only (see below)
    uint32_t* thin;       // [n_tiles * 64]: one dword per lane, the shape of the 2-bit code stream
    int64_t n_tiles;
};

template <int KIND, bool NT_THIN = false>
__global__ void __launch_bounds__(kBlock) probe_kernel(const ProbeArgs p) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = wave_uniform(threadIdx.x >> 6);
    const int64_t wt = (int64_t)blockIdx.x * (kBlock / kWave) + wave;
    if (wt >= p.n_tiles) return;
    const int64_t e = wt * kWaveTile + 4 * lane;
    float4 v[4];
    if (KIND == PROBE_WRITE_NT || KIND == PROBE_WRITE_NT_COOP) {
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
        for (int k = 0; k < 4; ++k) store_stream(p.dst + e + 256 * k, v[k]);
        return;
    }
    if (KIND == PROBE_WRITE_NT_COOP) {
        // wave j of the workgroup writes quarter j of each of the workgroup's four tiles
        // (n_tiles is a multiple of four, so all four tiles exist)
        const int64_t tile0 = (int64_t)blockIdx.x * (kBlock / kWave);
#pragma unroll
        for (int k = 0; k < 4; ++k) store_stream(p.dst + (tile0 + k) * kWaveTile + 256 * wave + 4 * lane, v[k]);
        return;
    }
    // the loads must be consumed: fold them into one word
    uint32_t x = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        x ^= __float_as_uint(v[k].x) ^ __float_as_uint(v[k].y) ^ __float_as_uint(v[k].z) ^ __float_as_uint(v[k].w);
    if (KIND == PROBE_READ_THIN_WRITE) {
        store_through<NT_THIN>(p.thin + wt * kWave + lane, x);     // 256 contiguous bytes per wave, as the code stream
    } else if (x == 0x7FC12345u) {
        p.dst[0] = 1.0f;                                     // practically never: keeps the loads alive
    }
}

bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

extern "C" int bench_probe(int kind, const float* src, float* dst, uint32_t* thin, int64_t n, void* stream) {
    constexpr int64_t kGroup = (int64_t)kWaveTile * (kBlock / kWave);      // 4096 floats per workgroup
    if (kind < PROBE_READ || kind > PROBE_WRITE_NT_COOP || n < kGroup || n % kGroup != 0) return -1;
    const bool reads = kind != PROBE_WRITE_NT && kind != PROBE_WRITE_NT_COOP;
    if ((reads && src == nullptr) || dst == nullptr || (kind == PROBE_READ_THIN_WRITE && thin == nullptr)) return -1;
    if ((reads && !aligned(src, 16)) || !aligned(dst, 16) || (thin != nullptr && !aligned(thin, 4))) return -2;
    const ProbeArgs a{src, dst, thin, n / kWaveTile};
    const int64_t blocks = a.n_tiles / (kBlock / kWave);
    if (blocks > 0x7FFFFFFF) return -1;
    const dim3 grid((unsigned)blocks), block(kBlock);
    hipStream_t s = (hipStream_t)stream;
    switch (kind) {
        case PROBE_READ: hipLaunchKernelGGL(probe_kernel<PROBE_READ>, grid, block, 0, s, a); break;
        case PROBE_READ_NT: hipLaunchKernelGGL(probe_kernel<PROBE_READ_NT>, grid, block, 0, s, a); break;
        case PROBE_WRITE_NT: hipLaunchKernelGGL(probe_kernel<PROBE_WRITE_NT>, grid, block, 0, s, a); break;
        case PROBE_COPY_NT: hipLaunchKernelGGL(probe_kernel<PROBE_COPY_NT>, grid, block, 0, s, a); break;
        case PROBE_READ_THIN_WRITE:
            // cache policy of the thin stream by its size, as the encoder chooses it
            if (n / 4 > kCodeStreamNtFrom) hipLaunchKernelGGL((probe_kernel<PROBE_READ_THIN_WRITE, true>), grid, block, 0, s, a);
            else hipLaunchKernelGGL((probe_kernel<PROBE_READ_THIN_WRITE, false>), grid, block, 0, s, a);
            break;
        default: hipLaunchKernelGGL(probe_kernel<PROBE_WRITE_NT_COOP>, grid, block, 0, s, a); break;
    }
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
