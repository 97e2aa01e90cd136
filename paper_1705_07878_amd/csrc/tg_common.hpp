// Shared device-side pieces of the TernGrad kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tg {

constexpr int kWave = 64;             // CDNA wavefront
constexpr int kBlock = 256;           // 4 waves per workgroup
constexpr int kWaveTile = 1024;       // elements one wave handles per step: 64 lanes x 4 x float4
constexpr uint32_t kTileWhole = 0x80000000u;   // tile_info[]: flag "no layer boundary inside the tile"
constexpr int kMaxWorkers = 64;
// base-3 container (five ternary values per byte): a workgroup of five waves covers five tiles
constexpr int kBase3Waves = 5;
constexpr int kBase3Block = kBase3Waves * kWave;        // 320 threads
constexpr int kBase3Elems = kBase3Waves * kWaveTile;    // 5120 elements <-> 1024 bytes

// Philox4x32 (Salmon et al., SC'11), published multipliers and key increments.
constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

struct U4 {
    uint32_t x, y, z, w;
};

// a ^ b ^ c in one instruction (v_bitop3_b32, truth table 0x96)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// min(|g|, tau) for tau >= 0 in one instruction.  fminf() would first canonicalise both
// operands (two extra instructions); the hardware minimum already returns the right
// value for every non-NaN input, denormals included.
__device__ __forceinline__ float min_abs(float g, float tau) {
    float r;
    asm("v_min_f32 %0, |%1|, %2" : "=v"(r) : "v"(g), "v"(tau));
    return r;
}

// max(m, |x|) in one instruction, same reasoning
__device__ __forceinline__ float max_abs(float m, float x) {
    float r;
    asm("v_max_f32 %0, |%1|, %2" : "=v"(r) : "v"(x), "v"(m));
    return r;
}

// A wave-uniform read of memory that no kernel writes while this one runs (tables, the gradients in
// the statistics pass), through the constant address space: a scalar load, which travels beside the
// vector loads in flight instead of queueing behind them.
template <typename T>
__device__ __forceinline__ T load_uniform(const T* p) {
    return *reinterpret_cast<const __attribute__((address_space(4))) T*>((uintptr_t)p);
}

// Ten rounds over counter (c0,c1,c2,c3) under key (k0,k1).  The key schedule is
// wave-uniform (it depends on the seed alone) and ends up in scalar registers.
__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    return U4{c0, c1, c2, c3};
}

// Streaming (non-temporal) 128-bit load: every input byte of these kernels is read exactly
// once, and the "nt" hint raises the achieved HBM read rate (measured: 6.5 -> 7.2 TB/s).
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float* p) {
    const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}

// Streaming (non-temporal) 128-bit store, one instruction by construction (global_store_dwordx4 nt):
// every output float of the decoders is written exactly once and never re-read by the kernel.
__device__ __forceinline__ void store_stream(float* p, const float4 v) {
    const f32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<f32x4*>(p));
}

// 128-bit store with sc1, and nt on top for outputs too large for the memory-side cache (the rule of the
// code stream below, for the same reasons): what the plain average of float layers writes.  Measured
// against a non-temporal store alone: 6 - 8 % faster on 240 MB of output, equal to 2 % faster on 4 GB.
// The store is written as assembly because no builtin carries the sc1 bit for a 128-bit store.  The
// compiler does not look inside the statement: it cannot know that a store of more than 64 bits needs a
// wait state before a vector instruction may overwrite the registers that hold its data (for the stores
// it emits itself it inserts that wait), so the wait is part of the statement.  (Tried as the policy of
// the decoders' float4 stores as well, where the values are recomputed right after a store - without the
// wait the momentum update then wrote corrupted velocities, caught by its parity test; with it, on 10^9
// elements x 8 workers against the non-temporal builtin: average 0.954 against 0.960 ms, update 1.51
// against 1.54 ms, decoder of 8-bit k fields 0.79 against 0.77 ms, whole step unchanged: not taken.)
template <bool NT>
__device__ __forceinline__ void store_through4(float* p, const float4 v) {
    const f32x4 t = {v.x, v.y, v.z, v.w};
    if (NT) asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" ::"v"(p), "v"(t) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" ::"v"(p), "v"(t) : "memory");
}

// Dword store of the thin code stream that accompanies the gradient read.  Always with the sc1
// cache-policy bit (4 % faster for the encoder than a plain store); with nt on top when the code
// buffers of a launch are too large to stay in the 256 MB memory-side cache.  Measured with 8 workers
// (encoder + the decoder that follows it, ms): 200 MB of codes 0.608 without nt / 0.655 with nt;
// 266 MB (VGG-A shapes) 0.82 / 0.87; 300 MB 0.965 / 0.973; 500 MB 1.64 / 1.62; 2 GB 6.43 / 6.18 - 6.34.
// Small jobs: the decoder finds the codes in the cache.  Large jobs: lines written WITHOUT nt slow down
// whatever kernel runs next (the decoder took 1.04 ms instead of 0.97 ms after 2 GB of plain or sc1
// stores, even with another kernel or an idle gap in between).
constexpr int64_t kCodeStreamNtFrom = (int64_t)288 << 20;     // bytes of codes per launch
template <bool NT>
__device__ __forceinline__ void store_through(uint32_t* p, uint32_t v) {
    if (NT) asm volatile("global_store_dword %0, %1, off sc1 nt" ::"v"(p), "v"(v) : "memory");
    else asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}

// value held by the neighbouring lane (lane ^ 1), via DPP quad_perm [1,0,3,2]
__device__ __forceinline__ uint32_t swap_adjacent(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);
}

// Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by index.  This maps a
// workgroup index to a virtual one such that every XCD works on runs of `run` consecutive virtual
// workgroups; the grid must be a multiple of 8 * run workgroups (indices past the work are skipped by
// the kernels' own bounds checks).
constexpr int kXcds = 8;
__device__ __forceinline__ int64_t xcd_run_index(const int64_t block, const int run) {
    const int64_t xcd = block % kXcds, j = block / kXcds;
    return ((j / run) * kXcds + xcd) * run + j % run;
}

__device__ __forceinline__ int wave_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

}  // namespace tg
