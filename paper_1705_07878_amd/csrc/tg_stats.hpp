// Per-layer clip threshold and scaler (Eq. 5 and Eq. 2) in one read of g.
//
// max|clip(g)| = min(max|g|, c*sigma), so sigma and the scaler come out of the
// same pass.  Sums are fp64 and taken about a per-layer pivot K = first element
// of the layer (shifted-data variance: exact for a constant layer, insensitive to
// a large mean).  No float atomics: every statistics chunk (8192 to 65536 elements, by the size of
// the job) is cut into segments, one per layer it touches; a workgroup reduces one large segment (or
// four small ones, a wave each) in a fixed tree and writes one partial per segment; a second small
// kernel folds the partials of each layer in a fixed order.  Results are bit-identical from run to
// run.  Large jobs take a second shape of the first kernel (clip_stats_wide_kernel).
#pragma once

#include "tg_common.hpp"

namespace tg {

// Two shapes of the statistics pass, by the total work of a call (elements of all workers):
//   * workgroups of 256 threads that loop over a chunk of 8192 to 65536 elements (larger chunks amortise
//     the per-workgroup cost, smaller ones keep enough workgroups in flight; measured best: 8192 for 25 M
//     elements, 16384 - 32768 for 244 M, 65536 from 1 G on);
//   * from kStatWideFrom elements on: workgroups of 1024 threads that read a chunk of 16384 elements in
//     one shot (four 128-bit loads per thread, no loop), mapped to the chunks so that every XCD reads runs
//     of kStatXcdRun consecutive chunks (1 MiB).  The bare pattern reads 8 x 10^9 elements at 92 % of the
//     8 TB/s peak where the loop over 65536 elements reaches 87.5 % (runs of 4 / 8 / 32 chunks 90.9 / 92.2 /
//     92.3 %, natural order 83 %; 512 threads 90 %; eight loads per thread 89 - 90 %; two 74 %: the
//     barrier and the launch of sixteen waves then weigh more than the reading); the kernel itself gains
//     2.5 % on 8 x 10^9 elements, 1 - 3 % on the VGG-A shapes and 2 % on one layer of 2.7 - 4.8 x 10^8
//     elements, and is level with the loop on 1.3 - 2.4 x 10^8 (the AlexNet shapes among them), hence the
//     threshold.  A wave per 1 - 4 KiB with a partial of its own reads at
//     50 - 85 %: the thin stream of partials costs what the code stream costs the encoder, so partials
//     stay rare (one per 64 KiB).
#ifndef TG_STAT_WIDE_FROM
#define TG_STAT_WIDE_FROM ((int64_t)1 << 28)
#endif
#ifndef TG_STAT_XCD_RUN
#define TG_STAT_XCD_RUN 16
#endif
constexpr int64_t kStatWideFrom = TG_STAT_WIDE_FROM;
constexpr int kStatWideBlock = 1024;
constexpr int kStatWideChunk = 16384;
constexpr int kStatXcdRun = TG_STAT_XCD_RUN;

// (chunks that a layer begins in take a slow path in the one-shot shape, so they have to be few: at most
// one in kStatWideMixedPer)
constexpr int64_t kStatWideMixedPer = 64;
__host__ __device__ constexpr bool stat_wide(const int64_t total_elements, const int64_t n_chunks, const int64_t mixed_chunks) {
    return total_elements >= kStatWideFrom && mixed_chunks * kStatWideMixedPer <= n_chunks;
}

// elements per statistics chunk of the looping shape (a workgroup reduces at most one chunk)
__host__ __device__ constexpr int stat_chunk(const int64_t total_elements) {
    return total_elements < ((int64_t)1 << 26) ? 8192
         : total_elements < ((int64_t)1 << 28) ? 16384
         : total_elements < ((int64_t)1 << 29) ? 32768 : 65536;
}

constexpr int kSmallSeg = 2048;         // segments up to this size are reduced by one wave, four per workgroup

// What one workgroup of the statistics pass reduces: a slot per wave, 32 contiguous bytes, so that
// one scalar load gives a wave everything it needs to address its data.
struct StatSlot {
    int64_t begin, end;             // element range of the wave's segment (a large segment: the same in all four slots)
    int64_t pivot;                  // index of the first element of that segment's layer
    int64_t seg_kind;               // 8 * (index of the segment) + count; count 0: one large segment, block-wide;
                                    // 1..4: the unit holds that many small segments, one per wave
};
struct StatUnit {
    StatSlot slot[kBlock / kWave];
};
static_assert(sizeof(StatUnit) == 128, "one record = two cache lines of 64 bytes");

struct StatsArgs {
    const float* grads[kMaxWorkers];
    const StatUnit* units;          // [n_units]
    double* psum;                   // [W][n_segs] sum (g - K)
    double* psq;                    // [W][n_segs] sum (g - K)^2
    float* pmax;                    // [W][n_segs] max |g|
    int64_t n_segs;
};

struct Acc {
    double s1, s2;
    float m;
};

__device__ __forceinline__ void acc_add(Acc& a, const float x, const double K) {
    const double d = (double)x - K;
    a.s1 += d;
    a.s2 = __builtin_fma(d, d, a.s2);
    a.m = max_abs(a.m, x);
}

__device__ __forceinline__ void acc_add4(Acc& a, const float4 v, const double K) {
    acc_add(a, v.x, K);
    acc_add(a, v.y, K);
    acc_add(a, v.z, K);
    acc_add(a, v.w, K);
}

// Sum / maximum over the 64 lanes in a fixed order, the same value in every lane: inside each row of
// 16 lanes four data-parallel-primitive steps (swap with the neighbour, with the neighbouring pair,
// rotate the row by 4 and by 8), then lanes 0, 16, 32, 48 are read out and folded.  (A butterfly of six
// cross-lane exchanges through the LDS crossbar takes several times as long, and a wave that has
// nothing left to load still holds its place on the SIMD while it reduces.)
constexpr int kDppSwap1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppSwap2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppRowRor4 = 0x124;
constexpr int kDppRowRor8 = 0x128;

template <int CTRL>
__device__ __forceinline__ double dpp_move(const double x) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

template <int CTRL>
__device__ __forceinline__ float dpp_move(const float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}

__device__ __forceinline__ double read_lane(const double x, const int l) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(x), l),
                            __builtin_amdgcn_readlane(__double2loint(x), l));
}

__device__ __forceinline__ float read_lane(const float x, const int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

__device__ __forceinline__ double wave_sum(double x) {
    x += dpp_move<kDppSwap1>(x);
    x += dpp_move<kDppSwap2>(x);
    x += dpp_move<kDppRowRor4>(x);
    x += dpp_move<kDppRowRor8>(x);
    return (read_lane(x, 0) + read_lane(x, 16)) + (read_lane(x, 32) + read_lane(x, 48));
}

__device__ __forceinline__ float wave_max(float x) {
    x = fmaxf(x, dpp_move<kDppSwap1>(x));
    x = fmaxf(x, dpp_move<kDppSwap2>(x));
    x = fmaxf(x, dpp_move<kDppRowRor4>(x));
    x = fmaxf(x, dpp_move<kDppRowRor8>(x));
    return fmaxf(fmaxf(read_lane(x, 0), read_lane(x, 16)), fmaxf(read_lane(x, 32), read_lane(x, 48)));
}

__device__ __forceinline__ Acc wave_reduce(Acc a) {
    a.s1 = wave_sum(a.s1);
    a.s2 = wave_sum(a.s2);
    a.m = wave_max(a.m);
    return a;
}

// The pivot as a double, converted where it is first needed.  The conversion is opaque to the
// compiler so that it stays behind the data loads of the iteration it is in: the pivot itself is
// still in flight when those are issued, and hoisting the conversion would wait for it first.
__device__ __forceinline__ double pivot_value(const float Kf) {
    double K;
    asm volatile("v_cvt_f64_f32 %0, %1" : "=v"(K) : "v"(Kf));
    return K;
}

// sums of one segment [b, e) over `nthr` cooperating threads (this thread is number t of them)
__device__ __forceinline__ Acc segment_sums(const float* __restrict__ g, const int64_t b, const int64_t e,
                                            const float Kf, const int t, const int nthr) {
    Acc a = {0.0, 0.0, 0.0f};
    const int64_t b4 = (b + 3) & ~(int64_t)3;
    const int64_t e4 = e & ~(int64_t)3;
    if (b4 < e4) {
        const float* gp = g + b4;
        const int64_t nv = (e4 - b4) >> 2;          // float4 groups
        int64_t i = t;
        // four streaming loads in flight per thread
        for (; i + 3 * nthr < nv; i += 4 * nthr) {
            const float4 v0 = load_stream(gp + 4 * i), v1 = load_stream(gp + 4 * (i + nthr));
            const float4 v2 = load_stream(gp + 4 * (i + 2 * nthr)), v3 = load_stream(gp + 4 * (i + 3 * nthr));
            __builtin_amdgcn_sched_barrier(0);      // all four are issued before the first one is waited for
            const double K = pivot_value(Kf);
            acc_add4(a, v0, K);
            acc_add4(a, v1, K);
            acc_add4(a, v2, K);
            acc_add4(a, v3, K);
        }
        // up to three groups are left for this thread: their loads are issued together as well
        const bool h0 = i < nv, h1 = i + nthr < nv, h2 = i + 2 * nthr < nv;
        float4 r0, r1, r2;
        if (h0) r0 = load_stream(gp + 4 * i);
        if (h1) r1 = load_stream(gp + 4 * (i + nthr));
        if (h2) r2 = load_stream(gp + 4 * (i + 2 * nthr));
        __builtin_amdgcn_sched_barrier(0);
        const double K = pivot_value(Kf);
        if (h0) acc_add4(a, r0, K);
        if (h1) acc_add4(a, r1, K);
        if (h2) acc_add4(a, r2, K);
        // ragged head and tail, at most 3 elements each
        if (t < b4 - b) acc_add(a, g[b + t], K);
        if (t < e - e4) acc_add(a, g[e4 + t], K);
    } else {
        const double K = pivot_value(Kf);
        for (int64_t i = b + t; i < e; i += nthr) acc_add(a, g[i], K);
    }
    return a;
}

// One workgroup per unit: either one large segment (a run of at most one chunk inside one layer),
// reduced by all 256 threads, or up to four small segments, one per wave.
__global__ void __launch_bounds__(kBlock) clip_stats_partial_kernel(const StatsArgs p) {
    constexpr int NT = kBlock, NW = kBlock / kWave;
    __shared__ double sh1[NW], sh2[NW];
    __shared__ float shm[NW];

    const int64_t unit = blockIdx.x;
    const int w = blockIdx.y;
    const float* __restrict__ g = p.grads[w];
    const int t = threadIdx.x;
    // everything a wave needs comes from its slot of the unit record, whatever the kind of unit (the
    // host repeats a large segment in all four slots): one load, which does not wait for the branch below
    const int wave = wave_uniform(t >> 6);
    const StatSlot& u = p.units[unit].slot[wave];
    const int64_t sg = u.seg_kind >> 3;
    const int count = (int)(u.seg_kind & 7);
    const int64_t sb = u.begin, se = u.end;
    // the pivot travels through the vector memory path, like the data and ahead of it: results
    // return in order, so waiting for it does not wait for the data loads issued behind it
    // (a uniform address would become a scalar load; a zero the compiler cannot see through keeps it
    // a vector load)
    int lane_zero;
    asm("v_mov_b32 %0, 0" : "=v"(lane_zero));
    const float K = g[u.pivot + lane_zero];

    if (count > 0) {
        // small segments: wave j takes segment first + j
        if (wave >= count) return;
        Acc a = segment_sums(g, sb, se, K, t & 63, kWave);
        a = wave_reduce(a);
        if ((t & 63) == 0) {
            const int64_t o = (int64_t)w * p.n_segs + sg;
            p.psum[o] = a.s1;
            p.psq[o] = a.s2;
            p.pmax[o] = a.m;
        }
        return;
    }

    Acc a = segment_sums(g, sb, se, K, t, NT);
    a = wave_reduce(a);
    if ((t & 63) == 0) {
        sh1[t >> 6] = a.s1;
        sh2[t >> 6] = a.s2;
        shm[t >> 6] = a.m;
    }
    __syncthreads();
    if (t == 0) {
        double s1 = sh1[0], s2 = sh2[0];
        float m = shm[0];
#pragma unroll
        for (int k = 1; k < NW; ++k) {
            s1 += sh1[k];
            s2 += sh2[k];
            m = fmaxf(m, shm[k]);
        }
        const int64_t o = (int64_t)w * p.n_segs + sg;
        p.psum[o] = s1;
        p.psq[o] = s2;
        p.pmax[o] = m;
    }
}

// ---- the one-shot shape for large jobs ----
// A workgroup of 1024 threads per chunk of 16384 elements.  The address of the data follows from the
// workgroup index alone, so the four loads of every thread are issued first; the chunk's record (which
// segments it holds, where their layer begins) and the pivot arrive while those are in flight.  A
// chunk inside one layer - all but a few - is then one segment and one partial; a chunk that layers
// begin in is reduced segment by segment with plain strided loads (the loads issued ahead are wasted).
struct StatChunk {
    int64_t seg0;                   // index of the chunk's first segment
    int64_t pivot;                  // index of the first element of that segment's layer
    int32_t nseg;                   // segments in the chunk
    int32_t pad0;
    int64_t pad1;
};
static_assert(sizeof(StatChunk) == 32, "two records per 64-byte line");

struct StatSeg {
    int64_t begin, end;             // element range
    int64_t pivot;                  // index of the first element of the segment's layer
    int64_t pad;
};

struct StatsWideArgs {
    const float* grads[kMaxWorkers];
    const StatChunk* chunks;        // [n_chunks]
    const StatSeg* segs;            // [n_segs]
    double* psum;
    double* psq;
    float* pmax;
    int64_t n_segs, n_chunks, n;
};

constexpr int kStatWideWaves = kStatWideBlock / kWave;

// fold of the workgroup's sixteen waves in a fixed order; thread 0 writes the partial of segment sg
__device__ __forceinline__ void wide_fold_store(const StatsWideArgs& p, Acc a, const int w, const int64_t sg,
                                                double* sh1, double* sh2, float* shm) {
    const int t = threadIdx.x;
    a = wave_reduce(a);
    if ((t & 63) == 0) {
        sh1[t >> 6] = a.s1;
        sh2[t >> 6] = a.s2;
        shm[t >> 6] = a.m;
    }
    __syncthreads();
    if (t == 0) {
        double s1 = sh1[0], s2 = sh2[0];
        float m = shm[0];
#pragma unroll
        for (int k = 1; k < kStatWideWaves; ++k) {
            s1 += sh1[k];
            s2 += sh2[k];
            m = fmaxf(m, shm[k]);
        }
        const int64_t o = (int64_t)w * p.n_segs + sg;
        p.psum[o] = s1;
        p.psq[o] = s2;
        p.pmax[o] = m;
    }
}

__global__ void __launch_bounds__(kStatWideBlock, 8) clip_stats_wide_kernel(const StatsWideArgs p) {
    __shared__ double sh1[kStatWideWaves], sh2[kStatWideWaves];
    __shared__ float shm[kStatWideWaves];

    // chunks in the XCD-aware order (the grid is rounded up to whole runs)
    const int64_t c = xcd_run_index(blockIdx.x, kStatXcdRun);
    if (c >= p.n_chunks) return;
    const int w = blockIdx.y;
    const float* __restrict__ g = p.grads[w];
    const int t = threadIdx.x;
    const int64_t e0 = c * kStatWideChunk;
    const bool full = e0 + kStatWideChunk <= p.n;
    float4 v[4];
    if (full) {
        const float* gp = g + e0 + 4 * t;
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = load_stream(gp + 4 * kStatWideBlock * k);
    }
    // the record and the pivot are scalar loads: they arrive beside the data, not behind it
    const StatChunk* r = p.chunks + c;
    const int64_t seg0 = load_uniform(&r->seg0);
    const int nseg = load_uniform(&r->nseg);
    if (full && nseg == 1) {
        const double K = (double)load_uniform(g + load_uniform(&r->pivot));
        Acc a = {0.0, 0.0, 0.0f};
#pragma unroll
        for (int k = 0; k < 4; ++k) acc_add4(a, v[k], K);
        wide_fold_store(p, a, w, seg0, sh1, sh2, shm);
        return;
    }
    if (full) {
        // a chunk that layers begin in: its data is in the registers already; every segment takes the
        // elements at its positions (the others add an exact zero), one fold and one partial per segment.
        // About 160 vector instructions per thread and segment, which is why the host takes this shape
        // only when chunks of this kind are few.
        for (int j = 0; j < nseg; ++j) {
            const StatSeg* sg = p.segs + seg0 + j;
            const int rb = (int)(load_uniform(&sg->begin) - e0), re = (int)(load_uniform(&sg->end) - e0);
            const double K = (double)load_uniform(g + load_uniform(&sg->pivot));
            Acc a = {0.0, 0.0, 0.0f};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float x[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int pos = 4 * kStatWideBlock * k + 4 * t + i;
                    const bool inside = pos >= rb && pos < re;
                    const double d = inside ? (double)x[i] - K : 0.0;
                    a.s1 += d;
                    a.s2 = __builtin_fma(d, d, a.s2);
                    a.m = inside ? max_abs(a.m, x[i]) : a.m;
                }
            }
            wide_fold_store(p, a, w, seg0 + j, sh1, sh2, shm);
            __syncthreads();        // the fold has read the wave sums before the next segment overwrites them
        }
        return;
    }
    // the ragged last chunk of the buffer: plain strided loads
    for (int j = 0; j < nseg; ++j) {
        const StatSeg* sg = p.segs + seg0 + j;
        const int64_t b = load_uniform(&sg->begin), e = load_uniform(&sg->end);
        const double K = (double)load_uniform(g + load_uniform(&sg->pivot));
        Acc a = {0.0, 0.0, 0.0f};
        for (int64_t i = b + t; i < e; i += kStatWideBlock) acc_add(a, g[i], K);
        wide_fold_store(p, a, w, seg0 + j, sh1, sh2, shm);
        __syncthreads();
    }
}

struct StatsFinalArgs {
    const int64_t* off;             // [L+1]
    const int64_t* layer_seg;       // [L+1] first segment of each layer
    const double* psum;
    const double* psq;
    const float* pmax;
    float* tau;                     // [W][L]
    float* s_local;                 // [W][L]
    int64_t n_segs;
    int32_t n_layers;
    float c;
    int32_t noclip;
    const uint8_t* layer_float;     // [L] or null: layers kept in floating point get tau = 0 and s_local = 0
};

__device__ __forceinline__ void finish_layer(const StatsFinalArgs& p, const int l, const int w,
                                             const double s1, const double s2, const float m) {
    const int64_t cnt = p.off[l + 1] - p.off[l];
    double sigma = 0.0;
    if (cnt > 0) {
        const double md = s1 / (double)cnt;                     // mean - K
        const double var = s2 / (double)cnt - md * md;
        sigma = var > 0.0 ? sqrt(var) : 0.0;
    }
    float tau = p.noclip ? __builtin_inff() : (float)((double)p.c * sigma);
    // a layer that is not ternarized (Section 4.2): threshold and scaler 0, so that the encoder writes
    // the code 00 for all of it and the decoder zeros, whatever the gradients hold
    if (p.layer_float != nullptr && p.layer_float[l] != 0) tau = 0.0f;
    const int64_t o = (int64_t)w * p.n_layers + l;
    p.tau[o] = tau;
    p.s_local[o] = fminf(m, tau);                               // Eq. 2 on the clipped layer
}

// Few layers (the networks of the paper): one workgroup of 1024 threads per layer and worker.
constexpr int kFinalBlock = 1024;

__global__ void __launch_bounds__(kFinalBlock) clip_stats_final_kernel(const StatsFinalArgs p) {
    __shared__ double sh1[kFinalBlock / kWave], sh2[kFinalBlock / kWave];
    __shared__ float shm[kFinalBlock / kWave];

    const int l = blockIdx.x, w = blockIdx.y, t = threadIdx.x;
    const int64_t sb = p.layer_seg[l], se = p.layer_seg[l + 1];
    const int64_t base = (int64_t)w * p.n_segs;
    Acc a = {0.0, 0.0, 0.0f};
    // (a long layer of a large job has tens of thousands of partials - 61 036 x 20 bytes per worker for 10^9
    // elements - and one workgroup reads them at what one CU can read, 58 GB/s: 21 us, 0.2 % of that job's
    // step; four or eight loads per thread in flight change nothing)
    for (int64_t i = sb + t; i < se; i += kFinalBlock) {
        a.s1 += p.psum[base + i];
        a.s2 += p.psq[base + i];
        a.m = fmaxf(a.m, p.pmax[base + i]);
    }
    a = wave_reduce(a);
    if ((t & 63) == 0) {
        sh1[t >> 6] = a.s1;
        sh2[t >> 6] = a.s2;
        shm[t >> 6] = a.m;
    }
    __syncthreads();
    if (t == 0) {
        double s1 = sh1[0], s2 = sh2[0];
        float m = shm[0];
#pragma unroll
        for (int k = 1; k < kFinalBlock / kWave; ++k) {
            s1 += sh1[k];
            s2 += sh2[k];
            m = fmaxf(m, shm[k]);
        }
        finish_layer(p, l, w, s1, s2, m);
    }
}

// Many layers (fine buckets): a thread per layer.  A layer with a few partials is folded by its own
// thread, one after the other; the layers of a wave that have more are then folded by the whole
// wave, layer after layer (lanes strided over the partials, fixed-order wave reduction).  Which of the two a
// layer gets depends on its number of partials alone, so the order of the additions is fixed.
constexpr int kFinalPerThreadFrom = 1024;   // layers
constexpr int kFinalSerial = 8;           // partials a single thread folds

__global__ void __launch_bounds__(kBlock) clip_stats_final_per_thread_kernel(const StatsFinalArgs p) {
    const int w = blockIdx.y, lane = threadIdx.x & 63;
    const int64_t l64 = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const bool have = l64 < p.n_layers;
    const int l = have ? (int)l64 : 0;
    const int64_t base = (int64_t)w * p.n_segs;
    int sb = 0, se = 0;                         // fewer than 2^31 segments (elements / chunk + layers)
    if (have) {
        sb = (int)p.layer_seg[l];
        se = (int)p.layer_seg[l + 1];
    }
    const bool coop = se - sb > kFinalSerial;
    if (have && !coop) {
        Acc a = {0.0, 0.0, 0.0f};
        for (int i = sb; i < se; ++i) {
            a.s1 += p.psum[base + i];
            a.s2 += p.psq[base + i];
            a.m = fmaxf(a.m, p.pmax[base + i]);
        }
        finish_layer(p, l, w, a.s1, a.s2, a.m);
    }
    unsigned long long todo = __ballot(coop);   // wave-uniform: every lane walks the same list
    while (todo != 0ull) {
        const int j = __ffsll((long long)todo) - 1;
        todo &= todo - 1ull;
        const int b = __shfl(sb, j, kWave), e = __shfl(se, j, kWave);
        Acc a = {0.0, 0.0, 0.0f};
        for (int i = b + lane; i < e; i += kWave) {
            a.s1 += p.psum[base + i];
            a.s2 += p.psq[base + i];
            a.m = fmaxf(a.m, p.pmax[base + i]);
        }
        a = wave_reduce(a);
        if (lane == j) finish_layer(p, l, w, a.s1, a.s2, a.m);
    }
}

__global__ void share_scalers_kernel(const float* __restrict__ s_local, float* __restrict__ s_shared,
                                     const int n_workers, const int n_layers) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n_layers) return;
    float m = s_local[l];
    for (int w = 1; w < n_workers; ++w) m = fmaxf(m, s_local[(int64_t)w * n_layers + l]);
    s_shared[l] = m;                                                // Eq. 4
}

// iteration counter kept in device memory (see tg_ternarize_pack_devstep)
__global__ void step_advance_kernel(uint32_t* step_dev, const uint32_t by) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *step_dev += by;
}

}  // namespace tg
