// Per-layer clip threshold and scaler (Eq. 5 and Eq. 2) in one read of g.
//
// max|clip(g)| = min(max|g|, c*sigma), so sigma and the scaler come out of the
// same pass.  Sums are fp64 and taken about a per-layer pivot K = first element
// of the layer (shifted-data variance: exact for a constant layer, insensitive to
// a large mean).  No float atomics: every statistics chunk (8192 to 65536 elements, by the size of
// the job) is cut into segments, one per layer it touches; a
// workgroup reduces one large segment (or four small ones, a wave each) in a fixed tree and
// writes one partial per segment; a second small kernel folds the partials of each layer in
// a fixed order.  Results are bit-identical from
// run to run.
#pragma once

#include "tg_common.hpp"

namespace tg {

// elements per statistics chunk (a workgroup reduces at most one chunk): 256 threads x 8..64 float4.
// Larger chunks amortise the per-workgroup cost, smaller ones keep enough workgroups in flight; the
// best size grows with the total work of a call (measured: 8192 for 25 M elements over all
// workers, 16384 - 32768 for 244 M, 65536 from 1 G on).
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

// xor butterfly: every lane ends with the same bits (a + b == b + a at each step)
__device__ __forceinline__ Acc wave_reduce(Acc a) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        a.s1 += __shfl_xor(a.s1, o, kWave);
        a.s2 += __shfl_xor(a.s2, o, kWave);
        a.m = fmaxf(a.m, __shfl_xor(a.m, o, kWave));
    }
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
    __shared__ double sh1[kBlock / kWave], sh2[kBlock / kWave];
    __shared__ float shm[kBlock / kWave];

    const int w = blockIdx.y;
    const float* __restrict__ g = p.grads[w];
    const int t = threadIdx.x;
    // everything a wave needs comes from its slot of the unit record, whatever the kind of unit (the
    // host repeats a large segment in all four slots): one load, which does not wait for the branch below
    const int wave = wave_uniform(t >> 6);
    const StatSlot& u = p.units[blockIdx.x].slot[wave];
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

    Acc a = segment_sums(g, sb, se, K, t, kBlock);
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
        for (int k = 1; k < kBlock / kWave; ++k) {
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
    const float tau = p.noclip ? __builtin_inff() : (float)((double)p.c * sigma);
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
// wave, layer after layer (lanes strided over the partials, xor butterfly).  Which of the two a
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
