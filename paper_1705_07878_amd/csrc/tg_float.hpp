// Plain average of W fp32 gradients, for layers that are NOT ternarized (Section 4.2 keeps the
// last classification layer in floating point).  Streaming: 4W bytes read + 4 written per
// element.  Sums are fp64 in worker order and rounded once, so the result does not depend
// on the launch shape.
#pragma once

#include "tg_common.hpp"

namespace tg {

struct FloatAvgArgs {
    const float* grads[kMaxWorkers];
    float* avg;
    int64_t n;
    int32_t n_workers;
    int32_t head;   // 0..3 leading elements before the first 16-byte boundary (the same for every buffer)
};

__device__ __forceinline__ void average_float_one(const FloatAvgArgs& p, const int64_t e, const double dW) {
    double s = 0.0;
    for (int w = 0; w < p.n_workers; ++w) s += (double)p.grads[w][e];
    p.avg[e] = (float)(s / dW);
}

template <bool NT_OUT>
__global__ void __launch_bounds__(kBlock) average_float_kernel(const FloatAvgArgs p) {
    const int64_t i = p.head + ((int64_t)blockIdx.x * kBlock + threadIdx.x) * 4;
    const double dW = (double)p.n_workers;
    if (blockIdx.x == 0 && threadIdx.x == 0)
        for (int64_t e = 0; e < p.head && e < p.n; ++e) average_float_one(p, e, dW);
    if (i >= p.n) return;
    if (i + 3 < p.n) {
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        int w = 0;
        // four workers' loads in flight at a time
        for (; w + 3 < p.n_workers; w += 4) {
            const float4 a = load_stream(p.grads[w] + i), b = load_stream(p.grads[w + 1] + i);
            const float4 c = load_stream(p.grads[w + 2] + i), d = load_stream(p.grads[w + 3] + i);
            s0 = (((s0 + (double)a.x) + (double)b.x) + (double)c.x) + (double)d.x;
            s1 = (((s1 + (double)a.y) + (double)b.y) + (double)c.y) + (double)d.y;
            s2 = (((s2 + (double)a.z) + (double)b.z) + (double)c.z) + (double)d.z;
            s3 = (((s3 + (double)a.w) + (double)b.w) + (double)c.w) + (double)d.w;
        }
        for (; w < p.n_workers; ++w) {
            const float4 a = load_stream(p.grads[w] + i);
            s0 += (double)a.x;
            s1 += (double)a.y;
            s2 += (double)a.z;
            s3 += (double)a.w;
        }
        const float4 o = make_float4((float)(s0 / dW), (float)(s1 / dW),
                                     (float)(s2 / dW), (float)(s3 / dW));
        store_through4<NT_OUT>(p.avg + i, o);
    } else {
        for (int64_t e = i; e < p.n; ++e) average_float_one(p, e, dW);
    }
}

}  // namespace tg
