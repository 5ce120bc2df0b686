// Server side of a round (paper Algorithm 1, server lines "Aggregate all update estimators" and
// "Updates the model"): decode M sparse payloads into the M estimator copies, then one dense pass
//     x <- x - gamma * sum_m w_m u_hat_m.
// The decode touches a few percent of the estimators; the model step reads M + 1 dense vectors and
// writes one: it is the other HBM-bound kernel of the method, 4 (M + 2) bytes per element.
#pragma once
#include <hip/hip_fp16.h>
#include "common.h"

namespace kimad {

constexpr uint32_t MAX_WORKERS = 16;         // must equal KIMAD_MAX_WORKERS of the public header

// The estimators and weights of the model step.  The arrays are indexed with compile-time
// constants only (unrolled loops): a run-time index into a by-value kernel argument makes the
// compiler copy the whole table to scratch memory in every thread.
struct ServerArgs {
    const float* u_hat[MAX_WORKERS];
    double w[MAX_WORKERS];
    uint32_t M;
    uint64_t d;
};

// One worker's payload into its estimator: one thread per pair.  The pair's layer is found by
// bisection in the worker's offsets; indices inside a payload are distinct, so the additions need
// no atomics.  The payload is what a worker sent, not something this library produced: every
// workgroup first checks the offsets (non-decreasing, starting at 0, the total within the buffers'
// capacity, the layer starts non-decreasing up to d) and leaves without a write if they are not; a
// pair whose index lies outside its layer is skipped.  Either way the status word gets err_payload.
__global__ __launch_bounds__(256) void k_server_decode(const uint32_t* __restrict__ idx, const float* __restrict__ val,
                                                       const uint64_t* __restrict__ off, uint64_t capacity_pairs,
                                                       float* u_hat, const uint64_t* __restrict__ layer_start, uint32_t L,
                                                       uint64_t d, int32_t* status, int32_t err_payload,
                                                       uint32_t value_f16) {
    __shared__ int bad;
    if (threadIdx.x == 0) bad = 0;
    __syncthreads();
    int mine = 0;
    for (uint32_t i = threadIdx.x; i <= L; i += 256u) {
        const uint64_t o = off[i], ls = layer_start[i];
        if (i == 0 && o != 0) mine = 1;
        if (i < L && (off[i + 1] < o || layer_start[i + 1] < ls)) mine = 1;
        if (i == L && (o > capacity_pairs || ls != d)) mine = 1;
    }
    if (mine) bad = 1;
    __syncthreads();
    if (bad) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicMin(status, err_payload);
        return;
    }
    const uint64_t total = off[L];
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t p = (uint64_t)blockIdx.x * 256u + threadIdx.x; p < total; p += stride) {
        uint32_t lo = 0, hi = L;                 // largest layer i with off[i] <= p
        while (hi - lo > 1) {
            const uint32_t mid = (lo + hi) >> 1;
            if (off[mid] <= p) lo = mid; else hi = mid;
        }
        const uint64_t first = layer_start[lo], n = layer_start[lo + 1] - first;
        const uint32_t t = idx[p];
        if ((uint64_t)t >= n) { atomicMin(status, err_payload); continue; }
        float* u = u_hat + first + t;
        // half-precision payloads carry binary16 bit patterns: the worker added the decoded value, so does the server
        const float v = value_f16 ? __half2float(__ushort_as_half(reinterpret_cast<const uint16_t*>(val)[p])) : val[p];
        gstore(u, gload(u) + v);
    }
}

// The model step, four elements per thread and trip; the tail and unaligned buffers take the
// scalar loop.  fp64 arithmetic per element, workers in order: every result is reproducible and
// equal to a plain sequential evaluation.
__global__ __launch_bounds__(256) void k_server_step(ServerArgs a, float* x, double gamma, uint32_t vec_ok) {
    const uint64_t gid = (uint64_t)blockIdx.x * 256u + threadIdx.x, stride = (uint64_t)gridDim.x * 256u;
    const uint64_t n4 = vec_ok ? a.d / 4 : 0;
    for (uint64_t q = gid; q < n4; q += stride) {
        const float4 xv = gload4_stream(x + 4 * q);
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
        for (uint32_t m = 0; m < MAX_WORKERS; ++m) {
            if (m < a.M) {
                const float4 u = gload4_stream(a.u_hat[m] + 4 * q);   // read once per step
                const double w = a.w[m];
                s0 = s0 + w * (double)u.x; s1 = s1 + w * (double)u.y;
                s2 = s2 + w * (double)u.z; s3 = s3 + w * (double)u.w;
            }
        }
        float4 r;
        r.x = (float)((double)xv.x - gamma * s0); r.y = (float)((double)xv.y - gamma * s1);
        r.z = (float)((double)xv.z - gamma * s2); r.w = (float)((double)xv.w - gamma * s3);
        gstore4(x + 4 * q, r);
    }
    for (uint64_t t = 4 * n4 + gid; t < a.d; t += stride) {
        double acc = 0.0;
#pragma unroll
        for (uint32_t m = 0; m < MAX_WORKERS; ++m)
            if (m < a.M) acc = acc + a.w[m] * (double)gload(a.u_hat[m] + t);
        gstore(x + t, (float)((double)gload(x + t) - gamma * acc));
    }
}

}  // namespace kimad
