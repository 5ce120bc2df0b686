// Knapsack allocation on the device (paper Appendix C; Section 3.2, Eq. optimisation).
//
// Table rows are indexed by cost in units of `unit` pairs; row i holds the least total error of
// layers 0..i at each exact cost.  Layers are visited in order, candidates in ascending j with a
// strict "<", and the answer ends at the smallest cost attaining the least total: every fp64
// add happens in the same order as in a plain sequential implementation, so the choice is
// reproducible bit for bit.
#pragma once
#include "common.h"

namespace kimad {

struct AllocBuffers {
    const double* E;         // [L][J]
    const uint32_t* Ktab;    // [L][J]
    uint32_t L, J;
    uint64_t unit;           // cost unit in pairs
    uint32_t cap;            // capacity in units
    double* row0;            // [cap+1]
    double* row1;            // [cap+1]
    uint8_t* choice;         // [L][stride]
    uint64_t stride;         // >= cap+1
    int32_t* j_out;
    uint64_t* K_out;
    uint64_t* offsets_out;
    int32_t* status;
    uint32_t* flags;         // [0] non-finite seen
};

constexpr double DP_INF = __builtin_huge_val();

__device__ __forceinline__ uint32_t units_of(uint32_t K, uint64_t unit) {
    return (uint32_t)(((uint64_t)K + unit - 1) / unit);
}

// Any Inf/NaN in the table?  Also seeds row 0 of the DP: 0 at cost 0, +inf elsewhere.
__global__ __launch_bounds__(256) void k_dp_init(AllocBuffers ab) {
    const uint32_t gid = blockIdx.x * 256u + threadIdx.x, gsz = gridDim.x * 256u;
    for (uint64_t t = gid; t < (uint64_t)ab.L * ab.J; t += gsz) {
        const double e = ab.E[t];
        if (!(e - e == 0.0)) atomicOr(&ab.flags[0], 1u);
    }
    for (uint64_t c = gid; c <= ab.cap; c += gsz) ab.row0[c] = c ? DP_INF : 0.0;
}

// One layer of the recurrence, one thread per cost cell (capacities too large for LDS rows).
__global__ __launch_bounds__(256) void k_dp_layer(AllocBuffers ab, uint32_t i, const double* prev, double* cur) {
    __shared__ double sE[KIMAD_MAX_J_CONST];
    __shared__ uint32_t sW[KIMAD_MAX_J_CONST];
    if (threadIdx.x < ab.J) {
        sE[threadIdx.x] = ab.E[(size_t)i * ab.J + threadIdx.x];
        sW[threadIdx.x] = units_of(ab.Ktab[(size_t)i * ab.J + threadIdx.x], ab.unit);
    }
    __syncthreads();
    const uint64_t c = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (c > ab.cap) return;
    double best = DP_INF;
    uint32_t bj = 0xFF;
    for (uint32_t j = 0; j < ab.J; ++j) {
        const uint32_t w = sW[j];
        if (w > c) break;                          // costs ascend with j
        const double t = prev[c - w] + sE[j];
        if (t < best) { best = t; bj = j; }
    }
    cur[c] = best;
    ab.choice[(size_t)i * ab.stride + c] = (uint8_t)bj;
}

// Candidate lists.  Candidates of one layer that cost the same number of units differ only in
// their error, and a table row is non-increasing in j: of such a run only the last (least error)
// can give the least total, and the strict "<" of the sequential scan keeps the lowest j of the
// run whose rounded total equals that least one.  So a run is evaluated at its last member and
// then backwards while the rounded total stays equal: the same winner as visiting every member, in
// about two additions instead of the run's length.  Runs whose errors are not non-increasing (only
// possible in a caller-supplied table) are kept as single candidates.  Candidates that cost more
// than the capacity are dropped.
struct DpLists {
    uint32_t* w;     // [L][J] cost in units of the entry
    uint8_t* jlo;    // [L][J] first member of the run
    uint8_t* jhi;    // [L][J] last member of the run
    uint32_t* n;     // [L] entries
};

__global__ __launch_bounds__(64) void k_dp_prep(AllocBuffers ab, DpLists dl) {
    const uint32_t i = blockIdx.x, j = threadIdx.x;
    __shared__ uint32_t sw[KIMAD_MAX_J_CONST];
    __shared__ double se[KIMAD_MAX_J_CONST];
    if (j < ab.J) {
        sw[j] = units_of(ab.Ktab[(size_t)i * ab.J + j], ab.unit);
        se[j] = ab.E[(size_t)i * ab.J + j];
    }
    __syncthreads();
    if (j == 0) {
        uint32_t n = 0;
        uint32_t a = 0;
        while (a < ab.J && sw[a] <= ab.cap) {
            uint32_t b = a;                       // maximal run [a, b] of equal cost with non-increasing error
            while (b + 1 < ab.J && sw[b + 1] == sw[a] && se[b + 1] <= se[b]) ++b;
            dl.w[(size_t)i * ab.J + n] = sw[a];
            dl.jlo[(size_t)i * ab.J + n] = (uint8_t)a;
            dl.jhi[(size_t)i * ab.J + n] = (uint8_t)b;
            ++n;
            a = b + 1;
        }
        dl.n[i] = n;
    }
}

// Whole recurrence in one workgroup with both rows in LDS (capacity up to DP_LDS_CELLS - 1).
// The next layer's errors and candidate list are fetched while the current layer is computed.
constexpr uint32_t DP_LDS_CELLS = 6144;
__global__ __launch_bounds__(1024) void k_dp_lds(AllocBuffers ab, DpLists dl) {
    __shared__ double rows[2][DP_LDS_CELLS];
    __shared__ double sE[2][KIMAD_MAX_J_CONST];
    __shared__ uint32_t sW[2][KIMAD_MAX_J_CONST];
    __shared__ uint32_t sJ[2][KIMAD_MAX_J_CONST];      // jlo | jhi << 8
    __shared__ uint32_t sN[2];
    const uint32_t tid = threadIdx.x;
    for (uint32_t c = tid; c <= ab.cap; c += 1024) rows[0][c] = c ? DP_INF : 0.0;
    auto fetch = [&](uint32_t i, uint32_t buf) {
        if (tid < ab.J) {
            sE[buf][tid] = ab.E[(size_t)i * ab.J + tid];
            sW[buf][tid] = dl.w[(size_t)i * ab.J + tid];
            sJ[buf][tid] = (uint32_t)dl.jlo[(size_t)i * ab.J + tid] | ((uint32_t)dl.jhi[(size_t)i * ab.J + tid] << 8);
        }
        if (tid == 64) sN[buf] = dl.n[i];
    };
    fetch(0, 0);
    __syncthreads();
    for (uint32_t i = 0; i < ab.L; ++i) {
        const uint32_t buf = i & 1;
        if (i + 1 < ab.L) fetch(i + 1, buf ^ 1);
        const double* prev = rows[i & 1];
        double* cur = rows[(i + 1) & 1];
        const uint32_t n = sN[buf];
        for (uint32_t c = tid; c <= ab.cap; c += 1024) {
            double best = DP_INF;
            uint32_t bj = 0xFF;
            for (uint32_t k = 0; k < n; ++k) {
                const uint32_t w = sW[buf][k];
                if (w > c) break;                          // costs ascend along the list
                const double p = prev[c - w];
                const uint32_t jj = sJ[buf][k];
                uint32_t j = jj >> 8;
                const double t = p + sE[buf][j];
                if (t < best) {
                    const uint32_t jlo = jj & 0xFFu;
                    while (j > jlo && p + sE[buf][j - 1] == t) --j;   // lowest member with the same rounded total
                    best = t;
                    bj = j;
                }
            }
            cur[c] = best;
            ab.choice[(size_t)i * ab.stride + c] = (uint8_t)bj;
        }
        __syncthreads();
    }
    // hand the last row to the final kernel
    const double* last = rows[ab.L & 1];
    for (uint32_t c = tid; c <= ab.cap; c += 1024) ab.row0[c] = last[c];
}

// Smallest cost attaining the least total, back-tracking, outputs.  One workgroup.
__global__ __launch_bounds__(1024) void k_dp_final(AllocBuffers ab, const double* last, int32_t err_infeasible,
                                                   int32_t err_nonfinite) {
    __shared__ double sv[16];
    __shared__ unsigned long long sc[16];
    __shared__ unsigned long long cstar;
    __shared__ int32_t st;
    const uint32_t tid = threadIdx.x;
    double best = DP_INF;
    unsigned long long bc = ~0ull;
    for (uint64_t c = tid; c <= ab.cap; c += 1024) {
        const double v = last[c];
        if (v < best) { best = v; bc = c; }     // ascending c per thread: keeps the smallest
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) {
        const double ov = __shfl_xor(best, d, 64);
        const unsigned long long oc = __shfl_xor(bc, d, 64);
        if (ov < best || (ov == best && oc < bc)) { best = ov; bc = oc; }
    }
    if (lane_id() == 0) { sv[tid >> 6] = best; sc[tid >> 6] = bc; }
    __syncthreads();
    if (tid == 0) {
        for (uint32_t w = 1; w < 16; ++w)
            if (sv[w] < best || (sv[w] == best && sc[w] < bc)) { best = sv[w]; bc = sc[w]; }
        int32_t s = 0;
        if (ab.flags[0]) s = err_nonfinite;
        else if (!(best < DP_INF)) s = err_infeasible;
        st = s;
        cstar = bc;
        *ab.status = s;
    }
    __syncthreads();
    if (st != 0) {
        for (uint32_t i = tid; i < ab.L; i += 1024) { ab.j_out[i] = 0; ab.K_out[i] = 0; }
        for (uint32_t i = tid; i <= ab.L; i += 1024) ab.offsets_out[i] = 0;
        return;
    }
    if (tid == 0) {
        uint64_t c = cstar;
        for (uint32_t i = ab.L; i-- > 0;) {
            const uint32_t j = ab.choice[(size_t)i * ab.stride + c];
            const uint32_t K = ab.Ktab[(size_t)i * ab.J + j];
            ab.j_out[i] = (int32_t)j;
            ab.K_out[i] = K;
            c -= units_of(K, ab.unit);
        }
        uint64_t run = 0;
        for (uint32_t i = 0; i < ab.L; ++i) { ab.offsets_out[i] = run; run += ab.K_out[i]; }
        ab.offsets_out[ab.L] = run;
    }
}

}  // namespace kimad
