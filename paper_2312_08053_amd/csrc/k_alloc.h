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
    uint32_t* jj;    // [L][J] first member of the run | last member << 8
    double* e;       // [L][J][2] error of the last member, error of the member before it (NaN for a single)
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
            const size_t o = (size_t)i * ab.J + n;
            dl.w[o] = sw[a];
            dl.jj[o] = a | (b << 8);
            dl.e[2 * o] = se[b];
            dl.e[2 * o + 1] = b > a ? se[b - 1] : __longlong_as_double(0x7FF8000000000000ll);
            ++n;
            a = b + 1;
        }
        dl.n[i] = n;
    }
}

// Whole allocation in one workgroup: recurrence with both rows in LDS, then the smallest cost
// attaining the least total, back-tracking through choice rows staged in LDS, and the outputs.
// Rows are stored behind `pad` cells of +inf, so a candidate that costs more than the cell needs no
// test: it reads +inf and cannot win.  The candidate list is read with uniform addresses (scalar
// loads); per entry and cell the work is one LDS read, one add, one compare and three selects.
constexpr uint32_t DP_ROW = 6144;               // doubles per LDS row: pad + cells
constexpr uint32_t DP_CELLS_PER_THREAD = 3;     // capacity + 1 <= 3072

__global__ __launch_bounds__(1024) void k_dp_fused(AllocBuffers ab, const uint32_t* __restrict__ ent_w,
                                                   const uint32_t* __restrict__ ent_jj, const double* __restrict__ ent_e,
                                                   const uint32_t* __restrict__ ent_n, int32_t err_infeasible,
                                                   int32_t err_nonfinite) {
    __shared__ double rows[2][DP_ROW];          // 96 KB; reused for the choice rows afterwards
    __shared__ double sE[2][2 * KIMAD_MAX_J_CONST];   // per entry: error of the last member, of the one before
    __shared__ uint32_t sW[2][KIMAD_MAX_J_CONST];
    __shared__ uint32_t sJ[2][KIMAD_MAX_J_CONST];
    __shared__ uint32_t sN[2];
    __shared__ double sv[16];
    __shared__ unsigned long long sc[16];
    __shared__ unsigned long long cstar;
    __shared__ int32_t st;
    const uint32_t tid = threadIdx.x;
    const uint32_t ncell = ab.cap + 1;
    const uint32_t pad = ncell;                 // every cost is <= cap
    for (uint32_t c = tid; c < pad + ncell; c += 1024) {
        rows[0][c] = c == pad ? 0.0 : DP_INF;
        rows[1][c] = DP_INF;
    }
    // Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits for the
    // acknowledgement of every global store and load in flight (the choice rows, the next layer's
    // list), which would put a memory round trip into each of the L sequential steps.
    auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    if (tid < ab.J) {
        const size_t o = tid;
        sW[0][tid] = ent_w[o]; sJ[0][tid] = ent_jj[o];
        sE[0][2 * tid] = ent_e[2 * o]; sE[0][2 * tid + 1] = ent_e[2 * o + 1];
    }
    if (tid == 64) sN[0] = ent_n[0];
    __syncthreads();
    for (uint32_t i = 0; i < ab.L; ++i) {
        const uint32_t buf = i & 1;
        // issue the loads of the next layer's list now, park them in LDS after this layer's work
        uint32_t nw = 0, nj = 0, nn = 0;
        double ne0 = 0.0, ne1 = 0.0;
        const bool more = i + 1 < ab.L;
        if (more && tid < ab.J) {
            const size_t o = (size_t)(i + 1) * ab.J + tid;
            nw = ent_w[o]; nj = ent_jj[o]; ne0 = ent_e[2 * o]; ne1 = ent_e[2 * o + 1];
        }
        if (more && tid == 64) nn = ent_n[i + 1];
        const double* prev = rows[i & 1] + pad;
        double* cur = rows[(i + 1) & 1] + pad;
        const uint32_t n = sN[buf];
        for (uint32_t c = tid; c < ncell; c += 1024) {
            double best = DP_INF;
            uint32_t bk = 0xFF;                 // winning entry | 0x100 if the run's previous member rounds to the same total
            // branch-free over the entries, so that the LDS reads of several entries are in flight together
#pragma unroll 4
            for (uint32_t k = 0; k < n; ++k) {
                const uint32_t w = sW[buf][k];
                const double e_hi = sE[buf][2 * k], e_prev = sE[buf][2 * k + 1];
                const double p = prev[(int32_t)c - (int32_t)w];
                const double t = p + e_hi;
                const bool upd = t < best;
                const bool collide = p + e_prev == t;            // never for a single: e_prev is NaN
                best = upd ? t : best;
                bk = upd ? (k | (collide ? 0x100u : 0u)) : bk;
            }
            const uint32_t k = bk & 0xFFu;
            uint32_t bj = k == 0xFFu ? 0xFFu : (sJ[buf][k] >> 8);
            if (bk & 0x100u) {
                // rare: the lowest member of the run whose rounded total equals the winner's
                const uint32_t jlo = sJ[buf][k] & 0xFFu;
                const double p = prev[(int32_t)c - (int32_t)sW[buf][k]];
                uint32_t j = bj - 1u;
                while (j > jlo && p + ab.E[(size_t)i * ab.J + j - 1] == best) --j;
                bj = j;
            }
            cur[c] = best;
            ab.choice[(size_t)i * ab.stride + c] = (uint8_t)bj;
        }
        if (more && tid < ab.J) {
            sW[buf ^ 1][tid] = nw; sJ[buf ^ 1][tid] = nj;
            sE[buf ^ 1][2 * tid] = ne0; sE[buf ^ 1][2 * tid + 1] = ne1;
        }
        if (more && tid == 64) sN[buf ^ 1] = nn;
        lds_barrier();
    }
    __syncthreads();
    // least total, smallest cost attaining it
    const double* last = rows[ab.L & 1] + pad;
    double best = DP_INF;
    unsigned long long bc = ~0ull;
    for (uint32_t c = tid; c < ncell; c += 1024) {
        const double v = last[c];
        if (v < best) { best = v; bc = c; }
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
    // back-tracking: stage the choice rows of a group of layers in LDS, walk them, next group
    uint8_t* stage = reinterpret_cast<uint8_t*>(&rows[0][0]);
    const uint32_t per_group = (uint32_t)(sizeof(rows) / ncell);
    uint32_t hi = ab.L;
    while (hi > 0) {
        const uint32_t lo_l = hi > per_group ? hi - per_group : 0u;
        __syncthreads();
        for (uint32_t x = tid; x < (hi - lo_l) * ncell; x += 1024) {
            const uint32_t i = lo_l + x / ncell, c = x % ncell;
            stage[x] = ab.choice[(size_t)i * ab.stride + c];
        }
        __syncthreads();
        if (tid == 0) {
            uint64_t c = cstar;
            for (uint32_t i = hi; i-- > lo_l;) {
                const uint32_t j = stage[(i - lo_l) * ncell + c];
                const uint32_t K = ab.Ktab[(size_t)i * ab.J + j];
                ab.j_out[i] = (int32_t)j;
                ab.K_out[i] = K;
                c -= units_of(K, ab.unit);
            }
            cstar = c;
        }
        hi = lo_l;
    }
    __syncthreads();
    if (tid == 0) {
        uint64_t run = 0;
        for (uint32_t i = 0; i < ab.L; ++i) { ab.offsets_out[i] = run; run += ab.K_out[i]; }
        ab.offsets_out[ab.L] = run;
    }
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
