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
    uint32_t* wall;  // [L][J] cost in units of candidate j
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
        dl.wall[(size_t)i * ab.J + j] = sw[j];
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
constexpr uint32_t DP_LIST_CAP = 2048;          // candidate-list entries held in LDS at a time
constexpr uint32_t DP_GROUP_MAX = 1024;         // layers per group at most (one thread plans one layer)

__global__ __launch_bounds__(1024) void k_dp_fused(AllocBuffers ab, const uint32_t* __restrict__ ent_w,
                                                   const uint32_t* __restrict__ ent_jj, const double* __restrict__ ent_e,
                                                   const uint32_t* __restrict__ ent_n,
                                                   const uint32_t* __restrict__ wall, int32_t err_infeasible,
                                                   int32_t err_nonfinite) {
    __shared__ double rows[2][DP_ROW];          // 96 KB; reused for the choice rows afterwards
    __shared__ double LE[2 * DP_LIST_CAP];      // 32 KB: per entry, error of the run's last member and of the one before
    __shared__ uint32_t LW[DP_LIST_CAP];        // 8 KB: cost in units
    __shared__ uint32_t LJ[DP_LIST_CAP];        // 8 KB: first member | last member << 8
    __shared__ uint32_t loff[DP_GROUP_MAX + 1]; // first entry of each layer of the group
    __shared__ uint32_t su[16];
    __shared__ uint32_t sh_g;
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
    // acknowledgement of every global store in flight (the choice rows), which would put a memory
    // round trip into each of the L sequential steps.
    auto lds_barrier = [] { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };
    // Layers are taken in groups whose candidate lists fit the LDS list buffer; the lists of a group
    // are copied in one sweep, so the memory latency is paid once per group, not once per layer.
    uint32_t i0 = 0;
    while (i0 < ab.L) {
        const uint32_t mine = (tid < DP_GROUP_MAX && i0 + tid < ab.L) ? ent_n[i0 + tid] : 0u;
        const uint32_t before = block_exclusive_scan<uint32_t>(mine, su, nullptr);
        if (tid == 0) sh_g = 0u;
        __syncthreads();
        const bool fits = tid < DP_GROUP_MAX && i0 + tid < ab.L && before + mine <= DP_LIST_CAP;
        if (fits) {
            loff[tid] = before;
            atomicMax(&sh_g, tid + 1u);          // layer counts are prefix-monotone: the group is layers 0..g-1
        }
        __syncthreads();
        const uint32_t g = sh_g;                 // >= 1: one layer has at most J <= 64 entries
        if (tid == g - 1u) loff[g] = before + mine;
        __syncthreads();
        for (uint32_t t = tid; t < g * ab.J; t += 1024) {
            const uint32_t layer = t / ab.J, k = t % ab.J;
            if (k < loff[layer + 1] - loff[layer]) {
                const size_t o = (size_t)(i0 + layer) * ab.J + k;
                const uint32_t d = loff[layer] + k;
                LW[d] = ent_w[o]; LJ[d] = ent_jj[o];
                LE[2 * d] = ent_e[2 * o]; LE[2 * d + 1] = ent_e[2 * o + 1];
            }
        }
        __syncthreads();
        for (uint32_t i = i0; i < i0 + g; ++i) {
            const double* prev = rows[i & 1] + pad;
            double* cur = rows[(i + 1) & 1] + pad;
            const uint32_t e0 = loff[i - i0], n = loff[i - i0 + 1] - e0;
            const uint32_t* lw = LW + e0;
            const uint32_t* lj = LJ + e0;
            const double* le = LE + 2 * e0;
            for (uint32_t c = tid; c < ncell; c += 1024) {
                double best = DP_INF;
                uint32_t bk = 0xFF;             // winning entry
#pragma unroll 8
                for (uint32_t k = 0; k < n; ++k) {
                    const double t = prev[(int32_t)c - (int32_t)lw[k]] + le[2 * k];
                    const bool upd = t < best;
                    best = upd ? t : best;
                    bk = upd ? k : bk;
                }
                uint32_t bj = 0xFFu;
                if (bk != 0xFFu) {
                    // Only the winner's run matters: if the member before its last one rounds to the same
                    // total (never for a single: that error is NaN), the lowest such member wins.
                    bj = lj[bk] >> 8;
                    const double p = prev[(int32_t)c - (int32_t)lw[bk]];
                    if (p + le[2 * bk + 1] == best) {
                        const uint32_t jlo = lj[bk] & 0xFFu;
                        uint32_t j = bj - 1u;
                        while (j > jlo && p + ab.E[(size_t)i * ab.J + j - 1] == best) --j;
                        bj = j;
                    }
                }
                cur[c] = best;
                ab.choice[(size_t)i * ab.stride + c] = (uint8_t)bj;
            }
            lds_barrier();
        }
        i0 += g;
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
    // back-tracking: stage the choice rows and the candidates' costs of a group of layers in LDS,
    // walk them, next group
    uint8_t* stage = reinterpret_cast<uint8_t*>(&rows[0][0]);
    const uint32_t wbytes = 4u * ab.J;
    const uint32_t per_layer = (ncell + wbytes + 3u) & ~3u;
    const uint32_t per_group = (uint32_t)(sizeof(rows) / per_layer);
    uint32_t hi = ab.L;
    while (hi > 0) {
        const uint32_t lo_l = hi > per_group ? hi - per_group : 0u;
        __syncthreads();
        for (uint32_t x = tid; x < (hi - lo_l) * ncell; x += 1024) {
            const uint32_t i = x / ncell, c = x % ncell;
            stage[i * per_layer + wbytes + c] = ab.choice[(size_t)(lo_l + i) * ab.stride + c];
        }
        for (uint32_t x = tid; x < (hi - lo_l) * ab.J; x += 1024) {
            const uint32_t i = x / ab.J, j = x % ab.J;
            reinterpret_cast<uint32_t*>(stage + i * per_layer)[j] = wall[(size_t)(lo_l + i) * ab.J + j];
        }
        __syncthreads();
        if (tid == 0) {
            uint64_t c = cstar;
            for (uint32_t i = hi; i-- > lo_l;) {
                const uint8_t* row = stage + (i - lo_l) * per_layer;
                const uint32_t j = row[wbytes + c];
                ab.j_out[i] = (int32_t)j;
                c -= reinterpret_cast<const uint32_t*>(row)[j];
            }
            cstar = c;
        }
        hi = lo_l;
    }
    __threadfence_block();
    __syncthreads();
    // sizes and offsets, in parallel
    unsigned long long carry = 0;
    for (uint32_t i0b = 0; i0b < ab.L; i0b += 1024) {
        const uint32_t i = i0b + tid;
        unsigned long long K = 0;
        if (i < ab.L) {
            K = ab.Ktab[(size_t)i * ab.J + (uint32_t)ab.j_out[i]];
            ab.K_out[i] = K;
        }
        unsigned long long tot;
        const unsigned long long ex = block_exclusive_scan<unsigned long long>(K, sc, &tot);
        if (i < ab.L) ab.offsets_out[i] = carry + ex;
        carry += tot;
    }
    if (tid == 0) ab.offsets_out[ab.L] = carry;
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
