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
// possible in a caller-supplied table) are kept as single candidates.  Candidates from the first
// one that costs more than the capacity are dropped (costs ascend with j).
struct DpLists {
    uint32_t* wall;  // [L][J] cost in units of candidate j
    uint32_t* w;     // [L][J] cost in units of the entry
    uint32_t* jj;    // [L][J] first member of the run | last member << 8
    double* e;       // [L][J][2] error of the last member, error of the member before it (NaN for a single)
    uint32_t* n;     // [L] entries
    uint32_t* bad;   // [L] 1 if the layer's table row holds an Inf or a NaN
};

// One wave per layer, one lane per candidate.
__global__ __launch_bounds__(64) void k_dp_prep(AllocBuffers ab, DpLists dl) {
    const uint32_t i = blockIdx.x, j = threadIdx.x;
    const bool valid = j < ab.J;
    uint32_t w = 0xFFFFFFFFu;
    double e = 0.0;
    if (valid) {
        w = units_of(ab.Ktab[(size_t)i * ab.J + j], ab.unit);
        e = ab.E[(size_t)i * ab.J + j];
        dl.wall[(size_t)i * ab.J + j] = w;
    }
    const uint64_t nonfinite = ballot(valid && !(e - e == 0.0));
    const uint64_t over = ballot(valid && w > ab.cap);
    const uint32_t n_in = over ? (uint32_t)__builtin_ctzll(over) : ab.J;
    const bool in = j < n_in;
    const uint32_t wprev = __shfl_up(w, 1, 64);
    const double eprev = __shfl_up(e, 1, 64);
    const bool start = in && (j == 0 || w != wprev || !(e <= eprev));
    const uint64_t smask = ballot(start);
    const uint64_t above = j < 63 ? smask & ~((2ull << j) - 1ull) : 0ull;
    const uint32_t b = (above ? (uint32_t)__builtin_ctzll(above) : n_in) - 1u;   // last member of the run starting here
    const double e_last = __shfl(e, (int)(b & 63u), 64);
    const double e_before = __shfl(e, (int)((b - 1u) & 63u), 64);
    if (start) {
        const size_t o = (size_t)i * ab.J + (uint32_t)__builtin_popcountll(smask & ((1ull << j) - 1ull));
        dl.w[o] = w;
        dl.jj[o] = j | (b << 8);
        dl.e[2 * o] = e_last;
        dl.e[2 * o + 1] = b > j ? e_before : __longlong_as_double(0x7FF8000000000000ll);
    }
    if (j == 0) {
        dl.n[i] = (uint32_t)__builtin_popcountll(smask);
        dl.bad[i] = nonfinite ? 1u : 0u;
    }
}

// The recurrence for capacities whose rows fit LDS, in three kernels:
//   k_dp_forward  one workgroup: least totals only (a min per candidate and cell), every row also
//                 written to global memory;
//   k_dp_choice   all (layer, cell) pairs in parallel: the winning candidate, from the stored rows;
//   k_dp_walk     one workgroup: status, smallest cost attaining the least total, back-tracking, outputs.
// Only the forward kernel is a sequential chain of L steps, so it carries nothing but the minimum:
// which candidate attains it is order-independent given the previous row and is found afterwards.
//
// LDS rows are stored behind DP_PAD cells of +inf, so a candidate that costs more than the cell
// needs no test: it reads +inf and cannot win.
constexpr uint32_t DP_PAD = 3072;               // cells of +inf before cost 0; also the largest row
constexpr uint32_t DP_ROW = 2 * DP_PAD;         // doubles per LDS row
constexpr uint32_t DP_LIST_CAP = 4096;          // candidate-list entries held in LDS at a time
constexpr uint32_t DP_FWD_THREADS = 512;
constexpr uint32_t DP_GROUP_MAX = DP_FWD_THREADS;  // layers per group at most (one thread plans one layer)

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits for the
// acknowledgement of every global store in flight, which would put a memory round trip into each
// of the L sequential steps.
constexpr uint32_t DP_UNROLL = 4;

// min of two doubles, neither a signalling NaN (the builtin would add a canonicalising max per operand)
__device__ __forceinline__ double min_f64(double a, double b) {
    double r;
    asm("v_min_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Thread t owns cells t, t+512, ... (CPT of them).  A wave keeps the layer's list in registers, one
// entry per lane, and broadcasts entry k with readlane: per entry and cell the work is one LDS
// read, one add and one min.
template <int CPT>
__global__ __launch_bounds__(DP_FWD_THREADS) void k_dp_forward(AllocBuffers ab, const uint32_t* __restrict__ ent_w,
                                                               const double* __restrict__ ent_e,
                                                               const uint32_t* __restrict__ ent_n,
                                                               double* __restrict__ rows_g, uint32_t rstride) {
    __shared__ double rows[2][DP_ROW];          // 96 KB
    __shared__ double LE[DP_LIST_CAP];          // 32 KB: error of the run's last member
    __shared__ uint32_t LW[DP_LIST_CAP];        // 16 KB: cost in bytes of row (units * 8)
    __shared__ uint32_t loff[DP_GROUP_MAX + 1]; // first entry of each layer of the group
    __shared__ uint32_t su[16];
    __shared__ uint32_t sh_g;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    const uint32_t ncell = ab.cap + 1;
    for (uint32_t c = tid; c < DP_ROW; c += DP_FWD_THREADS) {
        rows[0][c] = c == DP_PAD ? 0.0 : DP_INF;
        rows[1][c] = DP_INF;
    }
    for (uint32_t c = tid; c < ncell; c += DP_FWD_THREADS) rows_g[c] = c ? DP_INF : 0.0;
    // Layers are taken in groups whose candidate lists fit the LDS list buffer; the lists of a group
    // are copied in one sweep, so the memory latency is paid once per group, not once per layer.
    uint32_t i0 = 0;
    while (i0 < ab.L) {
        const uint32_t mine = (i0 + tid < ab.L) ? ent_n[i0 + tid] : 0u;
        const uint32_t before = block_exclusive_scan<uint32_t>(mine, su, nullptr);
        if (tid == 0) sh_g = 0u;
        __syncthreads();
        const bool fits = i0 + tid < ab.L && before + mine <= DP_LIST_CAP;
        if (fits) {
            loff[tid] = before;
            atomicMax(&sh_g, tid + 1u);          // layer counts are prefix-monotone: the group is layers 0..g-1
        }
        __syncthreads();
        const uint32_t g = sh_g;                 // >= 1: one layer has at most J <= 64 entries
        if (tid == g - 1u) loff[g] = before + mine;
        __syncthreads();
        for (uint32_t t = tid; t < g * ab.J; t += DP_FWD_THREADS) {
            const uint32_t layer = t / ab.J, k = t % ab.J;
            if (k < loff[layer + 1] - loff[layer]) {
                const size_t o = (size_t)(i0 + layer) * ab.J + k;
                const uint32_t d = loff[layer] + k;
                LW[d] = ent_w[o] * 8u;
                LE[d] = ent_e[2 * o];
            }
        }
        __syncthreads();
        // The list of the next layer is fetched into registers while the current layer is computed, and
        // the bounds of the one after that: nothing but the row itself is read on the critical path.
        auto fetch_list = [&](uint32_t b0, uint32_t b1, uint32_t& fw, double& fe) {
            fw = 0u; fe = DP_INF;
            if (lane < b1 - b0) { fw = LW[b0 + lane]; fe = LE[b0 + lane]; }
        };
        uint32_t n_next = loff[1] - loff[0], vw_next;
        double ve_next;
        fetch_list(loff[0], loff[1], vw_next, ve_next);
        uint32_t b0 = loff[min(1u, g)], b1 = loff[min(2u, g)];
        for (uint32_t i = i0; i < i0 + g; ++i) {
            const char* prev = reinterpret_cast<const char*>(rows[i & 1] + DP_PAD + tid);
            double* cur = rows[(i + 1) & 1] + DP_PAD + tid;
            const uint32_t n = __builtin_amdgcn_readfirstlane(n_next);
            const uint32_t vw = vw_next;
            const double ve = ve_next;
            n_next = b1 - b0;
            fetch_list(b0, b1, vw_next, ve_next);
            b0 = loff[min(i - i0 + 2u, g)]; b1 = loff[min(i - i0 + 3u, g)];
            const int ve_lo = (int)(uint32_t)__double_as_longlong(ve), ve_hi = (int)((uint64_t)__double_as_longlong(ve) >> 32);
            double best[CPT];
#pragma unroll
            for (int m = 0; m < CPT; ++m) best[m] = DP_INF;
            // DP_UNROLL entries per trip: all their row reads are issued before the first add.  Lanes
            // past the list hold (cost 0, +inf), so a padded trip changes nothing.
            for (uint32_t k0 = 0; k0 < n; k0 += DP_UNROLL) {
                double e[DP_UNROLL], p[DP_UNROLL][CPT];
#pragma unroll
                for (int u = 0; u < (int)DP_UNROLL; ++u) {
                    const uint32_t w8 = (uint32_t)__builtin_amdgcn_readlane((int)vw, (int)(k0 + u));
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane(ve_lo, (int)(k0 + u));
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane(ve_hi, (int)(k0 + u));
                    e[u] = __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
                    const char* q = prev - w8;
#pragma unroll
                    for (int m = 0; m < CPT; ++m)
                        p[u][m] = *reinterpret_cast<const double*>(q + (size_t)m * DP_FWD_THREADS * 8u);
                }
#pragma unroll
                for (int u = 0; u < (int)DP_UNROLL; ++u) {
#pragma unroll
                    for (int m = 0; m < CPT; ++m) best[m] = min_f64(best[m], p[u][m] + e[u]);
                }
            }
            double* out = rows_g + (size_t)(i + 1) * rstride + tid;
#pragma unroll
            for (int m = 0; m < CPT; ++m) {
                cur[m * DP_FWD_THREADS] = best[m];
                if (tid + m * DP_FWD_THREADS < ncell) out[m * DP_FWD_THREADS] = best[m];
            }
            lds_barrier();
        }
        i0 += g;
    }
}

// Winning candidate of every (layer, cell): candidates in list order with a strict "<", then the
// lowest member of the winner's run whose rounded total is the same.
__global__ __launch_bounds__(256) void k_dp_choice(AllocBuffers ab, DpLists dl, const double* __restrict__ rows_g,
                                                   uint32_t rstride) {
    __shared__ uint32_t lw[KIMAD_MAX_J_CONST], lj[KIMAD_MAX_J_CONST];
    __shared__ double le[2 * KIMAD_MAX_J_CONST];
    const uint32_t i = blockIdx.y, tid = threadIdx.x;
    const uint32_t n = dl.n[i];
    if (tid < n) {
        const size_t o = (size_t)i * ab.J + tid;
        lw[tid] = dl.w[o]; lj[tid] = dl.jj[o];
        le[2 * tid] = dl.e[2 * o]; le[2 * tid + 1] = dl.e[2 * o + 1];
    }
    __syncthreads();
    const uint32_t c = blockIdx.x * 256u + tid;
    if (c > ab.cap) return;
    const double* prev = rows_g + (size_t)i * rstride;
    double best = DP_INF;
    uint32_t bk = 0xFFu;
    for (uint32_t k = 0; k < n; ++k) {
        const uint32_t w = lw[k];
        if (w > c) break;                          // costs ascend along the list
        const double t = prev[c - w] + le[2 * k];
        if (t < best) { best = t; bk = k; }
    }
    uint32_t bj = 0xFFu;
    if (bk != 0xFFu) {
        // Only the winner's run matters: if the member before its last one rounds to the same total
        // (never for a single: that error is NaN), the lowest such member wins.
        bj = lj[bk] >> 8;
        const double p = prev[c - lw[bk]];
        if (p + le[2 * bk + 1] == best) {
            const uint32_t jlo = lj[bk] & 0xFFu;
            uint32_t j = bj - 1u;
            while (j > jlo && p + ab.E[(size_t)i * ab.J + j - 1] == best) --j;
            bj = j;
        }
    }
    ab.choice[(size_t)i * ab.stride + c] = (uint8_t)bj;
}

constexpr uint32_t DP_STAGE_BYTES = 128u * 1024u;

__global__ __launch_bounds__(1024) void k_dp_walk(AllocBuffers ab, const double* __restrict__ last,
                                                  const uint32_t* __restrict__ wall, const uint32_t* __restrict__ bad,
                                                  int32_t err_infeasible, int32_t err_nonfinite) {
    __shared__ __attribute__((aligned(16))) uint8_t stage[DP_STAGE_BYTES];
    __shared__ double sv[16];
    __shared__ unsigned long long sc[16];
    __shared__ unsigned long long cstar;
    __shared__ uint32_t any_bad;
    __shared__ int32_t st;
    const uint32_t tid = threadIdx.x;
    const uint32_t ncell = ab.cap + 1;
    if (tid == 0) any_bad = 0u;
    __syncthreads();
    uint32_t mybad = 0;
    for (uint32_t i = tid; i < ab.L; i += 1024) mybad |= bad[i];
    if (mybad) atomicOr(&any_bad, 1u);
    // least total, smallest cost attaining it
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
        if (any_bad) s = err_nonfinite;
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
    const uint32_t wbytes = 4u * ab.J;
    const uint32_t per_layer = (ncell + wbytes + 3u) & ~3u;
    const uint32_t per_group = DP_STAGE_BYTES / per_layer;
    uint32_t hi = ab.L;
    while (hi > 0) {
        const uint32_t lo_l = hi > per_group ? hi - per_group : 0u;
        __syncthreads();
        // one wave per layer row, four cells per lane and trip (rows start on 4-byte boundaries)
        for (uint32_t i = tid >> 6; i < hi - lo_l; i += 16) {
            const uint32_t* src = reinterpret_cast<const uint32_t*>(ab.choice + (size_t)(lo_l + i) * ab.stride);
            uint32_t* dst = reinterpret_cast<uint32_t*>(stage + i * per_layer + wbytes);
            for (uint32_t x = tid & 63u; x < (ncell + 3u) / 4u; x += 64) dst[x] = src[x];
            uint32_t* dw = reinterpret_cast<uint32_t*>(stage + i * per_layer);
            for (uint32_t j = tid & 63u; j < ab.J; j += 64) dw[j] = wall[(size_t)(lo_l + i) * ab.J + j];
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
