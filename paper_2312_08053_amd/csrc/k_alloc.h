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
    const uint32_t* Ktab;    // [L][J] pairs charged for candidate j (its size, or the dense size where that is cheaper)
    const uint32_t* Kout;    // [L][J] size sent for candidate j (Ktab itself without the dense fallback)
    uint32_t L, J;
    uint64_t unit;           // cost unit in pairs
    uint32_t cap;            // capacity in units
    double* row0;            // [cap+1]
    double* row1;            // [cap+1]
    uint8_t* choice;         // [L][stride]
    uint16_t* cprev;         // [L][stride] rows that fit LDS only: the cell the winning candidate came from
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

// Dense fallback: a layer never costs more than its bare values (n * 4 bytes), so a grid point at or beyond the
// break-even K * pair_bytes >= 4 n stands for sending the layer whole: error 0, K = n, charged
// ceil(4 n / pair_bytes) pairs (the levelling off at the uncompressed size of the paper's Section 4.2).
__global__ __launch_bounds__(256) void k_dense_view(const double* E, const uint32_t* Ktab, const LayerDesc* layers, uint32_t L,
                                                    uint32_t J, uint32_t pair_bytes, double* E_eff, uint32_t* Kcost,
                                                    uint32_t* Kout) {
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    if (t >= L * J) return;
    const uint64_t n = layers[t / J].n, K = Ktab[t];
    const bool dense = K * pair_bytes >= n * 4ull;
    E_eff[t] = dense ? 0.0 : E[t];
    Kcost[t] = dense ? (uint32_t)((n * 4ull + pair_bytes - 1u) / pair_bytes) : (uint32_t)K;
    Kout[t] = dense ? (uint32_t)n : (uint32_t)K;
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
    // candidates in ascending j with a strict "<", sixteen row reads asked for at a time (a candidate that
    // costs more than the cell reads cell 0 instead and is skipped; costs ascend with j)
    constexpr int BATCH = 16;
    for (uint32_t j0 = 0; j0 < ab.J; j0 += BATCH) {
        if (sW[j0] > c) break;
        double p[BATCH];
        uint32_t w[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            w[u] = j0 + (uint32_t)u < ab.J ? sW[j0 + u] : 0xFFFFFFFFu;
            p[u] = prev[w[u] <= c ? c - w[u] : 0];
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            if (w[u] > c) continue;
            const double t = p[u] + sE[j0 + u];
            if (t < best) { best = t; bj = j0 + (uint32_t)u; }
        }
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
// Two LDS shapes: rows of up to 3072 cells beside 3072 list records, or rows of up to 4224 cells (a
// discretisation factor of 4096 fits) beside 1024 records, i.e. more groups of fewer layers.
constexpr uint32_t DP_PAD = 3072;               // cells of +inf before cost 0; also the largest row of the first shape
constexpr uint32_t DP_LIST_CAP = 3072;          // list records held in LDS at a time, first shape
constexpr uint32_t DP_PAD_WIDE = 4224;          // the same for the second shape
constexpr uint32_t DP_LIST_CAP_WIDE = 1024;

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

// A wave holds 16 list records per register set, record k in lane k of every 16-lane row, and
// uses them through DPP row_newbcast operands, which hand lane K of each row to all its lanes:
//   row_addr_sub4  LDS address of the row cell minus record K's cost (v_add_u32 with the negated cost)
//   acc_rec_error4 t += record K's error, as fma(error, 1.0, t): one rounding of the exact sum, the same
//                  result as an add
// Both forms were checked against a 64-lane test pattern on gfx950, four records per call.  They
// are written as inline assembly: when the compiler folds a DPP move into a subtraction itself, the instruction it emits
// applied the broadcast to the other operand in that test.  Each waits two cycles first: a DPP
// operand must not be read directly after the vector instruction that wrote it, and the compiler
// does not know that the assembly reads through DPP.
template <int K>
__device__ __forceinline__ void row_addr_sub4(uint32_t base, uint32_t neg_cost, uint32_t (&q)[4]) {
    asm("s_nop 1\n\t"
        "v_add_u32_dpp %0, %4, %5 row_newbcast:%6 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_u32_dpp %1, %4, %5 row_newbcast:%7 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_u32_dpp %2, %4, %5 row_newbcast:%8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_add_u32_dpp %3, %4, %5 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1"
        : "=&v"(q[0]), "=&v"(q[1]), "=&v"(q[2]), "=&v"(q[3])
        : "v"(neg_cost), "v"(base), "n"(K), "n"(K + 1), "n"(K + 2), "n"(K + 3));
}
// t[u] += error of record K+u, four records at once (one wait for all of them)
template <int K>
__device__ __forceinline__ void acc_rec_error4(double (&t)[4], double err, double one) {
    asm("s_nop 1\n\t"
        "v_fmac_f64_dpp %0, %4, %5 row_newbcast:%6 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_fmac_f64_dpp %1, %4, %5 row_newbcast:%7 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_fmac_f64_dpp %2, %4, %5 row_newbcast:%8 row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "v_fmac_f64_dpp %3, %4, %5 row_newbcast:%9 row_mask:0xf bank_mask:0xf bound_ctrl:1"
        : "+v"(t[0]), "+v"(t[1]), "+v"(t[2]), "+v"(t[3])
        : "v"(err), "v"(one), "n"(K), "n"(K + 1), "n"(K + 2), "n"(K + 3));
}

// LDS pointers as 32-bit byte addresses, for address arithmetic in DPP instructions.
using lds_cdouble_ptr = const __attribute__((address_space(3))) double*;
__device__ __forceinline__ uint32_t lds_addr(const double* p) { return (uint32_t)(size_t)(lds_cdouble_ptr)p; }

// A list record as stored in LDS: x, y = the error's fp64 bits, z = minus the cost as a byte
// distance in the row.
__device__ __forceinline__ double rec_err(const uint4& r) { return __hiloint2double((int)r.y, (int)r.x); }

// One trip of the recurrence covers records 4*K4 .. 4*K4+3 of a block of 16: dp_issue starts its
// row reads, dp_consume does its arithmetic.  (Issuing trip t+1 before consuming trip t was tried
// and measured no faster: a wave issues an instruction every 8 to 10 cycles whatever it waits for,
// and the trip is bound by its instruction count.)
template <int NT, int CPT, int K4>
__device__ __forceinline__ void dp_issue(uint32_t neg_cost, uint32_t prev, double (&p)[4][CPT]) {
    constexpr int K = 4 * K4;
    uint32_t q[4];
    row_addr_sub4<K>(prev, neg_cost, q);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
#pragma unroll
        for (int m = 0; m < CPT; ++m)
            p[u][m] = *(lds_cdouble_ptr)(uintptr_t)(q[u] + (uint32_t)m * NT * 8u);
    }
}

template <int CPT, int K4>
__device__ __forceinline__ void dp_consume(const double (&p)[4][CPT], double err, double one, double (&best)[CPT]) {
    constexpr int K = 4 * K4;
#pragma unroll
    for (int m = 0; m < CPT; ++m) {
        double t[4] = {p[0][m], p[1][m], p[2][m], p[3][m]};
        acc_rec_error4<K>(t, err, one);
        best[m] = min_f64(min_f64(best[m], t[0]), min_f64(t[1], min_f64(t[2], t[3])));
    }
}

// Thread t owns cells t, t+NT, ... (CPT of them).  The lists of a group of layers sit in LDS as one
// stream of 16-byte records, each layer padded to a multiple of DP_UNROLL with records (cost 0,
// +inf) that change nothing.  A wave holds a layer's records in registers, record k of a block of
// 16 in lane k of every 16-lane row, and hands record k to all lanes with a DPP row broadcast
// (a readlane or a broadcast LDS read per record and wave costs several times the arithmetic).
// Per record and cell the work is one LDS read, one add and one min.  The records of the next
// layer are fetched while the current one is computed.
template <int NT, int CPT, uint32_t PAD = DP_PAD, uint32_t LCAP = DP_LIST_CAP>
__global__ __launch_bounds__(NT) void k_dp_forward(AllocBuffers ab, const uint32_t* __restrict__ ent_w,
                                                               const double* __restrict__ ent_e,
                                                               const uint32_t* __restrict__ ent_n,
                                                               double* __restrict__ rows_g, uint32_t rstride) {
    __shared__ double rows[2][2 * PAD];                 // 96 KB (132 KB in the wide shape)
    __shared__ uint4 recs[LCAP + 64];                   // 49 KB (17 KB); a layer's fetch may run 63 records past its list
    __shared__ uint32_t loff[NT + 1];         // first record of each layer of the group
    __shared__ uint32_t ln[NT];               // entries of each layer before padding
    __shared__ uint32_t ltr[NT + 1];          // trips of each layer; 0 after the last
    __shared__ uint32_t su[16];
    __shared__ uint32_t sh_g;
    const uint32_t tid = threadIdx.x;
    const uint32_t ncell = ab.cap + 1;
    for (uint32_t c = tid; c < 2 * PAD; c += NT) {
        rows[0][c] = c == PAD ? 0.0 : DP_INF;
        rows[1][c] = DP_INF;
    }
    for (uint32_t c = tid; c < ncell; c += NT) rows_g[c] = c ? DP_INF : 0.0;
    // Layers are taken in groups whose candidate lists fit the LDS list buffer; the lists of a group
    // are copied in one sweep, so the memory latency is paid once per group, not once per layer.
    uint32_t i0 = 0;
    while (i0 < ab.L) {
        const uint32_t n_mine = (i0 + tid < ab.L) ? ent_n[i0 + tid] : 0u;
        const uint32_t mine = (n_mine + DP_UNROLL - 1u) & ~(DP_UNROLL - 1u);
        const uint32_t before = block_exclusive_scan<uint32_t>(mine, su, nullptr);
        if (tid == 0) sh_g = 0u;
        __syncthreads();
        const bool fits = i0 + tid < ab.L && before + mine <= LCAP;
        if (fits) {
            loff[tid] = before;
            ln[tid] = n_mine;
            atomicMax(&sh_g, tid + 1u);          // layer counts are prefix-monotone: the group is layers 0..g-1
        }
        __syncthreads();
        const uint32_t g = sh_g;                 // >= 1: one layer has at most J <= 64 entries
        if (tid == g - 1u) loff[g] = before + mine;
        __syncthreads();
        // Lane k of a wave copies record k (a padded list has at most 64 of them) of one layer at a time,
        // four layers per trip with their loads issued together: the copy costs a few memory round trips,
        // not one per layer.  Idle positions read entry 0 of the table (a valid address) and drop it.
        static_assert(KIMAD_MAX_J_CONST == 64, "one lane per list record");
        {
            const uint32_t k = tid & 63u;
            constexpr uint32_t LSTEP = NT / 64;              // layers one trip of the workgroup covers
            for (uint32_t l0 = tid >> 6; l0 < g; l0 += 4u * LSTEP) {
                uint32_t at[4], w8[4];
                double e[4];
                bool act[4], real[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t layer = l0 + (uint32_t)u * LSTEP;
                    const bool in = layer < g;
                    const uint32_t first = in ? loff[layer] : 0u;
                    act[u] = in && k < loff[layer + 1] - first;
                    real[u] = act[u] && k < ln[layer];
                    at[u] = first + k;
                    const size_t o = real[u] ? (size_t)(i0 + layer) * ab.J + k : 0;
                    e[u] = ent_e[2 * o];
                    w8[u] = ent_w[o];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (!act[u]) continue;
                    const double ee = real[u] ? e[u] : DP_INF;
                    const uint32_t ww = real[u] ? w8[u] * 8u : 0u;
                    recs[at[u]] = make_uint4((uint32_t)__double2loint(ee), (uint32_t)__double2hiint(ee), 0u - ww, 0u);
                }
            }
        }
        // a layer's fetch and the row reads issued one trip ahead may run past the group's last
        // record: what they find there is (cost 0, +inf) as well
        if (tid < 64) recs[loff[g] + tid] = make_uint4(0u, 0x7FF00000u, 0u, 0u);
        for (uint32_t l = tid; l <= g; l += NT) ltr[l] = l < g ? (loff[l + 1] - loff[l]) / DP_UNROLL : 0u;
        __syncthreads();

        // The stream is contiguous, so the first record of the next layer follows from the trip
        // counts alone: its records are fetched while the current layer is computed, and the trip
        // counts are read two layers ahead, which keeps every list access off the critical path.
        const uint32_t sub = tid & 15u;
        auto fetch_layer = [&](uint32_t first, uint4 (&R)[4]) {
#pragma unroll
            for (int b = 0; b < 4; ++b) R[b] = recs[first + 16u * b + sub];
        };
        double one = 1.0;
        asm volatile("" : "+v"(one));          // keep 1.0 in a vector register pair
        uint4 Rn[4];
        fetch_layer(0u, Rn);
        uint32_t first = 0u;
        uint32_t nt_cur = __builtin_amdgcn_readfirstlane(ltr[0]);
        uint32_t nt_n1 = __builtin_amdgcn_readfirstlane(ltr[min(1u, g)]);
        uint32_t nt_n2 = ltr[min(2u, g)];
        double* out = rows_g + (size_t)i0 * rstride + tid;
        for (uint32_t i = i0; i < i0 + g; ++i) {
            // LDS byte address of this thread's first cell in the previous row
            const uint32_t prev = lds_addr(rows[i & 1] + PAD + tid);
            double* cur = rows[(i + 1) & 1] + PAD + tid;
            const uint32_t nt = nt_cur;
            const uint4 R0 = Rn[0], R1 = Rn[1], R2 = Rn[2], R3 = Rn[3];
            first += DP_UNROLL * nt;
            fetch_layer(first, Rn);
            nt_cur = nt_n1;
            nt_n1 = __builtin_amdgcn_readfirstlane(nt_n2);
            nt_n2 = ltr[min(i - i0 + 3u, g)];
            double best[CPT];
#pragma unroll
            for (int m = 0; m < CPT; ++m) best[m] = DP_INF;
            // trips in blocks of four: one register set of records per block
            if (nt) {
                uint4 Q0 = R0, Q1 = R1, Q2 = R2, Q3 = R3;
                uint32_t rem = nt;
                double p[4][CPT];
                for (;;) {
                    const double err = rec_err(Q0);
                    dp_issue<NT, CPT, 0>(Q0.z, prev, p);
                    dp_consume<CPT, 0>(p, err, one, best);
                    if (rem == 1) break;
                    dp_issue<NT, CPT, 1>(Q0.z, prev, p);
                    dp_consume<CPT, 1>(p, err, one, best);
                    if (rem == 2) break;
                    dp_issue<NT, CPT, 2>(Q0.z, prev, p);
                    dp_consume<CPT, 2>(p, err, one, best);
                    if (rem == 3) break;
                    dp_issue<NT, CPT, 3>(Q0.z, prev, p);
                    dp_consume<CPT, 3>(p, err, one, best);
                    if (rem == 4) break;
                    rem -= 4u;
                    Q0 = Q1; Q1 = Q2; Q2 = Q3;
                }
            }
            out += rstride;                      // row i + 1; a stored row holds NT * CPT cells, so no cell is tested
#pragma unroll
            for (int m = 0; m < CPT; ++m) {
                // (the last sweep of the wide shape runs past the row: those cells exist in the stored row only)
                if ((uint32_t)(m + 1) * NT <= PAD || tid + (uint32_t)m * NT < PAD) cur[m * NT] = best[m];
                out[m * NT] = best[m];
            }
            lds_barrier();
        }
        __syncthreads();                         // the next group overwrites the records
        i0 += g;
    }
}

// Winning candidate of every (layer, cell): candidates in list order with a strict "<", then the
// lowest member of the winner's run whose rounded total is the same.
__global__ __launch_bounds__(256) void k_dp_choice(AllocBuffers ab, DpLists dl, const double* __restrict__ rows_g,
                                                   uint32_t rstride) {
    __shared__ uint32_t lw[KIMAD_MAX_J_CONST], lj[KIMAD_MAX_J_CONST];
    __shared__ double le[2 * KIMAD_MAX_J_CONST];
    __shared__ double prev[DP_PAD_WIDE];       // the previous row up to this workgroup's last cell
    const uint32_t i = blockIdx.y, tid = threadIdx.x;
    const uint32_t n = dl.n[i];
    if (tid < n) {
        const size_t o = (size_t)i * ab.J + tid;
        lw[tid] = dl.w[o]; lj[tid] = dl.jj[o];
        le[2 * tid] = dl.e[2 * o]; le[2 * tid + 1] = dl.e[2 * o + 1];
    }
    // every candidate of a cell reads one cell of the previous row: from LDS, not one dependent
    // memory round trip per candidate
    {
        const double* prow = rows_g + (size_t)i * rstride;
        const uint32_t upto = min(blockIdx.x * 256u + 256u, ab.cap + 1u);
        for (uint32_t x = tid; x < upto; x += 256u) prev[x] = prow[x];
    }
    __syncthreads();
    const uint32_t c = blockIdx.x * 256u + tid;
    if (c > ab.cap) return;
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
    ab.cprev[(size_t)i * ab.stride + c] = bk != 0xFFu ? (uint16_t)(c - lw[bk]) : (uint16_t)0xFFFFu;
}

constexpr uint32_t DP_STAGE_BYTES = 128u * 1024u;
constexpr uint32_t DP_WALK_MAX_L = 4224;           // layers whose path cells k_dp_walk keeps in LDS: every layer costs at least one
                                                   // cell, so a feasible path through rows of at most 4224 cells has no more layers

__global__ __launch_bounds__(1024) void k_dp_walk(AllocBuffers ab, const double* __restrict__ last,
                                                  const uint32_t* __restrict__ bad,
                                                  int32_t err_infeasible, int32_t err_nonfinite) {
    __shared__ __attribute__((aligned(16))) uint8_t stage[DP_STAGE_BYTES];
    __shared__ uint16_t s_cell[DP_WALK_MAX_L];     // the path's cell per layer (a store to memory in the chain would be waited for)
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
        else if (!(best < DP_INF) || ab.L > DP_WALK_MAX_L) s = err_infeasible;   // (more layers than cells: no finite total)
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
    // Back-tracking.  The sequential part follows only the chain of cells: k_dp_choice stored, beside
    // every winner, the cell it came from, so a step is one LDS read.  The rows of a group of layers
    // are staged in LDS with one flat copy (they are contiguous, pitch a multiple of 16 bytes), walked
    // by one thread that notes each layer's cell, next group.  The winners are then looked up in parallel.
    const uint32_t pitch = (uint32_t)ab.stride;                      // cells per row
    const uint32_t per_group = DP_STAGE_BYTES / (2u * pitch);
    const uint16_t* srow = reinterpret_cast<const uint16_t*>(stage);
    uint32_t hi = ab.L;
    while (hi > 0) {
        const uint32_t lo_l = hi > per_group ? hi - per_group : 0u;
        const uint32_t nrows = hi - lo_l;
        __syncthreads();
        {
            const uint4* src = reinterpret_cast<const uint4*>(ab.cprev + (size_t)lo_l * pitch);
            uint4* dst = reinterpret_cast<uint4*>(stage);
            const uint32_t n16 = nrows * (pitch / 8u);
            for (uint32_t x0 = 0; x0 < n16; x0 += 8u * 1024u) {
                uint4 v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t x = x0 + k * 1024u + tid;
                    v[k] = x < n16 ? src[x] : make_uint4(0u, 0u, 0u, 0u);
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const uint32_t x = x0 + k * 1024u + tid;
                    if (x < n16) dst[x] = v[k];
                }
            }
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t c = (uint32_t)cstar;
            const uint16_t* row = srow + (size_t)nrows * pitch;
            for (uint32_t i = hi; i-- > lo_l;) {
                row -= pitch;
                s_cell[i] = (uint16_t)c;
                c = min((uint32_t)row[c], ab.cap);         // (a feasible path never meets the 0xFFFF of an empty cell)
            }
            cstar = c;
        }
        hi = lo_l;
    }
    __syncthreads();
    // winners along the path, sizes and offsets, in parallel
    unsigned long long carry = 0;
    for (uint32_t i0b = 0; i0b < ab.L; i0b += 1024) {
        const uint32_t i = i0b + tid;
        unsigned long long K = 0;
        if (i < ab.L) {
            const uint32_t j = ab.choice[(size_t)i * ab.stride + (uint32_t)s_cell[i]];
            ab.j_out[i] = (int32_t)j;
            K = ab.Kout[(size_t)i * ab.J + j];
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
    // Back-tracking: one thread follows the chain of cells, one choice per layer read from memory.  The
    // candidates' costs wait in LDS (when the table fits) so that the chain holds no second memory read
    // and no division; sizes and offsets follow in parallel.
    constexpr uint32_t W_LDS = 12288;
    __shared__ uint32_t sw[W_LDS];
    const uint32_t LJ = ab.L * ab.J;
    const bool w_in_lds = LJ <= W_LDS;
    if (w_in_lds)
        for (uint32_t t = tid; t < LJ; t += 1024) sw[t] = units_of(ab.Ktab[t], ab.unit);
    __syncthreads();
    if (tid == 0) {
        uint64_t c = cstar;
        for (uint32_t i = ab.L; i-- > 0;) {
            const uint32_t j = ab.choice[(size_t)i * ab.stride + c];
            ab.j_out[i] = (int32_t)j;
            c -= w_in_lds ? sw[i * ab.J + j] : units_of(ab.Ktab[(size_t)i * ab.J + j], ab.unit);
        }
    }
    __threadfence_block();
    __syncthreads();
    unsigned long long carry = 0;
    for (uint32_t i0b = 0; i0b < ab.L; i0b += 1024) {
        const uint32_t i = i0b + tid;
        unsigned long long K = 0;
        if (i < ab.L) {
            K = ab.Kout[(size_t)i * ab.J + (uint32_t)ab.j_out[i]];
            ab.K_out[i] = K;
        }
        unsigned long long tot;
        const unsigned long long ex = block_exclusive_scan<unsigned long long>(K, sc, &tot);
        if (i < ab.L) ab.offsets_out[i] = carry + ex;
        carry += tot;
    }
    if (tid == 0) ab.offsets_out[ab.L] = carry;
}

}  // namespace kimad
