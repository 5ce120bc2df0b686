// Knapsack allocation inside a band of cost cells (paper Appendix C; Section 3.2, Eq. optimisation).
//
// The recurrence of k_alloc.h visits every cost cell of every layer although the least total runs
// through a narrow corridor of them.  Two kernels cut the work down to that corridor without
// changing one bit of the result:
//
//   k_dp_bounds  Lagrangian bounds.  For a multiplier lambda >= 0 and any assignment,
//                    sum_i E_i  >=  sum_i min_k (E_ik + lambda w_ik)  -  lambda * (sum_i w_i),
//                so a path through cell c of row r (layers 0..r-1 spent exactly c units) totals at least
//                    max_lambda [A_r(lambda) - lambda c]  +  max_lambda [B_r(lambda) - lambda (cap - c)],
//                A_r, B_r the sums of the per-layer minima over the layers before / from r.  Any feasible
//                assignment gives an upper bound UB on the least total.  A cell whose lower bound exceeds
//                UB (by a margin far above the rounding of these sums) lies on no path that attains the
//                least total, and the cells that remain form an interval of every row: its band.
//   k_dp_banded  the recurrence on the band cells only; sources outside the previous row's band count
//                as +inf.
//
// Why the result is the same.  The sequential recurrence computes, per cell, the minimum over paths of
// the path's left-to-right fp64 sum, and fp64 addition is monotone, so removing cells can only raise
// a cell's value.  Every cell of a path that attains the least total T stays in its band (its lower
// bound is at most the path's real sum <= T (1 + tiny) <= UB (1 + tiny)); by induction along such a path
// each of its cells keeps its value and its winning candidate: the first candidate, in list order,
// that attains the cell's minimum comes from a cell that is itself on such a path, so it is in the
// band with its value unchanged, and the candidates before it still do not attain the minimum.  The
// last row therefore has the same minimum at the same cells, and back-tracking meets unchanged cells only.
#pragma once
#include "common.h"
#include "k_alloc.h"

namespace kimad {

constexpr uint32_t BAND_MAX_L = 1024;          // layers the banded allocation handles
constexpr uint32_t BAND_LCAP = 7168;           // list records held in LDS by the bounds kernel
constexpr uint32_t BAND_NLAM = 32;             // multipliers around the one found: lambda* rho^(m - 16)
constexpr uint32_t BAND_NLAM_MANY = 8;         // the same for more layers than the table of 32 fits LDS for
constexpr uint32_t BAND_L_FOR_32 = 416;
constexpr uint32_t BAND_GREEDY = 16;           // rounds of the greedy fill that tightens the upper bound
constexpr uint32_t BOUNDS_THREADS = 1024;
constexpr uint32_t BAND_EDGES_PER_THREAD = BAND_LCAP / BOUNDS_THREADS;   // 7

struct BandBuffers {
    uint32_t* lo;          // [L + 1] first cell of row r's band (row 0 is the start: cell 0)
    uint32_t* hi;          // [L + 1] last cell
    uint32_t* info;        // [16] max width, sum of widths, 1 if the bands are the whole rows, upgrades taken; rest: tracing
    // the list records that can connect the bands of consecutive rows, layer after layer (the only ones the
    // banded recurrence visits): layer i's are [live_off[i], live_off[i + 1])
    uint32_t* live_off;    // [L + 1]
    double* live_e;        // [L * J] error of the run's last member
    double* live_before;   // [L * J] error of the member before it (NaN for a single)
    uint32_t* live_w;      // [L * J] cost
    uint32_t* live_jj;     // [L * J] first member | last member << 8
};

__device__ __forceinline__ double max_f64(double a, double b) {   // neither a signalling NaN (see min_f64)
    double r;
    asm("v_max_f64 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// The value of another lane inside groups of 2, 4 or 8 neighbouring lanes, through DPP moves (a shuffle goes
// through the LDS crossbar: a dependent round trip per step).
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}
// maximum over the T lanes of a group (T = 1, 2, 4, 8), in every lane of it
template <int T>
__device__ __forceinline__ double group_max(double v) {
    if (T >= 2) v = max_f64(v, dpp_f64<0xB1>(v));      // quad_perm [1,0,3,2]
    if (T >= 4) v = max_f64(v, dpp_f64<0x4E>(v));      // quad_perm [2,3,0,1]
    if (T >= 8) v = max_f64(v, dpp_f64<0x141>(v));     // row_half_mirror: the other quad of the eight
    return v;
}

// Bands of all rows: T threads a row, PT multipliers each (T * PT = the number of multipliers).  Returns the
// sum of the widths of the rows whose first lane this thread is.
template <int T, int PT>
__device__ __forceinline__ uint32_t band_rows(const double* AT, uint32_t pitch, const double* s_lam, const double* s_btot,
                                              const uint16_t* s_cum, uint16_t* s_blo, uint16_t* s_bhi, const BandBuffers& bb,
                                              uint32_t L, uint32_t cap, double ub_m) {
    const uint32_t tid = threadIdx.x;
    uint32_t width = 0u;
    for (uint32_t r_base = 1u; r_base <= L; r_base += BOUNDS_THREADS / T) {
        const uint32_t r = r_base + tid / T, part = tid % T;
        const bool live_row = r <= L;
        const uint32_t rr = live_row ? r : L;      // (lanes past the last row repeat it: a group's lanes stay together)
        double a[PT], lm[PT], bt[PT];
#pragma unroll
        for (int u = 0; u < PT; ++u) {
            const uint32_t m = part + (uint32_t)u * T;
            a[u] = AT[(size_t)rr * pitch + m]; lm[u] = s_lam[m]; bt[u] = s_btot[m] - a[u];
        }
        auto within = [&](uint32_t c) {
            const double cd = (double)c, rd = (double)(cap - c);
            double pre = a[0] - lm[0] * cd, suf = bt[0] - lm[0] * rd;
#pragma unroll
            for (int u = 1; u < PT; ++u) {
                pre = max_f64(pre, a[u] - lm[u] * cd);
                suf = max_f64(suf, bt[u] - lm[u] * rd);
            }
            return group_max<T>(pre) + group_max<T>(suf) <= ub_m;
        };
        // One search per edge: towards cell 0, then towards the last cell.  Steps of 8, 32, 128, ... away from the
        // assignment's own cell until a probe falls outside (or the row's end is inside), then bisection between
        // the last cell inside and the first outside.
        const uint32_t on_path = s_cum[rr];
        uint32_t edge[2];
#pragma unroll 1
        for (int side = 0; side < 2; ++side) {
            const uint32_t room = side ? cap - on_path : on_path;  // cells between the path and the row's end
            uint32_t in = 0u, out = room + 1u;                      // distances from the path: `in` inside, `out` outside (room + 1: beyond the row)
            uint32_t stepd = 8u;
            while (out - in > 1u) {
                uint32_t probe;
                if (out == room + 1u) { probe = min(in + stepd, room); stepd *= 4u; }
                else probe = in + (out - in) / 2u;
                const uint32_t c = side ? on_path + probe : on_path - probe;
                if (within(c)) { in = probe; if (probe == room) break; }
                else out = probe;
            }
            edge[side] = side ? on_path + in : on_path - in;
        }
        if (live_row && part == 0u) {
            bb.lo[r] = edge[0]; bb.hi[r] = edge[1];
            s_blo[r] = (uint16_t)edge[0]; s_bhi[r] = (uint16_t)edge[1];
            width += edge[1] - edge[0] + 1u;
        }
    }
    return width;
}

// Bounds kernel: one workgroup of sixteen waves.
//   1  the lists go to LDS; per layer (one thread each) the lower convex hull of its (cost, error) points is
//      built in place: only hull vertices can minimise E + lambda w, and along the hull the slopes
//      (error saved per unit of cost) fall, so a layer's minimiser for a given lambda is found by bisection.
//      (A vertex dropped or kept by a rounding of the hull test changes such a minimum by rounding only, far
//      inside the margin below.)
//   2  the smallest lambda whose minimisers fit the capacity: the total cost at lambda is that of the cheapest
//      vertices plus the cost steps of all hull edges steeper than lambda; every thread keeps a few edges in
//      registers and the bit pattern of lambda (ordered like the doubles) is bisected;
//   3  upper bound: that assignment, then up to BAND_GREEDY single steps to a next hull vertex, steepest edge
//      that still fits first;
//   4  the table A[r][m] = sum over layers before r of the minimum at lambda_m, in LDS over the hulls;
//   5  the band of every row by a search outward from the assignment's own cell;
//   6  the live records of every layer, written out for the recurrence.
__global__ __launch_bounds__(BOUNDS_THREADS) void k_dp_bounds(AllocBuffers ab, DpLists dl, BandBuffers bb) {
    constexpr uint32_t NWAVES = BOUNDS_THREADS / 64;
    __shared__ __align__(16) unsigned char pool[BAND_LCAP * 18];        // 126 KB: hulls (HE, HS, HW), later the table A
    __shared__ uint16_t raw_w[BAND_LCAP];                               // 14 KB: the lists' costs as they came
    __shared__ uint16_t s_n[BAND_MAX_L], s_off[BAND_MAX_L], s_hn[BAND_MAX_L], s_q[BAND_MAX_L];
    __shared__ uint16_t s_cum[BAND_MAX_L + 2], s_blo[BAND_MAX_L + 2], s_bhi[BAND_MAX_L + 2];
    __shared__ uint32_t su[16];
    __shared__ double sd[16];
    __shared__ double s_lam[BAND_NLAM], s_btot[BAND_NLAM];
    __shared__ unsigned long long s_key[2];
    __shared__ uint32_t s_hist[2][64], s_dw[2];
    __shared__ uint32_t s_flag, s_wmax;
    double* const HE = reinterpret_cast<double*>(pool);                 // vertex errors
    double* const HS = HE + BAND_LCAP;                                  // slope of the edge to the next vertex; 0 where there is none
    uint16_t* const HW = reinterpret_cast<uint16_t*>(HS + BAND_LCAP);   // vertex costs (rows that fit LDS: below 65536)
    double* const AT = reinterpret_cast<double*>(pool);                 // [(L + 1)][nl + 1], once the hulls are done with
    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t L = ab.L, J = ab.J, cap = ab.cap;
#ifdef KIMAD_STAMPS
    unsigned long long stamp[10]; int ns = 0;
#define STAMP() do { stamp[ns++] = __builtin_readcyclecounter(); } while (0)
#else
#define STAMP() do {} while (0)
#endif
    STAMP();

    // ---- 1: sizes, offsets, lists into LDS
    const uint32_t my_n = tid < L ? min(dl.n[tid], 64u) : 0u;
    const uint32_t my_bad = tid < L ? (dl.bad[tid] | (my_n == 0u ? 1u : 0u)) : 0u;    // or a layer with no affordable candidate
    uint32_t n_tot;
    const uint32_t my_off = block_exclusive_scan<uint32_t>(my_n, su, &n_tot);
    if (tid == 0) { s_flag = 0u; s_key[0] = 0ull; s_key[1] = 0ull; s_wmax = 0u; }
    if (tid < 128u) s_hist[tid >> 6][tid & 63u] = 0u;
    __syncthreads();
    if (my_bad) s_flag = 1u;
    bool whole = n_tot > BAND_LCAP;
    if (tid < L && !whole) { s_n[tid] = (uint16_t)my_n; s_off[tid] = (uint16_t)my_off; }
    __syncthreads();
    whole = whole || s_flag != 0u;
    if (!whole) {
        for (uint32_t x = tid; x < BAND_LCAP; x += BOUNDS_THREADS) HS[x] = 0.0;
        // four layers' loads in flight per wave
        for (uint32_t i0 = wave * 4u; i0 < L; i0 += NWAVES * 4u) {
            double e[4];
            uint32_t w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t i = i0 + (uint32_t)u;
                const bool in = i < L && lane < s_n[min(i, L - 1u)];
                const size_t o = in ? (size_t)i * J + lane : 0;
                e[u] = dl.e[2 * o]; w[u] = dl.w[o];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t i = i0 + (uint32_t)u;
                if (i < L && lane < s_n[i]) { HE[s_off[i] + lane] = e[u]; HW[s_off[i] + lane] = (uint16_t)w[u]; raw_w[s_off[i] + lane] = (uint16_t)w[u]; }
            }
        }
    }
    __syncthreads();
    STAMP();
    // lower hull, in place, one thread per layer (the vertex count never exceeds the entries read); entries are
    // read four at a time
    double my_first_abs = 0.0;
    if (!whole && tid < L) {
        const uint32_t o = my_off;
        uint32_t hn = 0u;
        double te = 0.0, pe = 0.0;                       // top vertex and the one below it
        uint32_t tw = 0u, pw = 0u;
        for (uint32_t k0 = 0; k0 < my_n; k0 += 4u) {
            double e4[4];
            uint32_t w4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) { const uint32_t k = min(k0 + (uint32_t)u, my_n - 1u); e4[u] = HE[o + k]; w4[u] = HW[o + k]; }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (k0 + (uint32_t)u >= my_n) break;
                const double e = e4[u];
                const uint32_t w = w4[u];
                if (hn == 0u) { HE[o] = e; HW[o] = (uint16_t)w; hn = 1u; te = e; tw = w; my_first_abs = fabs(e); continue; }
                if (!(e < te)) continue;                      // costs no less, saves nothing: never a minimiser
                if (w == tw) { --hn; if (hn) { te = pe; tw = pw; if (hn >= 2u) { pe = HE[o + hn - 2u]; pw = HW[o + hn - 2u]; } } }
                // pop while the slope into the top is not above the slope out of it: (pe - te)(w - tw) <= (te - e)(tw - pw)
                while (hn >= 2u && (pe - te) * (double)(w - tw) <= (te - e) * (double)(tw - pw)) {
                    --hn; te = pe; tw = pw;
                    if (hn >= 2u) { pe = HE[o + hn - 2u]; pw = HW[o + hn - 2u]; }
                }
                if (hn == 0u) my_first_abs = fmax(my_first_abs, fabs(e));
                HE[o + hn] = e; HW[o + hn] = (uint16_t)w;
                pe = te; pw = tw; te = e; tw = w; ++hn;
            }
        }
        s_hn[tid] = (uint16_t)hn;
        my_first_abs = fmax(my_first_abs, fabs(te));
    }
    __syncthreads();
    if (!whole) {
        for (uint32_t i = wave; i < L; i += NWAVES) {
            const uint32_t hn = s_hn[i], o = s_off[i];
            if (lane + 1u < hn)
                HS[o + lane] = (HE[o + lane] - HE[o + lane + 1u]) / (double)((uint32_t)HW[o + lane + 1u] - (uint32_t)HW[o + lane]);
        }
    }
    __syncthreads();
    STAMP();
    // the vertex of layer i that minimises E + lam w: the number of its edges steeper than lam
    auto vertex_at = [&](uint32_t i, double lam) {
        const uint32_t o = s_off[i];
        uint32_t lo = 0u, hi = (uint32_t)s_hn[i] - 1u;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (HS[o + mid] > lam) lo = mid + 1u; else hi = mid;
        }
        return lo;
    };

    // ---- 2: the smallest multiplier that fits.  This thread's edges (slope, cost step) stay in registers.
    unsigned long long lo_b = 0ull, hi_b = 0ull;
    uint32_t room = 0u;
    if (!whole) {
        double sl[BAND_EDGES_PER_THREAD];
        uint32_t dw[BAND_EDGES_PER_THREAD];
        double steep = 0.0;
#pragma unroll
        for (int u = 0; u < (int)BAND_EDGES_PER_THREAD; ++u) {
            const uint32_t x = tid + (uint32_t)u * BOUNDS_THREADS;
            sl[u] = HS[x];
            dw[u] = sl[u] > 0.0 ? (uint32_t)HW[x + 1u] - (uint32_t)HW[x] : 0u;     // (HS is 0 wherever x + 1 is not on the same hull)
            steep = max_f64(steep, sl[u]);
        }
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) steep = max_f64(steep, __shfl_xor(steep, d, 64));
        if (lane == 0) sd[wave] = steep;
        uint32_t cheapest;
        (void)block_exclusive_scan<uint32_t>(tid < L ? (uint32_t)HW[my_off] : 0u, su, &cheapest);   // (has barriers)
        for (uint32_t v = 0; v < NWAVES; ++v) steep = max_f64(steep, sd[v]);
        __syncthreads();
        if (cheapest > cap) whole = true;                                   // nothing fits: the recurrence will say so
        else room = cap - cheapest;
        // The smallest multiplier (as a bit pattern: non-negative doubles order like their patterns) at which the
        // edges steeper than it fit the room.  Sixty-four-way search: the patterns between lo_b (does not fit, or 0)
        // and lo_b + 2^k are cut into 64 buckets, every edge inside adds its cost step to its bucket in LDS, and
        // every wave finds for itself the lowest bucket boundary at which what lies above fits: six bits of the
        // pattern per round and two barriers, down to a gap of 2^15 patterns (2^-37 relative: closer breakpoints
        // make no difference worth a round).
        if (!whole) {
            uint32_t above = 0u;                                             // cost steps of the edges at or beyond lo_b + 2^k
            uint32_t buf = 0u;
            for (int k = 63; k > 15; k -= 6) {
                const int sh = k - 6;                                        // log2 of a bucket's size
#pragma unroll
                for (int u = 0; u < (int)BAND_EDGES_PER_THREAD; ++u) {
                    const unsigned long long bits = (unsigned long long)__double_as_longlong(sl[u]);
                    // bucket b holds the patterns in (lo_b + b 2^sh, lo_b + (b + 1) 2^sh]
                    if (dw[u] && bits > lo_b && ((bits - lo_b - 1ull) >> sh) < 64ull)
                        atomicAdd(&s_hist[buf][(uint32_t)((bits - lo_b - 1ull) >> sh)], dw[u]);
                }
                __syncthreads();
                const uint32_t mine = s_hist[buf][lane];
                s_hist[buf ^ 1u][lane] = 0u;                                 // the other table, for the next round
                const uint32_t inc = wave_scan_add_u32(mine);                // buckets 0..lane
                const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
                const uint32_t from_here = tot - inc + mine;                 // buckets lane..63
                // cost at boundary m (edges strictly above lo_b + m 2^sh) = above + buckets m..63
                const uint64_t fits = ballot(above + from_here <= room);
                // boundary 64 always fits (the invariant); the lowest fitting boundary of 0..63, if any
                const uint32_t m = fits ? (uint32_t)__ffsll((long long)fits) - 1u : 64u;
                const uint32_t keep = m < 64u ? (uint32_t)__builtin_amdgcn_readlane((int)from_here, (int)min(m, 63u)) : 0u;
                above += keep;
                hi_b = lo_b + ((unsigned long long)m << sh);
                if (m > 0u) lo_b += (unsigned long long)(m - 1u) << sh;      // boundary m - 1 does not fit
                __syncthreads();
                buf ^= 1u;
                if (m == 0u) {
                    // boundary 0 itself fits: either everything fits (lo_b = 0: the multiplier is 0) or the gap has
                    // closed onto a pattern that does not fit and its successor that does
                    break;
                }
                // the next round looks inside (boundary m - 1, boundary m], a range of 2^sh patterns
            }
            // (a first round that finds even its last boundary too low ends beyond the finite patterns: the steepest
            // slope itself always fits, nothing being steeper)
            hi_b = min(hi_b, (unsigned long long)__double_as_longlong(steep));
        }
    }
    if (whole) {
        // no bound to use: whole rows, every record live (the lists copied as they are)
        for (uint32_t r = tid; r <= L; r += BOUNDS_THREADS) { bb.lo[r] = 0u; bb.hi[r] = r ? cap : 0u; }
        if (tid < L) bb.live_off[tid] = my_off;
        if (tid == 0) bb.live_off[L] = n_tot;
        if (tid < L) {
            for (uint32_t k = 0; k < my_n; ++k) {
                const size_t o = (size_t)tid * J + k, t = my_off + k;
                bb.live_e[t] = dl.e[2 * o]; bb.live_before[t] = dl.e[2 * o + 1];
                bb.live_w[t] = dl.w[o]; bb.live_jj[t] = dl.jj[o];
            }
        }
        if (tid == 0) { bb.info[0] = cap + 1u; bb.info[1] = L * (cap + 1u); bb.info[2] = 1u; bb.info[3] = 0u; }
        return;
    }
    const double lam_star = __longlong_as_double((long long)hi_b);
    STAMP();

    // ---- 3: a feasible assignment and its total; the greedy fill names the layer to step through one LDS maximum:
    // the slope's bit pattern with the low 10 bits replaced by 1023 - layer
    if (tid < L) s_q[tid] = (uint16_t)vertex_at(tid, lam_star);
    __syncthreads();
    uint32_t used;
    (void)block_exclusive_scan<uint32_t>(tid < L ? (uint32_t)HW[my_off + s_q[tid]] : 0u, su, &used);
    uint32_t left = cap - used;                                             // used <= cap: lam_star fits
    uint32_t upgrades = 0u;
    // A round: every layer whose next hull edge fits what is left bids with its slope; the steepest wins (lowest
    // layer among equals), its owner takes the step and says what it cost.  The bids of consecutive rounds go to two
    // words in turn, so a round needs two barriers.
    for (uint32_t round = 0; round < BAND_GREEDY && left > 0u; ++round) {
        const uint32_t buf = round & 1u;
        if (tid < L) {
            const uint32_t q = s_q[tid];
            if (q + 1u < s_hn[tid] && (uint32_t)HW[my_off + q + 1u] - (uint32_t)HW[my_off + q] <= left) {
                const unsigned long long key = ((unsigned long long)__double_as_longlong(HS[my_off + q]) & ~0x3FFull) | (1023u - tid);
                atomicMax(&s_key[buf], key);
            }
        }
        __syncthreads();
        const unsigned long long best = s_key[buf];
        if (best == 0ull) break;                                             // (the same word in every thread)
        if (tid == 1023u - (uint32_t)(best & 0x3FFull)) {
            const uint32_t q = s_q[tid];
            s_dw[buf] = (uint32_t)HW[my_off + q + 1u] - (uint32_t)HW[my_off + q];
            s_q[tid] = (uint16_t)(q + 1u);
            s_key[buf ^ 1u] = 0ull;                                          // the next round's word: last read before the previous round's second barrier
        }
        __syncthreads();
        left -= s_dw[buf];
        ++upgrades;
    }
    __syncthreads();
    double ub, abs_tot;
    (void)block_exclusive_scan<double>(tid < L ? HE[my_off + s_q[tid]] : 0.0, sd, &ub);
    (void)block_exclusive_scan<double>(my_first_abs, sd, &abs_tot);        // sum over layers of the largest |error| on the hull
    {
        const uint32_t w_mine = tid < L ? (uint32_t)HW[my_off + s_q[tid]] : 0u;
        const uint32_t before = block_exclusive_scan<uint32_t>(w_mine, su, nullptr);
        if (tid < L) s_cum[tid + 1u] = (uint16_t)(before + w_mine);
        if (tid == 0) s_cum[0] = 0u;
    }
    const double ub_m = ub + 1e-9 * (fabs(ub) + abs_tot);
    STAMP();

    // ---- 4: multipliers around lam_star; per (layer, multiplier) the minimum, then prefix sums over the layers
    const uint32_t nl = L <= BAND_L_FOR_32 ? BAND_NLAM : BAND_NLAM_MANY, pitch = nl + 1u;
    if (tid < nl) {
        // (lam_star may be 0 when everything fits: the set then collapses and the bands stay wide)
        double f = 1.0;
        const int p = (int)tid - (int)(nl / 2u);
        for (int q = 0; q < (p < 0 ? -p : p); ++q) f *= 1.15;
        s_lam[tid] = p < 0 ? lam_star / f : lam_star * f;
    }
    __syncthreads();
    constexpr int PER_THREAD = (BAND_L_FOR_32 * BAND_NLAM + BOUNDS_THREADS - 1) / BOUNDS_THREADS;   // 13 (and 1024 * 8 / 1024 = 8)
    double val[PER_THREAD];
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const uint32_t x = tid + (uint32_t)u * BOUNDS_THREADS;
        val[u] = 0.0;
        if (x < L * nl) {
            const uint32_t i = x / nl, m = x % nl;
            const double lam = s_lam[m];
            const uint32_t o = s_off[i] + vertex_at(i, lam);
            val[u] = HE[o] + lam * (double)HW[o];
        }
    }
    __syncthreads();                                     // the hulls are done with: the pool becomes the table
#pragma unroll
    for (int u = 0; u < PER_THREAD; ++u) {
        const uint32_t x = tid + (uint32_t)u * BOUNDS_THREADS;
        if (x < L * nl) AT[(size_t)(x / nl + 1u) * pitch + x % nl] = val[u];
    }
    if (tid < nl) AT[tid] = 0.0;
    __syncthreads();
    if (tid < nl) {
        // one thread per multiplier runs down its column (rows are read eight ahead)
        double run = 0.0;
        uint32_t r = 1u;
        for (; r + 8u <= L + 1u; r += 8u) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = AT[(size_t)(r + (uint32_t)u) * pitch + tid];
#pragma unroll
            for (int u = 0; u < 8; ++u) { run += v[u]; AT[(size_t)(r + (uint32_t)u) * pitch + tid] = run; }
        }
        for (; r <= L; ++r) { run += AT[(size_t)r * pitch + tid]; AT[(size_t)r * pitch + tid] = run; }
        s_btot[tid] = run;
    }
    __syncthreads();
    STAMP();

    // ---- 5: the band of every row
    uint32_t width;
    if (nl == BAND_NLAM) {
        if (L <= 128u) width = band_rows<8, 4>(AT, pitch, s_lam, s_btot, s_cum, s_blo, s_bhi, bb, L, cap, ub_m);
        else width = band_rows<4, 8>(AT, pitch, s_lam, s_btot, s_cum, s_blo, s_bhi, bb, L, cap, ub_m);
    } else {
        width = band_rows<1, BAND_NLAM_MANY>(AT, pitch, s_lam, s_btot, s_cum, s_blo, s_bhi, bb, L, cap, ub_m);
    }
    if (tid == 0) { bb.lo[0] = 0u; bb.hi[0] = 0u; s_blo[0] = 0u; s_bhi[0] = 0u; }
    __syncthreads();
    STAMP();

    // ---- 6: the records that can connect the bands of rows i and i + 1: a cell of each differ by a cost in
    // [lo' - hi, hi' - lo]; costs ascend along a list, so they are a run of it
    uint32_t kf = 0u, cnt = 0u;
    if (tid < L) {
        const uint32_t plo = s_blo[tid], phi = s_bhi[tid], clo = s_blo[tid + 1u], chi = s_bhi[tid + 1u];
        if (chi >= plo) {
            const uint32_t w_min = clo > phi ? clo - phi : 0u, w_max = chi - plo;
            uint32_t k = 0u;
            while (k < my_n && (uint32_t)raw_w[my_off + k] < w_min) ++k;
            kf = k;
            while (k < my_n && (uint32_t)raw_w[my_off + k] <= w_max) ++k;
            cnt = k - kf;
        }
    }
    uint32_t total_live;
    const uint32_t at = block_exclusive_scan<uint32_t>(cnt, su, &total_live);
    if (tid < L) { bb.live_off[tid] = at; s_q[tid] = (uint16_t)at; s_hn[tid] = (uint16_t)(kf | (cnt << 8)); }
    if (tid == 0) bb.live_off[L] = total_live;
    __syncthreads();
    for (uint32_t i0 = wave * 8u; i0 < L; i0 += NWAVES * 8u) {
        double e[8], b[8];
        uint32_t w[8], jj[8], dst[8];
        bool in[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t i = min(i0 + (uint32_t)u, L - 1u);
            const uint32_t f = (uint32_t)s_hn[i] & 0xFFu, c = (uint32_t)s_hn[i] >> 8;
            in[u] = i0 + (uint32_t)u < L && lane < c;
            const size_t o = in[u] ? (size_t)i * J + f + lane : 0;
            dst[u] = (uint32_t)s_q[i] + lane;
            e[u] = dl.e[2 * o]; b[u] = dl.e[2 * o + 1]; w[u] = dl.w[o]; jj[u] = dl.jj[o];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (in[u]) { bb.live_e[dst[u]] = e[u]; bb.live_before[dst[u]] = b[u]; bb.live_w[dst[u]] = w[u]; bb.live_jj[dst[u]] = jj[u]; }
    }
    STAMP();
#ifdef KIMAD_STAMPS
    if (tid == 0) for (int q = 1; q < ns; ++q) bb.info[4 + q - 1] = (uint32_t)(stamp[q] - stamp[q - 1]);
#endif
    // diagnostics
    uint32_t wsum;
    (void)block_exclusive_scan<uint32_t>(width, su, &wsum);
    if (tid >= 1u && tid <= L) atomicMax(&s_wmax, (uint32_t)s_bhi[tid] - (uint32_t)s_blo[tid] + 1u);
    __syncthreads();
    if (tid == 0) { bb.info[0] = s_wmax; bb.info[1] = wsum; bb.info[2] = 0u; bb.info[3] = upgrades; }
}

// The recurrence on the band cells, by one workgroup of sixteen waves.  Both rows sit in LDS, indexed from their
// band's first cell.  Only the list records that can connect the bands of the two rows are visited (k_dp_bounds
// wrote them out, layer after layer); they wait in LDS, a group of layers at a time.
//
// The chain of L layers is sequential and a layer is little work (a hundred-odd cells, a few records each), so a
// layer is spread over the whole workgroup: a group of NP = 1, 2, 4, 8 or 16 neighbouring lanes shares a cell,
// lane s of the group takes records s, s + NP, ... in ascending order with a strict "<", and the group's minimum of
// (total, record) in that order, the total first, is formed with DPP moves (no LDS traffic).  That is the candidate
// the sequential scan of the whole list with a strict "<" would have kept: the first one, in list order, that attains
// the minimum.  The group's first lane then takes the lowest member of the winner's run whose rounded total is the
// same, and stores the cell's value, its winner and the cell it came from.  One barrier per layer.
//
// When the bands are narrow enough the winners stay in LDS (a global store inside the loop would be waited for
// before the registers it used can be written again); otherwise they go to the tables in memory, as in the
// whole-row recurrence.  The least total of the last row at its smallest cost, the walk back through the winners
// and the outputs j, K and offsets follow in the same launch.
constexpr uint32_t BANDED_THREADS = 1024;
static_assert(BANDED_THREADS >= BAND_MAX_L, "the set-up and the outputs give a thread to every layer");
constexpr uint32_t BAND_LIVE_CAP = 2048;       // live records held in LDS at a time
constexpr uint32_t BANDED_POOL = 140 * 1024;   // bytes of LDS carved at run time: two rows, live records, winners

// (total, record) of another lane of the group; the smaller pair stays
template <int CTRL>
__device__ __forceinline__ void take_min_dpp(double& t, uint32_t& k) {
    const double ot = dpp_f64<CTRL>(t);
    const uint32_t ok = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)k, CTRL, 0xF, 0xF, false);
    if (ot < t || (ot == t && ok < k)) { t = ot; k = ok; }
}
template <int NP>
__device__ __forceinline__ void group_min_pair(double& t, uint32_t& k) {
    if (NP >= 2) take_min_dpp<0xB1>(t, k);       // quad_perm [1,0,3,2]
    if (NP >= 4) take_min_dpp<0x4E>(t, k);       // quad_perm [2,3,0,1]
    if (NP >= 8) take_min_dpp<0x141>(t, k);      // row_half_mirror: the other quad of the eight
    if (NP >= 16) take_min_dpp<0x140>(t, k);     // row_mirror: the other eight of the sixteen
}

struct BandedLds {
    double* row0; double* row1;
    double* l_e; double* l_before; uint32_t* l_w; uint32_t* l_jj;
    uint32_t* out_w;
    uint32_t live_cap;
};

// one layer: NP lanes per cell
template <int NP, bool IN_LDS>
__device__ __forceinline__ void banded_layer(const AllocBuffers& ab, const BandedLds& z, uint32_t i, uint32_t base, uint32_t n,
                                             uint32_t plo, uint32_t pspan, uint32_t clo, uint32_t chi, uint32_t wc) {
    const uint32_t tid = threadIdx.x, sub = tid % NP, J = ab.J;
    const double* prow = (i & 1u) ? z.row1 : z.row0;
    double* crow = (i & 1u) ? z.row0 : z.row1;
    for (uint32_t c0 = clo; c0 <= chi; c0 += BANDED_THREADS / NP) {
        const uint32_t c = c0 + tid / NP, cm = c - plo;
        double best = DP_INF;
        uint32_t bk = 0xFFu;
        if (c <= chi) {
            for (uint32_t k = sub; k < n; k += NP) {
                const uint32_t src = cm - z.l_w[base + k];      // a cell cheaper than the record wraps far beyond the span
                if (src <= pspan) {
                    const double t = prow[src] + z.l_e[base + k];
                    if (t < best) { best = t; bk = k; }
                }
            }
        }
        group_min_pair<NP>(best, bk);
        if (sub == 0u && c <= chi) {
            uint32_t bj = 0xFFu, from = 0xFFFFu;
            if (bk != 0xFFu) {
                const uint32_t wj = z.l_jj[base + bk];
                from = c - z.l_w[base + bk];
                const double bp = prow[from - plo];
                bj = wj >> 8;
                if (bp + z.l_before[base + bk] == best) {
                    const uint32_t jlo = wj & 0xFFu;
                    uint32_t j = bj - 1u;
                    while (j > jlo && bp + ab.E[(size_t)i * J + j - 1u] == best) --j;
                    bj = j;
                }
            }
            crow[c - clo] = best;
            if (IN_LDS) {
                z.out_w[wc + (c - clo)] = bj | (from << 16);
            } else {
                ab.choice[(size_t)i * ab.stride + c] = (uint8_t)bj;
                ab.cprev[(size_t)i * ab.stride + c] = (uint16_t)from;
            }
        }
    }
}

template <bool IN_LDS>
__device__ __forceinline__ void banded_layers(const AllocBuffers& ab, const BandBuffers& bb, const BandedLds& z,
                                              const uint32_t* s_lo, const uint32_t* s_hi, const uint32_t* s_off,
                                              const uint32_t* s_wcum) {
    const uint32_t tid = threadIdx.x;
    const uint32_t L = ab.L;
    uint32_t i = 0;
    while (i < L) {
        // a group of layers whose live records fit LDS (at least one layer: a list has at most 64 records)
        const uint32_t g0 = s_off[i];
        uint32_t i1 = i + 1u;
        while (i1 < L && s_off[i1 + 1u] - g0 <= z.live_cap) ++i1;
        const uint32_t gcount = min(s_off[i1] - g0, z.live_cap);
        for (uint32_t t = tid; t < gcount; t += BANDED_THREADS) {
            z.l_e[t] = bb.live_e[g0 + t]; z.l_before[t] = bb.live_before[g0 + t];
            z.l_w[t] = bb.live_w[g0 + t]; z.l_jj[t] = bb.live_jj[g0 + t];
        }
        lds_barrier();
        for (; i < i1; ++i) {
            const uint32_t base = s_off[i] - g0, n = s_off[i + 1u] - s_off[i];
            const uint32_t plo = s_lo[i], pspan = s_hi[i] - plo, clo = s_lo[i + 1u], chi = s_hi[i + 1u], wc = s_wcum[i];
            // lanes per cell: as many as there are records, up to 16 (all of these are the same in every lane)
            if (n <= 1u) banded_layer<1, IN_LDS>(ab, z, i, base, n, plo, pspan, clo, chi, wc);
            else if (n <= 2u) banded_layer<2, IN_LDS>(ab, z, i, base, n, plo, pspan, clo, chi, wc);
            else if (n <= 4u) banded_layer<4, IN_LDS>(ab, z, i, base, n, plo, pspan, clo, chi, wc);
            else if (n <= 8u) banded_layer<8, IN_LDS>(ab, z, i, base, n, plo, pspan, clo, chi, wc);
            else banded_layer<16, IN_LDS>(ab, z, i, base, n, plo, pspan, clo, chi, wc);
            lds_barrier();                       // the next layer reads this row (and the next group overwrites the records)
        }
    }
}

__global__ __launch_bounds__(BANDED_THREADS) void k_dp_banded(AllocBuffers ab, BandBuffers bb, const uint32_t* __restrict__ bad,
                                                              int32_t err_infeasible, int32_t err_nonfinite) {
    __shared__ __align__(16) unsigned char pool[BANDED_POOL];
    __shared__ uint32_t s_lo[BAND_MAX_L + 1], s_hi[BAND_MAX_L + 1], s_off[BAND_MAX_L + 1], s_wcum[BAND_MAX_L + 1];
    __shared__ uint8_t s_j[BAND_MAX_L];
    __shared__ uint32_t su[16];
    __shared__ unsigned long long su64[16];
    __shared__ uint32_t s_wmax, s_bad;
    __shared__ unsigned long long s_best;        // bits of the least total (non-negative doubles order like their bit patterns)
    __shared__ uint32_t s_bc;
    const uint32_t tid = threadIdx.x;
    const uint32_t L = ab.L, J = ab.J, cap = ab.cap;
#ifdef KIMAD_STAMPS
    const unsigned long long t_begin = __builtin_readcyclecounter();
#endif
    if (tid == 0) { s_wmax = 1u; s_bad = 0u; s_best = ~0ull; s_bc = 0xFFFFFFFFu; }
    __syncthreads();
    // bands, live offsets, cumulative widths: rows 0..L (L <= BAND_MAX_L = the workgroup's size; row L by thread 0 again)
    uint32_t wd = 0u;
    for (uint32_t r = tid; r <= L; r += BANDED_THREADS) {
        const uint32_t lo = min(bb.lo[r], cap), hi = max(lo, min(bb.hi[r], cap));
        s_lo[r] = lo; s_hi[r] = hi; s_off[r] = bb.live_off[r];
    }
    if (tid < L && bad[tid]) s_bad = 1u;
    __syncthreads();
    // s_wcum[i] = first word of layer i's winners = widths of rows 1..i (row 0 stores nothing); thread r - 1 owns row r
    if (tid < L) wd = s_hi[tid + 1u] - s_lo[tid + 1u] + 1u;
    if (wd) atomicMax(&s_wmax, wd);
    uint32_t total_words;
    const uint32_t before = block_exclusive_scan<uint32_t>(wd, su, &total_words);
    if (tid < L) s_wcum[tid] = before;
    __syncthreads();
    const uint32_t wmax = s_wmax;
    const bool any_bad = s_bad != 0u;
    // carve the pool
    const uint32_t wr = (wmax + 63u) & ~63u;                                  // cells per row buffer
    const uint32_t total_live = s_off[L];
    BandedLds z;
    z.live_cap = min(max(total_live, 64u), BAND_LIVE_CAP);
    z.row0 = reinterpret_cast<double*>(pool);
    z.row1 = z.row0 + wr;
    z.l_e = z.row1 + wr;
    z.l_before = z.l_e + z.live_cap;
    z.l_w = reinterpret_cast<uint32_t*>(z.l_before + z.live_cap);
    z.l_jj = z.l_w + z.live_cap;
    z.out_w = z.l_jj + z.live_cap;
    const uint32_t used_bytes = (uint32_t)(reinterpret_cast<unsigned char*>(z.out_w) - pool);
    const uint32_t out_cap = (BANDED_POOL - used_bytes) / 4u;                 // (two rows of 4224 cells and 2048 records leave 23 KB)
    const bool in_lds = total_words <= out_cap;
    if (tid == 0) z.row0[0] = 0.0;
    lds_barrier();
    if (in_lds) banded_layers<true>(ab, bb, z, s_lo, s_hi, s_off, s_wcum);
    else banded_layers<false>(ab, bb, z, s_lo, s_hi, s_off, s_wcum);
#ifdef KIMAD_STAMPS
    const unsigned long long t_layers = __builtin_readcyclecounter();
#endif
    // ---- least total of the last row, smallest cost attaining it (totals are sums of squares: never negative, so
    // their bit patterns order like the numbers; +inf stays the largest)
    const uint32_t llo = s_lo[L], lhi = s_hi[L];
    const double* lrow = (L & 1u) ? z.row1 : z.row0;
    {
        double best = DP_INF;
        for (uint32_t c = llo + tid; c <= lhi; c += BANDED_THREADS) best = min_f64(best, lrow[c - llo]);
        atomicMin(&s_best, (unsigned long long)__double_as_longlong(best));
        __syncthreads();
        const double least = __longlong_as_double((long long)s_best);
        for (uint32_t c = llo + tid; c <= lhi; c += BANDED_THREADS)
            if (lrow[c - llo] == least) atomicMin(&s_bc, c);
        __syncthreads();
    }
    const double best = __longlong_as_double((long long)s_best);
    const uint32_t bc = s_bc;
    int32_t st = 0;
    if (any_bad) st = err_nonfinite;
    else if (!(best < DP_INF)) st = err_infeasible;
    if (tid == 0) *ab.status = st;
    if (st != 0) {
        for (uint32_t i = tid; i < L; i += BANDED_THREADS) { ab.j_out[i] = 0; ab.K_out[i] = 0; }
        for (uint32_t i = tid; i <= L; i += BANDED_THREADS) ab.offsets_out[i] = 0;
        return;
    }
    // ---- back-tracking by one thread, winners into LDS
    if (tid == 0) {
        uint32_t c = bc;
        if (in_lds) {
            for (uint32_t i = L; i-- > 0;) {
                const uint32_t word = z.out_w[s_wcum[i] + (c - s_lo[i + 1u])];
                s_j[i] = (uint8_t)word;
                c = min(word >> 16, cap);
            }
        } else {
            for (uint32_t i = L; i-- > 0;) {
                s_j[i] = ab.choice[(size_t)i * ab.stride + c];
                c = min((uint32_t)ab.cprev[(size_t)i * ab.stride + c], cap);
            }
        }
    }
    __syncthreads();
    // ---- sizes and offsets
    {
        unsigned long long K = 0ull;
        uint32_t j = 0u;
        if (tid < L) { j = s_j[tid]; K = ab.Kout[(size_t)tid * J + min(j, J - 1u)]; }
        unsigned long long total;
        const unsigned long long off = block_exclusive_scan<unsigned long long>(K, su64, &total);
        if (tid < L) { ab.j_out[tid] = (int32_t)j; ab.K_out[tid] = K; ab.offsets_out[tid] = off; }
        if (tid == 0) ab.offsets_out[L] = total;
    }
#ifdef KIMAD_STAMPS
    if (tid == 0) {
        bb.info[12] = (uint32_t)(t_layers - t_begin); bb.info[13] = (uint32_t)(__builtin_readcyclecounter() - t_begin);
        bb.info[14] = in_lds ? 1u : 0u; bb.info[15] = total_live;
    }
#endif
}

}  // namespace kimad
