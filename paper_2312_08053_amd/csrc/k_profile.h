// Error-profile kernels: two streaming histogram passes over g, h for the tiled layers, two
// per-layer scan kernels, and a whole-layer LDS sort for small layers.
//
// What they compute is the Errors matrix of the paper's Appendix C with the squared-l2 error of
// Section 3.2 (Eq. norm decomposition): E_ij = sum of x^2 over the entries TopK_{K_ij} drops.
#pragma once
#include "common.h"

namespace kimad {

struct ProfileBuffers {
    const LayerDesc* layers;
    const uint32_t* tile_layer;   // tile -> layer
    const uint32_t* big_layer;    // big index -> layer
    const uint32_t* small_layer;  // small index -> layer
    uint32_t tile_elems;          // elements per tile (multiple of 2048, <= 32768)
    // pass 1
    uint32_t* cnt1;               // [B][4096]
    uint64_t* sq1;                // [B][4096]
    // boundary bins
    uint8_t* lut1;                // [B][4096] digit-1 bin -> slot or NO_SLOT
    uint32_t* nslots;             // [B]
    uint32_t* slot_bin;           // [B][64]
    // pass 2
    uint32_t* cnt2;               // [B][SLOT_STRIDE][128]
    uint64_t* sq2;                // [B][SLOT_STRIDE][128]
    uint32_t* slot_cnt;           // [B][SLOT_STRIDE] totals of the slots the single pass counted itself (k_reduce_parts)
    uint64_t* slot_sq;            // [B][SLOT_STRIDE]
    // per target (layer-major, stride J)
    uint32_t* tgt_slot;           // slot, or NO_SLOT when K == n (nothing dropped)
    uint32_t* tgt_r;              // entries selected inside the boundary bin (1..count)
    uint32_t* tgt_above1;         // entries in higher digit-1 bins
    double* tgt_below;            // sum of squares of all lower digit-1 bins
    // threshold cache for the compaction pass
    uint32_t* sel_prefix;         // 19-bit prefix
    uint32_t* sel_above;          // entries with a greater prefix
    uint32_t* sel_amb;            // entries with an equal prefix
    uint32_t* diag;               // [0] uncertified entries, [1] entries fixed by the exact fallback,
                                  // [2] pool entries handed out
    // exact digit-1 histograms of the last single-pass profile: the prediction of the next one
    uint32_t* hprev;              // [B][4096]
    unsigned long long* gprev;    // [4096] their sum over the layers
    uint32_t* fresh;              // 1 while the threshold cache and the candidates describe the current g - h:
                                  // set by the profile's last kernels, cleared by the compression
    // exact fallback for entries whose bound is not tight: last-digit histograms of their prefix bins
    uint32_t* layer_flag;         // [B] layer has at least one pool entry
    uint32_t pool_cap;            // pool entries the plan holds: min(B * J, POOL_LIMIT)
    uint32_t* pool_prefix;        // [pool_cap]
    uint32_t* pool_big;           // [pool_cap]
    uint32_t* pool_t0;            // [pool_cap] first target (li * J + j) of the run sharing the prefix
    uint32_t* pool_cnt;           // [pool_cap] targets in that run
    uint32_t* pool_hist;          // [pool_cap][4096]
    uint32_t* tgt_unsel;          // dropped entries inside the prefix bin
    double* tgt_base;             // E without the prefix bin's share
    // fused single-pass profile
    LayerState* state;            // [B]
    const uint64_t* big_tmp0;     // [B] start of the layer's region in the candidate buffer (LayerDesc::tmp0)
    // histograms of the streaming pass, one copy ("part") per workgroup and segment of a layer
    unsigned long long* parts;    // [nparts][PART_STRIDE] packed LDS entries as they were, then the exact bin-0 sum
    const uint32_t* wg_part0;     // [workgroups] first part of each workgroup (its parts follow in order)
    const uint32_t* big_part0;    // [B] first part of each big layer
    const uint32_t* big_nparts;   // [B]
    const uint32_t* chunk_big;    // chunk -> big index
    const uint32_t* chunk_first;  // chunk -> first chunk of its layer
    uint32_t nchunks_total;
    const uint32_t* swg_layer;    // sampling workgroup -> layer
    const uint32_t* swg_first;    // sampling workgroup -> its first sampled group in that layer
    uint32_t* shist;              // [B][4096] digit-1 counts of the sample
    unsigned long long* ghist;    // [4096] sample counts of all layers, scaled by the sampling stride
    uint8_t* lutc;                // [B][4096] digit-1 bin -> slot PRE_SLOTS.. filled from the candidates
    uint32_t* cursor;             // [B] candidate entries handed out so far
    uint32_t* spill_over;         // [B] a reservation did not fit the layer's region
    uint32_t* rec_start;          // per chunk: start inside the layer's candidate region
    uint32_t* rec_cnt;            // per chunk: candidates written
    uint32_t* tmp_idx;
    float* tmp_x;
};

// Pool of exact last-digit histograms: one entry per (layer, threshold prefix) whose error bound is
// too wide.  A layer has at most J such prefixes, so B * J entries can never run out; plans with
// more than POOL_LIMIT of them hold POOL_LIMIT, and a candidate that finds the pool full gets NaN
// in the table (the allocation then reports a non-finite table instead of using a loose value).
constexpr uint32_t POOL_LIMIT = 65536;          // 16 KB each: at most 1 GB
constexpr uint32_t POOL_GRID = 256;             // workgroups of the exact scan (it normally finds nothing)
constexpr uint32_t POOL_NONE = 0xFFFFFFFFu;

// ---------------------------------------------------------------------------------------------
// Pass 1: per-layer histogram of digit 1 with counts and integer sums of squares.
// One workgroup per tile; the histogram lives in LDS as packed 64-bit entries.
__global__ __launch_bounds__(256) void k_hist1(ProfileBuffers pb) {
    __shared__ unsigned long long hist[D1_BINS];
    __shared__ unsigned long long sq0;         // exact squares of bin 0 (tiny denormals)
    const uint32_t tid = threadIdx.x;
    for (uint32_t b = tid; b < D1_BINS; b += 256) hist[b] = 0ull;
    if (tid == 0) sq0 = 0ull;
    __syncthreads();

    const uint32_t tile = blockIdx.x;
    const uint32_t li = pb.tile_layer[tile];
    const LayerDesc L = pb.layers[li];
    const uint32_t vbase = (tile - L.tile0) * pb.tile_elems;
    const uint32_t iters = pb.tile_elems / 1024u;

    for (uint32_t it = 0; it < iters; it += 2) {
        Quad q[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) load_quad(L, vbase + (it + u) * 1024u + tid * 4u, q[u]);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = q[u].key[c];
                if (key == KEY_INVALID) continue;
                const uint32_t bin = key >> D1_SHIFT;
                if (bin != 0u) {
                    atomicAdd(&hist[bin], CNT_ONE | (unsigned long long)sq_fixed(key));
                } else {
                    atomicAdd(&hist[0], CNT_ONE);
                    if (key) atomicAdd(&sq0, sq_exact(key));
                }
            }
        }
    }
    __syncthreads();
    uint32_t* cnt = pb.cnt1 + (size_t)L.big * D1_BINS;
    unsigned long long* sq = reinterpret_cast<unsigned long long*>(pb.sq1) + (size_t)L.big * D1_BINS;
    for (uint32_t b = tid; b < D1_BINS; b += 256) {
        const unsigned long long v = hist[b];
        if (v) {
            atomicAdd(&cnt[b], (uint32_t)(v >> 48));
            const unsigned long long s = b ? (v & SQ_MASK) : sq0;
            if (s) atomicAdd(&sq[b], s);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Scan 1: per big layer, locate every candidate's boundary bin in digit 1.
// targets: K values, row `li` of a [L][J] table.
__global__ __launch_bounds__(256) void k_scan1(ProfileBuffers pb, const uint32_t* Ktab, uint32_t J) {
    __shared__ uint32_t cnt[D1_BINS];
    __shared__ uint32_t above[D1_BINS];      // entries in strictly higher bins
    __shared__ double below[D1_BINS];        // squares in strictly lower bins
    __shared__ uint32_t su[16];
    __shared__ double sd[16];
    __shared__ uint32_t tbin[MAX_SLOTS];
    __shared__ double sh_total;              // squares of the whole layer (what K = 0 drops)
    const uint32_t tid = threadIdx.x;
    const uint32_t big = blockIdx.x;
    const uint32_t li = pb.big_layer[big];
    const LayerDesc L = pb.layers[li];
    const uint32_t* gcnt = pb.cnt1 + (size_t)big * D1_BINS;
    const uint64_t* gsq = pb.sq1 + (size_t)big * D1_BINS;

    // thread t owns bins 16t .. 16t+15
    uint32_t c[16];
    double s[16];
    uint32_t csum = 0;
    double ssum = 0.0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const uint32_t b = tid * 16u + k;
        c[k] = gcnt[b];
        s[k] = sq_to_double(b, gsq[b], c[k]);
        csum += c[k];
        ssum += s[k];
    }
    uint32_t ctot;
    const uint32_t cex = block_exclusive_scan<uint32_t>(csum, su, &ctot);
    const double sex = block_exclusive_scan<double>(ssum, sd, nullptr);
    {
        uint32_t run_c = cex;      // entries in bins below the current one
        double run_s = sex;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t b = tid * 16u + k;
            cnt[b] = c[k];
            below[b] = run_s;
            run_c += c[k];
            above[b] = ctot - run_c;
            run_s += s[k];
        }
        if (tid == 255u) sh_total = run_s;
    }
    uint8_t* lut = pb.lut1 + (size_t)big * D1_BINS;
    for (uint32_t b = tid; b < D1_BINS; b += 256) lut[b] = (uint8_t)NO_SLOT;
    __syncthreads();

    if (tid < J) {
        const uint32_t K = Ktab[(size_t)li * J + tid];
        uint32_t bin = 0xFFFFFFFFu;
        if (K == 0u) pb.tgt_below[(size_t)li * J + tid] = sh_total;      // nothing kept: everything is dropped
        if (K != 0u && K < L.n) {
            // smallest bin with above[bin] < K (above is non-increasing, above[4095] = 0)
            uint32_t lo = 0, hi = D1_BINS - 1;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (above[mid] < K) hi = mid; else lo = mid + 1;
            }
            bin = lo;
            pb.tgt_r[(size_t)li * J + tid] = K - above[bin];
            pb.tgt_above1[(size_t)li * J + tid] = above[bin];
            pb.tgt_below[(size_t)li * J + tid] = below[bin];
        }
        tbin[tid] = bin;
    }
    __syncthreads();
    if (tid == 0) {
        // Targets are sorted by K, so equal boundary bins are adjacent.
        uint32_t ns = 0, last = 0xFFFFFFFFu;
        for (uint32_t j = 0; j < J; ++j) {
            const uint32_t bin = tbin[j];
            uint32_t slot = NO_SLOT;
            if (bin != 0xFFFFFFFFu) {
                if (bin != last) {
                    lut[bin] = (uint8_t)ns;
                    pb.slot_bin[(size_t)big * SLOT_STRIDE + ns] = bin;
                    last = bin;
                    ++ns;
                }
                slot = ns - 1;
            }
            pb.tgt_slot[(size_t)li * J + j] = slot;
        }
        pb.nslots[big] = ns;
        LayerState st;
        st.spill_bin = D1_BINS; st.nslots_d = ns; st.nslots_t = 0; st.redo = 1;
        st.spill_cnt = 0; st.spill_valid = 0; st.slot_lo = 0; st.pad = 0;
        pb.state[big] = st;
    }
}

// ---------------------------------------------------------------------------------------------
// Pass 2: digit-2 histograms (count + squares) of the entries that fall in a boundary bin.
// Workgroups take tiles in a grid-stride loop.  `gate` (optional) points at a device word that is
// zero when no layer needs this pass: the single-pass profile launches it as a fallback that
// normally has nothing to do, with a small grid that leaves after one load, and with `coarse` set
// so that the recount holds the same numbers the pass itself would have put into the slot.
__global__ __launch_bounds__(512) void k_hist2(ProfileBuffers pb, uint32_t ntiles, const uint32_t* gate,
                                               uint32_t coarse) {
    __shared__ unsigned long long sub[MAX_SLOTS * D2_BINS];   // 64 KB
    __shared__ unsigned long long sub0[D2_BINS];              // exact squares when the slot is bin 0
    __shared__ uint8_t lut[D1_BINS];
    const uint32_t tid = threadIdx.x;
    if (gate && *gate == 0u) return;
    for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t li = pb.tile_layer[tile];
    const LayerDesc L = pb.layers[li];
    const LayerState st = pb.state[L.big];
    const uint32_t ns = st.nslots_d;
    if (!st.redo || ns == 0) continue;
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(pb.lut1 + (size_t)L.big * D1_BINS);
        uint32_t* dst = reinterpret_cast<uint32_t*>(lut);
        for (uint32_t b = tid; b < D1_BINS / 4; b += 512) dst[b] = src[b];
    }
    for (uint32_t b = tid; b < ns * D2_BINS; b += 512) sub[b] = 0ull;
    if (tid < D2_BINS) sub0[tid] = 0ull;
    __syncthreads();

    const uint32_t vbase = (tile - L.tile0) * pb.tile_elems;
    const uint32_t iters = pb.tile_elems / 2048u;
    for (uint32_t it = 0; it < iters; it += 2) {
        Quad q[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (it + u < iters) load_quad(L, vbase + (it + u) * 2048u + tid * 4u, q[u]);
            else { q[u].key[0] = q[u].key[1] = q[u].key[2] = q[u].key[3] = KEY_INVALID; }
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = q[u].key[c];
                if (key == KEY_INVALID) continue;
                const uint32_t bin = key >> D1_SHIFT;
                const uint32_t slot = lut[bin];
                if (slot == NO_SLOT) continue;
                const uint32_t d2 = (key >> D2_SHIFT) & (D2_BINS - 1);
                if (bin != 0u) {
                    atomicAdd(&sub[slot * D2_BINS + d2],
                              CNT_ONE | (unsigned long long)(coarse ? sq_coarse(key) : sq_fixed(key)));
                } else {
                    atomicAdd(&sub[slot * D2_BINS + d2], CNT_ONE);
                    if (key) atomicAdd(&sub0[d2], sq_exact(key));
                }
            }
        }
    }
    __syncthreads();
    uint32_t* cnt = pb.cnt2 + (size_t)L.big * SLOT_STRIDE * D2_BINS;
    unsigned long long* sq = reinterpret_cast<unsigned long long*>(pb.sq2) + (size_t)L.big * SLOT_STRIDE * D2_BINS;
    const uint32_t slot0 = lut[0];   // slot of bin 0, if it is a boundary bin
    for (uint32_t b = tid; b < ns * D2_BINS; b += 512) {
        const unsigned long long v = sub[b];
        if (v) {
            atomicAdd(&cnt[b], (uint32_t)(v >> 48));
            const unsigned long long s = (b / D2_BINS == slot0) ? sub0[b % D2_BINS] : (v & SQ_MASK);
            if (s) atomicAdd(&sq[b], s);
        }
    }
    __syncthreads();                            // the next tile reuses the LDS tables
    }
}

// ---------------------------------------------------------------------------------------------
// Scan 2: per big layer and candidate, locate the boundary inside digit 2, assemble E_ij and
// remember the 19-bit threshold prefix.  What is left undecided is how the `unsel` smallest of
// the `m` entries sharing that prefix split the prefix bin's exact sum of squares Q; their
// magnitudes differ by at most 2^-11 relative, and the estimate below is clamped to rigorous
// bounds.  Entries whose bound is not tight enough are counted in diag[0].
__device__ __forceinline__ float prefix_lo(uint32_t prefix) { return __uint_as_float(prefix << D2_SHIFT); }

// One wave per candidate: every lane holds two digit-2 bins of the candidate's boundary bin.
// `flagged` and `prefix_out` come back the same in every lane.
// What a target's loads bring: first what its index addresses, then what its slot addresses.  A wave looks after
// several targets; it asks for all of one kind together, so that the round trips to memory are two per wave, not
// two per target.
struct Scan2Target {
    uint32_t K, slot, r, above1;
    double below;
    uint32_t bin;
    uint2 c;
    ulonglong2 q;
};
__device__ __forceinline__ void scan2_load_target(const ProfileBuffers& pb, const uint32_t* Ktab, size_t t, Scan2Target& T) {
    T.K = Ktab[t];
    T.slot = pb.tgt_slot[t];
    T.r = pb.tgt_r[t];
    T.above1 = pb.tgt_above1[t];
    T.below = pb.tgt_below[t];
}
__device__ __forceinline__ void scan2_load_slot(const ProfileBuffers& pb, uint32_t big, Scan2Target& T) {
    const uint32_t lane = lane_id();
    T.bin = pb.slot_bin[(size_t)big * SLOT_STRIDE + T.slot];
    T.c = reinterpret_cast<const uint2*>(pb.cnt2 + ((size_t)big * SLOT_STRIDE + T.slot) * D2_BINS)[lane];
    T.q = reinterpret_cast<const ulonglong2*>(pb.sq2 + ((size_t)big * SLOT_STRIDE + T.slot) * D2_BINS)[lane];
}
__device__ __forceinline__ void scan2_target(const ProfileBuffers& pb, const Scan2Target& T, uint32_t n, size_t t,
                                             double* err_table, double tol, double widen, bool* flagged,
                                             uint32_t* prefix_out) {
    const uint32_t lane = lane_id();
    const uint32_t K = T.K;
    if (T.slot == NO_SLOT) {                    // K == n (or K == 0): nothing / everything dropped
        if (lane == 0) {
            if (err_table) err_table[t] = (K == 0u) ? T.below : 0.0;
            pb.sel_prefix[t] = 0u;
            pb.sel_above[t] = (K == 0u) ? 0u : n;
            pb.sel_amb[t] = 0u;
            pb.tgt_unsel[t] = 0u;
            pb.tgt_base[t] = 0.0;
        }
        return;
    }
    const uint32_t bin = T.bin;
    const uint32_t r = T.r;
    const uint2 c = T.c;
    const ulonglong2 q = T.q;
    // walk digit 2 from the top until r entries are covered: the boundary is the highest bin u > 0
    // with (entries above u) + cnt[u] >= r, or bin 0
    const uint32_t incl = wave_scan_add_u32(c.x + c.y);
    const uint32_t tot = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    const uint32_t above_hi = tot - incl;       // entries above bin 2*lane+1
    const uint32_t above_lo = above_hi + c.y;   // entries above bin 2*lane
    const uint64_t m_hi = ballot(above_hi + c.y >= r), m_lo = ballot(above_lo + c.x >= r);
    const int u_hi = m_hi ? 2 * (63 - __clzll((long long)m_hi)) + 1 : 0;
    const int u_lo = m_lo ? 2 * (63 - __clzll((long long)m_lo)) : 0;
    const int u = max(u_hi, u_lo);
    const int src = u >> 1;
    const uint32_t acc = (u & 1) ? __shfl(above_hi, src, 64) : __shfl(above_lo, src, 64);
    const uint32_t m = (u & 1) ? __shfl(c.y, src, 64) : __shfl(c.x, src, 64);
    const unsigned long long squ = (u & 1) ? __shfl(q.y, src, 64) : __shfl(q.x, src, 64);
    const uint32_t rsel = r - acc;              // 1..m selected inside the prefix bin
    const uint32_t unsel = m - rsel;
    double below2 = ((int)(2u * lane) < u ? sq_to_double(bin, q.x, c.x) : 0.0) +
                    ((int)(2u * lane + 1u) < u ? sq_to_double(bin, q.y, c.y) : 0.0);
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) below2 += __shfl_xor(below2, d, 64);
    const uint32_t prefix = (bin << D2_BITS) | (uint32_t)u;
    double est = 0.0, half_gap = 0.0;
    if (unsel) {
        const double Q = sq_to_double(bin, squ, m);
        if ((bin >> 4) == 255u) {
            // Inf/NaN entries: the dropped ones are the lowest keys, i.e. the infinities first.
            const uint64_t nans = squ;
            const uint64_t infs = (uint64_t)m - nans;
            est = (uint64_t)unsel > infs ? __longlong_as_double(0x7FF8000000000000ll)
                                         : __longlong_as_double(0x7FF0000000000000ll);
        } else {
            // The dropped entries are the `unsel` smallest of m values in [lo, hi) whose squares sum
            // to Q: at least unsel*lo^2 and Q - rsel*hi^2, at most their mean share and unsel*hi^2.
            const double lo = (double)prefix_lo(prefix), hi = (double)prefix_lo(prefix + 1u);
            const double ub = fmin(((double)unsel / (double)m) * Q, (double)unsel * hi * hi);
            const double lb = fmin(ub, fmax((double)unsel * lo * lo, Q - (double)rsel * hi * hi));
            est = 0.5 * (lb + ub);
            half_gap = 0.5 * (ub - lb);
        }
    }
    const double base = T.below + below2;
    const double E = base + est;
    // single-pass slots hold midpoints of intervals 2^-23 wide (relative): part of the bound
    half_gap += E * widen;
    if (lane == 0) {
        if (err_table) err_table[t] = E;
        pb.sel_prefix[t] = prefix;
        pb.sel_above[t] = T.above1 + acc;
        pb.sel_amb[t] = m;
        pb.tgt_unsel[t] = unsel;
        pb.tgt_base[t] = base;
    }
    *flagged = err_table != nullptr && half_gap > tol * E;
    *prefix_out = prefix;
}

// One workgroup per big layer, one wave per candidate at a time.  Candidates whose error bound is
// too wide are then grouped by prefix (equal prefixes are adjacent because K ascends) and each
// group gets one pool entry for the exact last-digit pass.
constexpr uint32_t SCAN2_THREADS = 1024;
__global__ __launch_bounds__(SCAN2_THREADS) void k_scan2(ProfileBuffers pb, const uint32_t* Ktab, uint32_t J,
                                                         double* err_table, double tol, double widen) {
    __shared__ uint32_t sh_prefix[KIMAD_MAX_J_CONST];
    __shared__ uint32_t sh_flag[KIMAD_MAX_J_CONST];
    __shared__ uint32_t sh_pool[KIMAD_MAX_J_CONST];     // pool entries this layer has taken
    __shared__ uint32_t sh_npool;
    if (threadIdx.x == 0) sh_npool = 0u;
    const uint32_t big = blockIdx.x;
    const uint32_t li = pb.big_layer[big];
    constexpr uint32_t WAVES = SCAN2_THREADS / 64, PER_WAVE = KIMAD_MAX_J_CONST / WAVES;
    static_assert(PER_WAVE * WAVES == KIMAD_MAX_J_CONST, "every wave looks after the same number of targets");
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t n = pb.layers[li].n;
    Scan2Target T[PER_WAVE];
#pragma unroll
    for (uint32_t u = 0; u < PER_WAVE; ++u) {
        const uint32_t jj = wave + u * WAVES;
        T[u].slot = NO_SLOT; T[u].K = 1u; T[u].r = 0u; T[u].above1 = 0u; T[u].below = 0.0;
        if (jj < J) scan2_load_target(pb, Ktab, (size_t)li * J + jj, T[u]);
    }
#pragma unroll
    for (uint32_t u = 0; u < PER_WAVE; ++u) {
        T[u].bin = 0u; T[u].c = make_uint2(0u, 0u); T[u].q = make_ulonglong2(0ull, 0ull);
        if (T[u].slot != NO_SLOT) scan2_load_slot(pb, big, T[u]);
    }
#pragma unroll
    for (uint32_t u = 0; u < PER_WAVE; ++u) {
        const uint32_t jj = wave + u * WAVES;
        bool fl = false;
        uint32_t px = 0xFFFFFFFFu - jj;         // distinct dummy for idle slots and K == n
        if (jj < J) scan2_target(pb, T[u], n, (size_t)li * J + jj, err_table, tol, widen, &fl, &px);
        if (lane_id() == 0) { sh_prefix[jj] = px; sh_flag[jj] = fl ? 1u : 0u; }
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const uint32_t j = threadIdx.x;
        const bool flagged = sh_flag[j] != 0u;
        const uint32_t prefix = sh_prefix[j];
        const uint32_t prev = __shfl_up(prefix, 1, 64);
        const bool head = j == 0 || prev != prefix;
        const uint64_t heads = ballot(head), flags = ballot(flagged);
        // run of this lane: from its head (highest head bit at or below j) to the lane before the next head
        const uint64_t below_or_eq = heads & (~0ull >> (63 - j));
        const uint32_t h0 = 63u - (uint32_t)__clzll((long long)below_or_eq);
        const uint64_t after = heads & ~((2ull << j) - 1ull);
        const uint32_t h1 = after ? (uint32_t)__ffsll((long long)after) - 1u : 64u;   // exclusive end
        const uint64_t run_mask = (h1 >= 64 ? ~0ull : ((1ull << h1) - 1ull)) & ~((1ull << h0) - 1ull);
        const bool run_flagged = (flags & run_mask) != 0;
        if (flagged) atomicAdd(&pb.diag[0], 1u);
        if (head && run_flagged && j < J) {
            const uint32_t f = atomicAdd(&pb.diag[2], 1u);
            if (f < pb.pool_cap) {
                pb.pool_prefix[f] = prefix;
                pb.pool_big[f] = big;
                pb.pool_t0[f] = li * J + j;
                pb.pool_cnt[f] = h1 - h0;
                pb.layer_flag[big] = 1u;
                sh_pool[atomicAdd(&sh_npool, 1u)] = f;
            } else {
                // pool full: no loose value leaves this call
                for (uint32_t k = h0; k < h1 && k < J; ++k)
                    err_table[(size_t)li * J + k] = __longlong_as_double(0x7FF8000000000000ll);
            }
        }
    }
    __syncthreads();
    // The pool's histograms share their memory with the streaming pass's histogram parts (dead by now): an
    // entry is cleared here, by the workgroup that takes it, before the exact pass counts into it.
    static_assert(D3_BINS == 4u * SCAN2_THREADS, "one 16-byte store per thread clears an entry");
    for (uint32_t k = 0; k < sh_npool; ++k)
        reinterpret_cast<uint4*>(pb.pool_hist + (size_t)sh_pool[k] * D3_BINS)[threadIdx.x] = make_uint4(0u, 0u, 0u, 0u);
}

// Exact fallback, pass: last-digit histogram of every pooled prefix bin.  One workgroup per tile;
// tiles of layers without pool entries return at once.
__global__ __launch_bounds__(256) void k_hist3p(ProfileBuffers pb, uint32_t ntiles) {
    __shared__ uint32_t pfx[KIMAD_MAX_J_CONST];   // a layer has at most J pooled prefixes
    __shared__ uint32_t pid[KIMAD_MAX_J_CONST];
    __shared__ uint32_t npool;
    const uint32_t tid = threadIdx.x;
    if (pb.diag[2] == 0u) return;               // no pool entries at all: the usual case
    for (uint32_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint32_t li = pb.tile_layer[tile];
    const LayerDesc L = pb.layers[li];
    if (!pb.layer_flag[L.big]) continue;
    __syncthreads();                            // the previous tile's readers are done with the lists
    if (tid == 0) npool = 0;
    __syncthreads();
    const uint32_t total = min(pb.diag[2], pb.pool_cap);
    for (uint32_t f = tid; f < total; f += 256) {
        if (pb.pool_big[f] == (uint32_t)L.big) {
            const uint32_t k = atomicAdd(&npool, 1u);
            if (k < KIMAD_MAX_J_CONST) { pfx[k] = pb.pool_prefix[f]; pid[k] = f; }
        }
    }
    __syncthreads();
    const uint32_t np = min(npool, (uint32_t)KIMAD_MAX_J_CONST);
    const uint32_t vbase = (tile - L.tile0) * pb.tile_elems;
    const uint32_t iters = pb.tile_elems / 1024u;
    for (uint32_t it = 0; it < iters; ++it) {
        Quad q;
        load_quad(L, vbase + it * 1024u + tid * 4u, q);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t key = q.key[c];
            uint32_t f = POOL_NONE;
            if (key != KEY_INVALID) {
                const uint32_t p = key >> D2_SHIFT;
                for (uint32_t k = 0; k < np; ++k) if (pfx[k] == p) f = pid[k];
            }
            const bool a = f != POOL_NONE;
            const uint64_t am = ballot(a);
            if (am == 0) continue;
            // one atomic per wave when all matching lanes hold the same key (constants, zeros)
            const uint32_t first_lane = (uint32_t)__ffsll((long long)am) - 1u;
            const uint32_t k0 = __shfl(key, first_lane, 64);
            if (ballot(a && key != k0) == 0) {
                if (lane_id() == first_lane) atomicAdd(&pb.pool_hist[(size_t)f * D3_BINS + (key & (D3_BINS - 1))], (uint32_t)__popcll(am));
            } else if (a) {
                atomicAdd(&pb.pool_hist[(size_t)f * D3_BINS + (key & (D3_BINS - 1))], 1u);
            }
        }
    }
    }
}

// Exact fallback, scan: one workgroup per pool entry.  With the full key known, the squares of the
// `unsel` smallest entries of the prefix bin are summed exactly in fp64, smallest first.
__global__ __launch_bounds__(256) void k_scan3p(ProfileBuffers pb, double* err_table, uint32_t mark_fresh) {
    __shared__ uint32_t su[16];
    __shared__ double sd[16];
    __shared__ uint32_t cum[D3_BINS];      // entries in lower digits
    __shared__ double sumsq[D3_BINS];      // their squares
    const uint32_t tid = threadIdx.x;
    const uint32_t total = min(pb.diag[2], pb.pool_cap);
    if (blockIdx.x == 0 && tid == 0 && mark_fresh) *pb.fresh = 1u;     // the grid profile's last kernel on the caller's stream
    for (uint32_t f = blockIdx.x; f < total; f += gridDim.x) {
    __syncthreads();                            // the previous entry's readers are done with the tables
    const uint32_t prefix = pb.pool_prefix[f];
    const uint32_t* h = pb.pool_hist + (size_t)f * D3_BINS;
    uint32_t c[16];
    double s[16];
    uint32_t csum = 0;
    double ssum = 0.0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const uint32_t d3 = tid * 16u + k;
        c[k] = h[d3];
        const double v = (double)__uint_as_float((prefix << D2_SHIFT) | d3);
        s[k] = (double)c[k] * v * v;
        csum += c[k];
        ssum += s[k];
    }
    const uint32_t cex = block_exclusive_scan<uint32_t>(csum, su, nullptr);
    const double sex = block_exclusive_scan<double>(ssum, sd, nullptr);
    {
        uint32_t rc = cex;
        double rs = sex;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            cum[tid * 16u + k] = rc;
            sumsq[tid * 16u + k] = rs;
            rc += c[k];
            rs += s[k];
        }
    }
    __syncthreads();
    const uint32_t t0 = pb.pool_t0[f], cnt = pb.pool_cnt[f];
    for (uint32_t k = tid; k < cnt; k += 256) {
        const uint32_t t = t0 + k;
        const uint32_t unsel = pb.tgt_unsel[t];
        double U = 0.0;
        if (unsel) {
            // largest digit d with cum[d] < unsel: digits below d are dropped whole
            uint32_t lo = 0, hi = D3_BINS - 1;
            while (lo < hi) {
                const uint32_t mid = (lo + hi + 1) >> 1;
                if (cum[mid] < unsel) lo = mid; else hi = mid - 1;
            }
            const double v = (double)__uint_as_float((prefix << D2_SHIFT) | lo);
            U = sumsq[lo] + (double)(unsel - cum[lo]) * v * v;
        }
        err_table[t] = pb.tgt_base[t] + U;
        atomicAdd(&pb.diag[1], 1u);
    }
    }
}

// ---------------------------------------------------------------------------------------------
// Small layers: the whole layer is sorted in LDS by (magnitude descending, index ascending);
// E_ij is the suffix sum of squares in sorted order, in fp64.  One workgroup per layer.
// Sort key: (0x7fffffff - key) << 32 | index, ascending.
template <uint32_t THREADS>
__device__ __forceinline__ void bitonic_sort_lds(unsigned long long* a, uint32_t P) {
    for (uint32_t k = 2; k <= P; k <<= 1) {
        for (uint32_t jj = k >> 1; jj > 0; jj >>= 1) {
            for (uint32_t t = threadIdx.x; t < P / 2; t += THREADS) {
                const uint32_t i = 2 * t - (t & (jj - 1));     // index with bit jj clear
                const uint32_t l = i + jj;
                const bool up = ((i & k) == 0);
                const unsigned long long x = a[i], y = a[l];
                if ((x > y) == up) { a[i] = y; a[l] = x; }
            }
            __syncthreads();
        }
    }
}

__device__ __forceinline__ uint32_t next_pow2(uint32_t n) {
    uint32_t p = 1;
    while (p < n) p <<= 1;
    return p;
}

__device__ __forceinline__ void load_sorted_small(const LayerDesc& L, unsigned long long* a, uint32_t P) {
    for (uint32_t e = threadIdx.x; e < P; e += blockDim.x) {
        unsigned long long v = ~0ull;
        if (e < L.n) {
            const uint32_t key = key_of(gload(L.g + e) - gload(L.h + e));
            v = ((unsigned long long)(0x7FFFFFFFu - key) << 32) | e;
        }
        a[e] = v;
    }
    __syncthreads();
}

constexpr uint32_t SMALL_THREADS = 1024;

__global__ __launch_bounds__(SMALL_THREADS) void k_small_profile(ProfileBuffers pb, const uint32_t* Ktab, uint32_t J,
                                                                 double* err_table, uint32_t mark_fresh) {
    __shared__ unsigned long long a[SMALL_MAX];       // 64 KB
    __shared__ double loc[SMALL_THREADS];             // per-thread sums, then exclusive suffix sums
    __shared__ double sd[16];
    const uint32_t li = pb.small_layer[blockIdx.x];
    const LayerDesc L = pb.layers[li];
    if (blockIdx.x == 0 && threadIdx.x == 0 && mark_fresh) *pb.fresh = 1u;   // (plans without tiled layers have no other profile kernel)
    const uint32_t P = next_pow2(L.n < 2 ? 2 : L.n);
    load_sorted_small(L, a, P);
    bitonic_sort_lds<SMALL_THREADS>(a, P);
    // thread t owns ranks [t*per, (t+1)*per) and sums their squares from the smallest upward
    const uint32_t per = P / SMALL_THREADS ? P / SMALL_THREADS : 1u;
    const uint32_t tid = threadIdx.x;
    double local = 0.0;
    for (uint32_t k = per; k-- > 0;) {
        const uint32_t rk = tid * per + k;
        if (rk < L.n) {
            const uint32_t key = 0x7FFFFFFFu - (uint32_t)(a[rk] >> 32);
            const double v = (double)__uint_as_float(key);
            local += v * v;
        }
    }
    loc[tid] = local;
    __syncthreads();
    // exclusive suffix over threads: scan the per-thread sums in reversed thread order
    const double rv = loc[SMALL_THREADS - 1u - tid];
    const double ex = block_exclusive_scan<double>(rv, sd, nullptr);
    __syncthreads();
    loc[SMALL_THREADS - 1u - tid] = ex;               // sum of the squares owned by all later threads
    __syncthreads();
    if (tid < J) {
        const uint32_t K = Ktab[(size_t)li * J + tid];
        double E = 0.0;
        if (K < L.n) {
            // ranks >= K are dropped: everything owned by later threads, then the tail of K's owner
            const uint32_t owner = K / per;
            E = loc[owner];
            for (uint32_t rk = (owner + 1) * per; rk-- > K;) {
                if (rk < L.n) {
                    const uint32_t key = 0x7FFFFFFFu - (uint32_t)(a[rk] >> 32);
                    const double v = (double)__uint_as_float(key);
                    E += v * v;
                }
            }
        }
        err_table[(size_t)li * J + tid] = E;
    }
}

}  // namespace kimad
