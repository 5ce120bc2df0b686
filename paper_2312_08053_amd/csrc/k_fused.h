// Single-pass error profile.
//
// The classic profile (k_profile.h) reads g and h twice: once to find every candidate's boundary
// bin in digit 1, once to histogram digit 2 inside those bins.  Here a sampling pre-pass over
// ~1/16 of each layer (a plan's first profile; later ones use the exact digit-1 histogram the previous
// profile left: successive gradients of a layer are distributed alike) predicts, per layer,
//   * which digit-1 bins can hold the boundary of a "dense" candidate (K beyond the top few
//     percent): those bins get digit-2 slots before the pass, and
//   * a spill bin: every entry at or above it (the top few percent, sized from the budget hint)
//     is written to the candidate buffer as (index, x), in index order inside each chunk.
// One streaming pass then builds the exact digit-1 histogram, the digit-2 histograms of the
// predicted bins and the candidate buffer.  Candidates whose boundary lies in the spilled range
// get their digit-2 histograms from the candidate buffer (a few percent of the data), and the
// compaction later selects from the candidates instead of reading g and h again.
//
// Nothing in the result depends on the prediction: a boundary that falls outside what was
// predicted marks the layer for a recount by the classic full pass (LayerState::redo), and a
// chosen K beyond the spilled range makes the compaction read g and h for that layer.
//
// Computes the same quantities as k_profile.h: the Errors matrix of the paper's Appendix C with
// the squared-l2 error of Section 3.2.
#pragma once
#include "common.h"
#include "k_profile.h"

namespace kimad {

constexpr uint32_t SAMPLE_GROUPS_PER_WG = 48;   // sampled chunks one sampling workgroup reads: three per wave (every
                                                // workgroup ends with a flush of its histogram through global
                                                // atomics, which is what the kernel's time is made of: fewer, longer
                                                // workgroups were faster at every size tried, 4 to 48)
constexpr uint32_t FUSED_THREADS = 1024;
constexpr uint32_t FUSED_WAVES = FUSED_THREADS / 64;

__device__ __forceinline__ uint32_t hash32(uint32_t a) {
    a ^= a >> 16; a *= 0x7feb352du; a ^= a >> 15; a *= 0x846ca68bu; a ^= a >> 16;
    return a;
}

// Chunk of the layer read by sampled group `gidx`: one per `stride` chunks, at a hashed phase.
__device__ __forceinline__ uint32_t sampled_chunk(uint32_t gidx, uint32_t stride) {
    return gidx * stride + (stride > 1 ? hash32(gidx * 2654435761u + 12345u) % stride : 0u);
}

// ---------------------------------------------------------------------------------------------
// Sampling pre-pass: digit-1 counts of the sampled chunks.
// One wave per sampled chunk: all of a workgroup's loads are in flight together.
constexpr uint32_t SAMPLE_THREADS = 1024;
__global__ __launch_bounds__(SAMPLE_THREADS) void k_sample(ProfileBuffers pb) {
    __shared__ uint32_t hist[D1_BINS];
    const uint32_t tid = threadIdx.x, wave = tid >> 6, lane = lane_id();
    for (uint32_t b = tid; b < D1_BINS; b += SAMPLE_THREADS) hist[b] = 0u;
    __syncthreads();
    const uint32_t li = pb.swg_layer[blockIdx.x];
    const LayerDesc L = pb.layers[li];
    const uint32_t first = pb.swg_first[blockIdx.x];
    for (uint32_t k = wave; k < SAMPLE_GROUPS_PER_WG; k += SAMPLE_THREADS / 64) {
        const uint32_t chunk = sampled_chunk(first + k, L.sstride);
        if (chunk >= L.nchunks) continue;
        const uint32_t vbase = chunk * CHUNK;
        Quad q[NQ];
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) load_quad(L, vbase + u * 256u + lane * 4u, q[u]);
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (q[u].key[c] != KEY_INVALID) atomicAdd(&hist[q[u].key[c] >> D1_SHIFT], 1u);
    }
    __syncthreads();
    uint32_t* sh = pb.shist + (size_t)L.big * D1_BINS;
    for (uint32_t b = tid; b < D1_BINS; b += SAMPLE_THREADS) {
        const uint32_t v = hist[b];
        if (v) {
            atomicAdd(&sh[b], v);
            atomicAdd(&pb.ghist[b], (unsigned long long)v * L.sstride);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Prediction: per big layer, the spill bin and the digit-1 bins that get a slot.
// `budget_pairs` = expected budget of the following allocation in pairs (0 = unknown).
// `counts` / `gcounts`: per layer and summed digit-1 counts to predict from: the sample of k_sample (scaled to the
// population through the layer's size), or the exact histogram of the previous profile on this plan (successive
// gradients of a layer are distributed alike; a layer whose boundary bins moved is recounted like any other
// misprediction).  `fold_zero`: also clear what a profile must find at zero (no separate clearing launch).
__global__ __launch_bounds__(256) void k_predict(ProfileBuffers pb, const uint32_t* Ktab, uint32_t J,
                                                 unsigned long long budget_pairs, const uint32_t* __restrict__ counts,
                                                 const unsigned long long* __restrict__ gcounts, uint32_t fold_zero) {
    __shared__ uint32_t above[D1_BINS];        // sample entries in strictly higher bins
    __shared__ uint32_t bitmap[D1_BINS / 32];
    __shared__ uint32_t su[16];
    __shared__ unsigned long long s64[16];
    __shared__ uint32_t sh_gbin, sh_spill, sh_ns;
    const uint32_t tid = threadIdx.x, big = blockIdx.x;
    const uint32_t li = pb.big_layer[big];
    const LayerDesc L = pb.layers[li];

    // this layer's sample counts are asked for together with the global ones of step (1)
    uint32_t c[16], csum = 0;
    {
        const uint4* sh4 = reinterpret_cast<const uint4*>(counts + (size_t)big * D1_BINS + tid * 16u);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint4 v = sh4[k];
            c[4 * k] = v.x; c[4 * k + 1] = v.y; c[4 * k + 2] = v.z; c[4 * k + 3] = v.w;
        }
    }
    // (1) global threshold bin: the highest bin b with (entries of all layers in bins >= b) >= 2.5 x budget
    {
        unsigned long long gc[16], sum = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) { gc[k] = gcounts[tid * 16u + k]; sum += gc[k]; }
        unsigned long long tot;
        const unsigned long long ex = block_exclusive_scan<unsigned long long>(sum, s64, &tot);
        unsigned long long ab = tot - ex - sum;            // entries above this thread's bins
        const unsigned long long want = budget_pairs * 5ull / 2ull;
        if (tid == 0) sh_gbin = 0u;                        // budget beyond everything: bin 0
        __syncthreads();
        if (budget_pairs && ab < want && ab + sum >= want) {
#pragma unroll
            for (int k = 15; k >= 0; --k) {
                if (ab + gc[k] >= want) { sh_gbin = tid * 16u + k; break; }
                ab += gc[k];
            }
        }
        __syncthreads();
    }
    // (2) this layer's sample: suffix counts
#pragma unroll
    for (int k = 0; k < 16; ++k) csum += c[k];
    uint32_t ns_total;
    const uint32_t cex = block_exclusive_scan<uint32_t>(csum, su, &ns_total);
    {
        uint32_t run = cex;
#pragma unroll
        for (int k = 0; k < 16; ++k) { run += c[k]; above[tid * 16u + k] = ns_total - run; }
    }
    if (tid < D1_BINS / 32) bitmap[tid] = 0u;
    __syncthreads();
    const double scale = (double)L.n / (double)(ns_total ? ns_total : 1u);   // population per sample entry
    // smallest bin with above[bin] < k, i.e. the bin holding the sample entry of rank k (k >= 1)
    auto find_bin = [&](uint32_t k) {
        uint32_t lo = 0, hi = D1_BINS - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi) >> 1;
            if (above[mid] < k) hi = mid; else lo = mid + 1;
        }
        return lo;
    };
    if (tid == 0) {
        // Spill everything down to the global threshold bin; at least the top 2 % (the sparse upper
        // tail would otherwise need a slot per candidate) and twice the smallest grid size (plus
        // 3 sigma of the sample count); at most an eighth of the layer.
        const uint32_t K0 = Ktab[(size_t)li * J];
        const double k0s = 2.0 * (double)K0 / scale;
        uint32_t floor_rank = (uint32_t)fmin((double)ns_total, ceil(k0s + 3.0 * sqrt(k0s) + 2.0));
        floor_rank = max(floor_rank, max(1u, ns_total / 50u));
        uint32_t b = find_bin(floor_rank);
        if (budget_pairs) b = min(b, sh_gbin);
        // never more than the top eighth of the layer: the bin that holds the entry of that rank is spilled only
        // if all of it still lies inside (a layer's candidate region has room for a little more than that share)
        const uint32_t k8 = max(1u, ns_total / 8u);
        uint32_t bc = find_bin(k8);
        if ((bc == 0u ? ns_total : above[bc - 1u]) > k8) ++bc;     // D1_BINS: nothing is spilled
        sh_spill = max(b, bc);
    }
    __syncthreads();
    const uint32_t spill_bin = sh_spill;
    // (3) bins that may hold a candidate's boundary: +-5 sigma of the sample rank, every bin in between.
    // Bin 0 (zeros and the tiniest denormals) never gets a slot here: its squares need the exact
    // accumulators of the full recount.
    if (tid < J) {
        const uint32_t K = Ktab[(size_t)li * J + tid];
        if (K < L.n) {
            const double ks = (double)K / scale;
            const double sg = sqrt(fmax(0.0, ks * (1.0 - ks / (double)ns_total)));
            const double klo = floor(ks - 5.0 * sg) - 2.0, khi = ceil(ks + 5.0 * sg) + 2.0;
            const uint32_t rlo = (uint32_t)fmin((double)ns_total, fmax(1.0, klo));
            const uint32_t rhi = (uint32_t)fmin((double)ns_total, fmax(1.0, khi));
            const uint32_t btop = find_bin(rlo), bbot = khi > (double)ns_total ? 0u : find_bin(rhi);
            // A boundary in the spilled range can also be resolved from the candidates, which is
            // cheap only where few entries lie above it: skip the prediction for the sparse top
            // (fewer than 64 sample entries above), where it would cost many bins.
            const bool sparse_top = ks < 64.0 && bbot >= spill_bin;
            if (!sparse_top)
                for (uint32_t b = max(bbot, 1u); b <= btop; ++b) atomicOr(&bitmap[b >> 5], 1u << (b & 31));
        }
    }
    __syncthreads();
    // (4) slots: one run of consecutive bins from the lowest marked bin (low bins hold the most
    // entries) to the highest, at most PRE_SLOTS.  A run lets the streaming pass find an entry's slot
    // with a subtraction instead of a table look-up; what is cut off at the top lies in the spilled
    // range or makes the layer a redo.
    uint8_t* lut = pb.lut1 + (size_t)big * D1_BINS;
    for (uint32_t b = tid; b < D1_BINS; b += 256) lut[b] = (uint8_t)NO_SLOT;
    __syncthreads();
    // lowest and highest marked bin: one bitmap word per thread
    if (tid == 0) { sh_gbin = D1_BINS; sh_ns = 0u; }      // reused: lowest / highest marked bin
    __syncthreads();
    if (tid < D1_BINS / 32) {
        const uint32_t m = bitmap[tid];
        if (m) {
            atomicMin(&sh_gbin, tid * 32u + (uint32_t)__ffs((int)m) - 1u);
            atomicMax(&sh_ns, tid * 32u + 31u - (uint32_t)__clz((int)m));
        }
    }
    __syncthreads();
    uint32_t lo_bin = sh_gbin, ns = 0;
    if (lo_bin < D1_BINS) ns = min(PRE_SLOTS, sh_ns - lo_bin + 1u); else lo_bin = 0;
    if (tid < ns) {
        lut[lo_bin + tid] = (uint8_t)tid;
        pb.slot_bin[(size_t)big * SLOT_STRIDE + tid] = lo_bin + tid;
    }
    if (tid == 0) {
        LayerState st;
        st.spill_bin = spill_bin; st.nslots_d = ns; st.nslots_t = 0; st.redo = 0;
        st.spill_cnt = 0; st.spill_valid = 0; st.slot_lo = lo_bin; st.pad = 0;
        pb.state[big] = st;
    }
    if (fold_zero) {
        // chunk records start out as "nothing spilled": every workgroup clears an equal share of all layers' records
        // (a layer's own workgroup clearing them made the largest layer's the last to finish by far)
        const uint32_t per = (pb.nchunks_total + gridDim.x - 1u) / gridDim.x;
        const uint32_t c_lo = big * per, c_hi = min(pb.nchunks_total, c_lo + per);
        for (uint32_t c = c_lo + tid; c < c_hi; c += 256) pb.rec_cnt[c] = 0u;
        if (tid == 0) { pb.layer_flag[big] = 0u; pb.cursor[big] = 0u; pb.spill_over[big] = 0u; }
        if (big == 0u && tid < 4u) pb.diag[tid] = 0u;
        if (big == 0u && tid == 4u) *pb.fresh = 0u;
    }
}

// ---------------------------------------------------------------------------------------------
// The streaming pass.  Persistent grid: workgroup w owns a contiguous range of chunks, walks it
// layer by layer, and keeps that layer's histograms in LDS as one array of packed entries
// [count:20 | sum:44] of (significand^2 >> 24): 4096 digit-1 bins, then up to PRE_SLOTS slots x 128 digit-2
// bins.  Entries whose bin has a slot are counted only there.  Bin 0 (zeros, tiniest denormals)
// keeps exact squares in a separate accumulator.  One wave handles one chunk at a time: 4 quads per
// lane, one LDS atomic per entry, then spilling, ranked by prefix scans over the lanes, of the entries at or above the layer's
// spill bin, staged through LDS so that the candidate writes are coalesced.
//
// The packed sums drop the low 24 bits of each square: the true sum of (square >> 16) lies in
// [256 S, 256 S + 256 count); k_reduce_parts stores the midpoint and the scans widen their bounds by
// half that interval (2^-23 relative).
constexpr uint32_t PK_ENTRIES = D1_BINS + PRE_SLOTS * D2_BINS;     // 17920 entries, 140 KB
constexpr uint32_t STAGE = 128;                                    // candidates a wave stages per round
constexpr uint32_t PART_STRIDE = PK_ENTRIES + 8;                   // entries of one part: the LDS array, then the bin-0 sum

__device__ __forceinline__ unsigned long long pk_term(uint32_t key) {
    const uint32_t m = key & 0x7FFFFFu, e = key >> 23;
    const uint32_t m24 = e ? (m | 0x800000u) : m;
    return e == 255u ? (unsigned long long)(m != 0u) : ((unsigned long long)m24 * m24) >> PK_SHIFT;
}

struct MainCtx {
    unsigned long long* pk;
    unsigned long long* sq0;
    uint32_t lo19;         // 19-bit key prefix of the first digit-2 entry of the first slot
    uint32_t span;         // digit-2 entries of all slots: a key is in a slot bin iff (key >> 12) - lo19 < span
    uint32_t spill_key;
};

// LDS entry of a key: inside the run of slot bins the digit-2 entries of consecutive bins are
// consecutive 19-bit prefixes, so the entry is the prefix minus the run's first one
__device__ __forceinline__ uint32_t main_entry(const MainCtx& cx, uint32_t k) {
    const uint32_t rel = (k >> D2_SHIFT) - cx.lo19;
    return rel < cx.span ? D1_BINS + rel : (k >> D1_SHIFT);
}

// histogram updates and spill flags of one chunk.  A chunk that lies inside the layer and holds
// only normal numbers (no zeros, denormals, Inf, NaN) takes a branch-free path.
__device__ __forceinline__ void main_count(const MainCtx& cx, const float (&x)[NQ][4], uint32_t valid,
                                           uint32_t (&selm)[NQ]) {
    // exponent field 0 or 255 anywhere in the lane's 16 keys: smallest and largest key
    uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
    for (int u = 0; u < (int)NQ; ++u) {
        const uint32_t k0 = key_of(x[u][0]), k1 = key_of(x[u][1]), k2 = key_of(x[u][2]), k3 = key_of(x[u][3]);
        kmin = min(min(kmin, k0), min(min(k1, k2), k3));
        kmax = max(max(kmax, k0), max(max(k1, k2), k3));
    }
    const bool special = kmin < 0x00800000u || kmax >= 0x7F800000u;
    const bool plain = ballot(special || valid != (1u << (4 * NQ)) - 1u) == 0;
    if (plain) {
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) {
            uint32_t sel = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t k = key_of(x[u][c]);
                const uint32_t m24 = (k & 0x7FFFFFu) | 0x800000u;
                // the shifted square has 24 bits: as a 32-bit value it is the low word of the packed
                // operand and the count's 1 is a constant high word
                const unsigned long long sq = (unsigned long long)m24 * m24;
                const uint32_t t = __builtin_amdgcn_alignbit((uint32_t)(sq >> 32), (uint32_t)sq, PK_SHIFT);
                atomicAdd(&cx.pk[main_entry(cx, k)], PK_ONE | (unsigned long long)t);
                sel |= (k >= cx.spill_key ? 1u : 0u) << c;
            }
            selm[u] = sel;
        }
        return;
    }
#pragma unroll
    for (int u = 0; u < (int)NQ; ++u) {
        selm[u] = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (!(valid & (1u << (4 * u + c)))) continue;
            const uint32_t k = key_of(x[u][c]);
            if ((k >> D1_SHIFT) != 0u) {
                atomicAdd(&cx.pk[main_entry(cx, k)], PK_ONE | pk_term(k));
            } else {
                atomicAdd(&cx.pk[0], PK_ONE);
                if (k) atomicAdd(cx.sq0, sq_exact(k));
            }
            if (k >= cx.spill_key) selm[u] |= 1u << c;
        }
    }
}

// Spilling without global stores in the steady state.  A store in the loop would make every wait
// for the next chunk's loads a wait for the store acknowledgements as well, and a returning global
// atomic per reservation serialises thousands of waves on one address.  So:
//   * the workgroup owns the slice of the layer's candidate region that corresponds to its chunks
//     (REGION_PER_CHUNK entries of space per chunk, a third more than the largest share of a layer
//     that k_predict lets spill), handed out in units of SPILL_UNIT entries; a slice that still runs
//     out marks the layer's spill as incomplete (spill_over) and the layer is served by the passes
//     that read g and h instead, like any other misprediction;
//   * a wave takes blocks of 128 entries from an LDS cursor, fills its current block in an LDS window,
//     and writes the window out with coalesced stores only when the next chunk does not fit (a chunk
//     with more than a block's worth takes exactly what it needs, rounded up to the unit);
//   * chunk records wait in LDS until that flush.  A chunk's candidates are always contiguous.
constexpr uint32_t PEND = 16;                   // chunk records a wave holds back

struct WaveSpill {
    uint2* win;           // LDS window of the current block: (index, bits of x)
    uint32_t* pend;       // LDS: PEND x (chunk, start, count)
    uint32_t* lds_cursor; // blocks handed out in this workgroup's slice
    uint32_t* over;       // the layer's spill_over flag
    uint32_t slice_units; // units of SPILL_UNIT entries the slice holds
    uint32_t slice_rel;   // first entry of the slice, relative to the layer's region (chunk records are region-relative)
    uint32_t blk;         // region-relative start of the current block (valid if have_blk)
    uint32_t fill;        // entries in the window
    uint32_t flushed;     // of which already written
    uint32_t npend;
    bool have_blk;
};

__device__ __forceinline__ void spill_flush(const ProfileBuffers& pb, WaveSpill& ws, uint64_t tmp0) {
    const uint32_t lane = lane_id();
    wave_sync_lds();
    if (ws.have_blk) {
        for (uint32_t k = ws.flushed + lane; k < ws.fill; k += 64) {
            const uint64_t o = tmp0 + ws.blk + k;
            const uint2 e = ws.win[k];
            pb.tmp_idx[o] = e.x;
            pb.tmp_x[o] = __uint_as_float(e.y);
        }
        ws.flushed = ws.fill;
    }
    if (lane < ws.npend) {
        const uint32_t chunk = ws.pend[3 * lane];
        pb.rec_start[chunk] = ws.pend[3 * lane + 1];
        pb.rec_cnt[chunk] = ws.pend[3 * lane + 2];
    }
    ws.npend = 0;
    wave_sync_lds();
}

// take room for `entries` consecutive entries of the slice; returns the region-relative index of the
// first.  *ok is false when the slice has no room left for them: nothing may be written then, and the
// layer is marked.
constexpr uint32_t SPILL_UNIT = 8;
__device__ __forceinline__ uint32_t spill_take(WaveSpill& ws, uint32_t entries, bool* ok) {
    const uint32_t nu = (entries + SPILL_UNIT - 1u) / SPILL_UNIT;
    uint32_t b = 0;
    if (lane_id() == 0) b = atomicAdd(ws.lds_cursor, nu);
    b = __builtin_amdgcn_readfirstlane(b);
    *ok = b + nu <= ws.slice_units;             // (the cursor grows by at most 128 units per chunk: no wrap)
    if (!*ok && lane_id() == 0) *ws.over = 1u;
    return ws.slice_rel + b * SPILL_UNIT;
}

// One chunk of the streaming pass for one wave: histogram updates, ranks of the entries to spill,
// space for them, window writes, chunk record.
__device__ __forceinline__ void main_chunk(const ProfileBuffers& pb, const MainCtx& cx, const LayerDesc& L, WaveSpill& ws,
                                           uint32_t chunk, const float (&x)[NQ][4], uint32_t valid) {
    const uint32_t lane = lane_id();
    const uint32_t vbase = (chunk - L.chunk0) * CHUNK;
    uint32_t selm[NQ];
    main_count(cx, x, valid, selm);
    // ranks in index order (quad, lane, element): per quad a prefix sum over the lanes of the lane's
    // count (0..4); two quads share a scan in 16-bit fields (a quad holds at most 256)
    static_assert(NQ == 4, "two packed scans cover four quads");
    const uint32_t n0 = __popc(selm[0]), n1 = __popc(selm[1]), n2 = __popc(selm[2]), n3 = __popc(selm[3]);
    const uint32_t s01 = wave_scan_add_u32(n0 | (n1 << 16)), s23 = wave_scan_add_u32(n2 | (n3 << 16));
    const uint32_t t01 = (uint32_t)__builtin_amdgcn_readlane((int)s01, 63), t23 = (uint32_t)__builtin_amdgcn_readlane((int)s23, 63);
    const uint32_t t0 = t01 & 0xFFFFu, t1 = t01 >> 16, t2 = t23 & 0xFFFFu;
    const uint32_t total = t0 + t1 + t2 + (t23 >> 16);
    uint32_t rowbase[NQ];
    rowbase[0] = (s01 & 0xFFFFu) - n0;
    rowbase[1] = t0 + (s01 >> 16) - n1;
    rowbase[2] = t0 + t1 + (s23 & 0xFFFFu) - n2;
    rowbase[3] = t0 + t1 + t2 + (s23 >> 16) - n3;
    if (total == 0) return;                      // records start out as "nothing spilled"
    if (total <= STAGE) {
        if (!ws.have_blk || ws.fill + total > STAGE || ws.npend == PEND) {
            spill_flush(pb, ws, L.tmp0);
            if (!ws.have_blk || ws.fill + total > STAGE) {
                bool ok;
                ws.blk = spill_take(ws, STAGE, &ok);
                ws.fill = 0; ws.flushed = 0; ws.have_blk = ok;
                if (!ok) return;                 // the chunk's record stays "nothing spilled"; the layer is marked
            }
        }
        const uint32_t at = ws.fill;
        // Few entries are spilled, so a lane rarely holds more than one per quad: write in rounds,
        // every lane its next selected entry of the quad (ascending element), until no lane has one
        // left.  On average that is fewer than two wave-wide writes per quad instead of four.
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) {
            uint32_t m = selm[u];
            uint32_t pos = at + rowbase[u];
            const uint32_t idx0 = vbase + u * 256u + lane * 4u - L.mis;
            while (ballot(m != 0u)) {
                if (m) {
                    const float xv = (m & 1u) ? x[u][0] : (m & 2u) ? x[u][1] : (m & 4u) ? x[u][2] : x[u][3];
                    ws.win[pos] = make_uint2(idx0 + (uint32_t)__builtin_ctz(m), __float_as_uint(xv));
                    ++pos;
                    m &= m - 1u;
                }
            }
        }
        if (lane == 0) {
            ws.pend[3 * ws.npend] = chunk;
            ws.pend[3 * ws.npend + 1] = ws.blk + at;
            ws.pend[3 * ws.npend + 2] = total;
        }
        ws.fill += total;
        ws.npend += 1;
    } else {
        // a dense chunk: its own run of blocks, written through the window in rounds
        spill_flush(pb, ws, L.tmp0);
        ws.have_blk = false;
        bool ok;
        const uint32_t start = spill_take(ws, total, &ok);
        if (!ok) return;
        const uint64_t base = L.tmp0 + start;
        for (uint32_t r0 = 0; r0 < total; r0 += STAGE) {
#pragma unroll
            for (int u = 0; u < (int)NQ; ++u) {
                uint32_t pos = rowbase[u];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    if (selm[u] & (1u << c)) {
                        const uint32_t k = pos - r0;
                        if (k < STAGE) {
                            ws.win[k] = make_uint2(vbase + u * 256u + lane * 4u + c - L.mis, __float_as_uint(x[u][c]));
                        }
                        ++pos;
                    }
                }
            }
            wave_sync_lds();
#pragma unroll
            for (uint32_t k = lane; k < STAGE; k += 64) {
                if (r0 + k < total) {
                    const uint64_t o = base + r0 + k;
                    const uint2 e = ws.win[k];
                    pb.tmp_idx[o] = e.x;
                    pb.tmp_x[o] = __uint_as_float(e.y);
                }
            }
            wave_sync_lds();
        }
        if (lane == 0) { pb.rec_start[chunk] = start; pb.rec_cnt[chunk] = total; }
    }
}

__global__ __launch_bounds__(FUSED_THREADS) void k_main(ProfileBuffers pb, uint32_t chunks_per_wg) {
    __shared__ __align__(16) unsigned long long pk[PK_ENTRIES];   // 140 KB
    __shared__ unsigned long long sq0;
    __shared__ uint2 stage[FUSED_WAVES * STAGE];                  // 16 KB: per-wave block windows
    __shared__ uint32_t pend[FUSED_WAVES * PEND * 3];             // 3 KB
    __shared__ uint32_t lds_cursor;
    __shared__ uint32_t next_chunk;                               // first chunk of the segment no wave has taken yet
    const uint32_t tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t c_begin = blockIdx.x * chunks_per_wg;
    const uint32_t c_end = min(pb.nchunks_total, c_begin + chunks_per_wg);
    uint32_t cur = c_begin;
    uint32_t part = pb.wg_part0[blockIdx.x];
    while (cur < c_end) {
        const uint32_t big = pb.chunk_big[cur];
        const uint32_t li = pb.big_layer[big];
        const LayerDesc L = pb.layers[li];
        const LayerState st = pb.state[big];
        const uint32_t seg_end = min(min(c_end, L.chunk0 + L.nchunks), cur + PK_MAX_CHUNKS);
        const uint32_t used = D1_BINS + st.nslots_d * D2_BINS;
        for (uint32_t b = tid; b < used; b += FUSED_THREADS) pk[b] = 0ull;
        if (tid == 0) { sq0 = 0ull; lds_cursor = 0u; next_chunk = cur + FUSED_WAVES; }
        __syncthreads();
        MainCtx cx;
        cx.pk = pk; cx.sq0 = &sq0;
        cx.lo19 = st.slot_lo << (D1_SHIFT - D2_SHIFT); cx.span = st.nslots_d * D2_BINS;
        cx.spill_key = st.spill_bin >= D1_BINS ? 0x80000000u : (st.spill_bin << D1_SHIFT);
        WaveSpill ws;
        ws.win = stage + wave * STAGE;
        ws.pend = pend + wave * PEND * 3; ws.lds_cursor = &lds_cursor;
        ws.over = pb.spill_over + big;
        ws.slice_rel = (cur - L.chunk0) * REGION_PER_CHUNK;
        ws.slice_units = (seg_end - cur) * (REGION_PER_CHUNK / SPILL_UNIT);
        ws.blk = 0; ws.fill = 0; ws.flushed = 0; ws.npend = 0; ws.have_blk = false;

        // (Fetching the wave's next chunk while the current one is worked on was tried at 16, 12 and 8
        // waves per workgroup: no gain.  Measured with one thing removed at a time, the candidate and
        // record stores cost this pass 4 % and the histogram atomics nothing; a workgroup streams its
        // share about as fast as a bare loop of the same loads does.  The pass ends with its slowest
        // workgroup, a tenth behind the average.)
        // Waves take chunks from a counter, not in a fixed rotation: a wave's pace varies with what it
        // finds (spills, flushes, memory), and with fixed shares the segment's end waited for its slowest
        // wave for a good tenth of the pass.  The next chunk is asked for before the current one is
        // worked on, so the counter's round trip is never waited for.  No result depends on which wave
        // had which chunk.
        uint32_t chunk = cur + wave;
        while (chunk < seg_end) {
            uint32_t taken = 0;
            if (lane_id() == 0) taken = atomicAdd(&next_chunk, 1u);
            QuadGH q[NQ];
            float x[NQ][4];
            uint32_t valid = 0;
            load_chunk<NQ>(L, (chunk - L.chunk0) * CHUNK, q, valid);
#pragma unroll
            for (int u = 0; u < (int)NQ; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) x[u][c] = q[u].g[c] - q[u].h[c];
            main_chunk(pb, cx, L, ws, chunk, x, valid);
            chunk = __builtin_amdgcn_readfirstlane(taken);
        }
        spill_flush(pb, ws, L.tmp0);
        __syncthreads();
        // This segment's histogram goes out as it is, with plain coalesced stores, as one "part" of the
        // layer; k_reduce_parts adds the parts up.  (Adding into the layer's arrays with global atomics
        // from here held every workgroup of a layer up on the same cache lines at the same moment.)
        ulonglong2* out = reinterpret_cast<ulonglong2*>(pb.parts + (size_t)part * PART_STRIDE);
        const ulonglong2* pk2 = reinterpret_cast<const ulonglong2*>(pk);
        for (uint32_t b = tid; b < used / 2u; b += FUSED_THREADS) out[b] = pk2[b];   // `used` is even
        if (tid == 0) pb.parts[(size_t)part * PART_STRIDE + PK_ENTRIES] = sq0;
        ++part;
        // the next segment clears the LDS array: its reads above must be done, the stores need not be
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        cur = seg_end;
    }
}

// ---------------------------------------------------------------------------------------------
// Sum of a layer's parts, written in the layout the scans read: digit-1 counts and sums, then the
// digit-2 tables of all SLOT_STRIDE slots (zero beyond the slots the pass counted, where k_hist2c
// adds).  Counts as they are; sums as midpoints in units of 2^16 (exponent 255: the NaN count;
// bin 0: the exact squares).  One thread per entry, the parts' loads issued four at a time.
constexpr uint32_t LAYER_ENTRIES = D1_BINS + SLOT_STRIDE * D2_BINS;
constexpr uint32_t REDUCE_ENTRIES = 128;        // entries per workgroup: two per lane, each of the 4 waves takes a quarter of the parts
__global__ __launch_bounds__(256) void k_reduce_parts(ProfileBuffers pb) {
    __shared__ unsigned long long sh_c[3][REDUCE_ENTRIES], sh_t[3][REDUCE_ENTRIES];
    const uint32_t big = blockIdx.y, lane = threadIdx.x & 63u, w = threadIdx.x >> 6;
    const uint32_t e = blockIdx.x * REDUCE_ENTRIES + 2u * lane;     // and e + 1; `used` is even
    // The totals over the layers that the prediction of this profile read are done with (that launch has ended), and
    // the scan that follows this one adds the new ones up: cleared here, between the two.
    if (blockIdx.x == 0u && big == 0u)
        for (uint32_t b = threadIdx.x; b < D1_BINS; b += 256u) pb.gprev[b] = 0ull;
    const uint32_t used = D1_BINS + pb.state[big].nslots_d * D2_BINS;
    const uint32_t p0 = pb.big_part0[big], np = pb.big_nparts[big];
    unsigned long long cnt[2] = {0, 0}, t[2] = {0, 0};
    if (e < used) {
        const unsigned long long* src = pb.parts + (size_t)p0 * PART_STRIDE + e;
        auto take = [&](const ulonglong2 v) {
            cnt[0] += v.x >> 44; t[0] += v.x & PK_MASK;
            cnt[1] += v.y >> 44; t[1] += v.y & PK_MASK;
        };
        auto part = [&](uint32_t k) { return *reinterpret_cast<const ulonglong2*>(src + (size_t)k * PART_STRIDE); };
        uint32_t k = w;
        for (; k + 12 < np; k += 16) {
            const ulonglong2 v0 = part(k), v1 = part(k + 4), v2 = part(k + 8), v3 = part(k + 12);
            take(v0); take(v1); take(v2); take(v3);
        }
        for (; k < np; k += 4) take(part(k));
    }
    if (w) {
        sh_c[w - 1][2 * lane] = cnt[0]; sh_c[w - 1][2 * lane + 1] = cnt[1];
        sh_t[w - 1][2 * lane] = t[0]; sh_t[w - 1][2 * lane + 1] = t[1];
    }
    __syncthreads();
    if (w || e >= LAYER_ENTRIES) return;
#pragma unroll
    for (int q = 0; q < 3; ++q) {
        cnt[0] += sh_c[q][2 * lane]; cnt[1] += sh_c[q][2 * lane + 1];
        t[0] += sh_t[q][2 * lane]; t[1] += sh_t[q][2 * lane + 1];
    }
    unsigned long long slot_sq = 0;               // this lane's share of the slot's total (blocks beyond the digit-1 bins)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const uint32_t eu = e + (uint32_t)u;
        unsigned long long s2 = 0;
        if (cnt[u]) {
            const uint32_t bin = eu < D1_BINS ? eu : pb.slot_bin[(size_t)big * SLOT_STRIDE + (eu - D1_BINS) / D2_BINS];
            if ((bin >> 4) == 255u) {
                s2 = t[u];
            } else if (eu == 0u) {
                for (uint32_t q = 0; q < np; ++q) s2 += pb.parts[(size_t)(p0 + q) * PART_STRIDE + PK_ENTRIES];
            } else {
                s2 = (t[u] << 8) + (cnt[u] << 7);
            }
        }
        if (eu < D1_BINS) {
            pb.cnt1[(size_t)big * D1_BINS + eu] = (uint32_t)cnt[u];
            reinterpret_cast<unsigned long long*>(pb.sq1)[(size_t)big * D1_BINS + eu] = s2;
        } else {
            const size_t o = (size_t)big * SLOT_STRIDE * D2_BINS + (eu - D1_BINS);
            pb.cnt2[o] = (uint32_t)cnt[u];
            reinterpret_cast<unsigned long long*>(pb.sq2)[o] = s2;
            slot_sq += s2;
        }
    }
    // a workgroup beyond the digit-1 bins holds exactly one slot: its totals, which stand for the slot's bin in the
    // digit-1 histogram (the pass counts an entry of a slot bin in the slot only), go out with it
    static_assert(REDUCE_ENTRIES == D2_BINS && D1_BINS % REDUCE_ENTRIES == 0, "one workgroup per slot");
    if (blockIdx.x >= D1_BINS / REDUCE_ENTRIES) {
        unsigned long long slot_cnt = cnt[0] + cnt[1];
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) {
            slot_cnt += __shfl_xor(slot_cnt, d, 64);
            slot_sq += __shfl_xor(slot_sq, d, 64);
        }
        if (lane == 0) {
            const size_t o = (size_t)big * SLOT_STRIDE + (blockIdx.x - D1_BINS / REDUCE_ENTRIES);
            pb.slot_cnt[o] = (uint32_t)slot_cnt;
            pb.slot_sq[o] = slot_sq;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// After the pass: exact digit-1 histogram (slot bins contribute the totals of their digit-2
// bins), boundary bin per candidate, and what each boundary needs:
//   - its bin already has a slot                          -> nothing
//   - its bin is in the spilled range                     -> a slot PRE_SLOTS.. filled from the candidates
//   - neither (prediction missed), or slots run out       -> redo: exact slots, full recount
__global__ __launch_bounds__(256) void k_scan1x(ProfileBuffers pb, const uint32_t* Ktab, uint32_t J) {
    __shared__ uint32_t cnt[D1_BINS];
    __shared__ uint32_t above[D1_BINS];
    __shared__ double below[D1_BINS];
    __shared__ uint32_t su[16];
    __shared__ double sd[16];
    __shared__ uint32_t tbin[MAX_SLOTS];
    __shared__ uint8_t lut[D1_BINS];
    __shared__ uint32_t sh_redo;
    __shared__ uint32_t slot_c[PRE_SLOTS];
    __shared__ unsigned long long slot_s[PRE_SLOTS];
    const uint32_t tid = threadIdx.x, big = blockIdx.x;
    const uint32_t li = pb.big_layer[big];
    const LayerDesc L = pb.layers[li];
    LayerState st = pb.state[big];
    const uint32_t* gcnt = pb.cnt1 + (size_t)big * D1_BINS;
    const uint64_t* gsq = pb.sq1 + (size_t)big * D1_BINS;
    uint8_t* glut = pb.lut1 + (size_t)big * D1_BINS;
    uint8_t* glutc = pb.lutc + (size_t)big * D1_BINS;
    // this thread's sixteen digit-1 entries: asked for now, with the table and the slot totals below, so
    // that the three groups of loads share one memory round trip instead of taking one per phase
    uint4 craw[4];
    ulonglong2 sraw[8];
    {
        const uint4* c4 = reinterpret_cast<const uint4*>(gcnt + tid * 16u);
        const ulonglong2* s2 = reinterpret_cast<const ulonglong2*>(gsq + tid * 16u);
#pragma unroll
        for (int k = 0; k < 4; ++k) craw[k] = c4[k];
#pragma unroll
        for (int k = 0; k < 8; ++k) sraw[k] = s2[k];
    }
    {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(glut);
        uint32_t* dst = reinterpret_cast<uint32_t*>(lut);
        for (uint32_t b = tid; b < D1_BINS / 4; b += 256) dst[b] = src[b];
    }
    // totals of the slots the pass counted (k_reduce_parts summed them)
    static_assert(PRE_SLOTS <= 256, "one thread per slot");
    if (tid < st.nslots_d) {
        slot_c[tid] = pb.slot_cnt[(size_t)big * SLOT_STRIDE + tid];
        slot_s[tid] = pb.slot_sq[(size_t)big * SLOT_STRIDE + tid];
    }
    if (tid == 0) sh_redo = 0u;
    __syncthreads();
    uint32_t c[16];
    double s[16];
    uint32_t csum = 0;
    double ssum = 0.0;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const uint32_t b = tid * 16u + k;
        const uint32_t slot = lut[b];
        const uint4 cq = craw[k >> 2];
        uint32_t cc = (k & 3) == 0 ? cq.x : (k & 3) == 1 ? cq.y : (k & 3) == 2 ? cq.z : cq.w;
        unsigned long long ss = (k & 1) ? sraw[k >> 1].y : sraw[k >> 1].x;
        if (slot != NO_SLOT) { cc += slot_c[slot]; ss += slot_s[slot]; }
        c[k] = cc;
        s[k] = sq_to_double(b, ss, cc);
        csum += cc;
        ssum += s[k];
    }
    {
        // the exact histogram stays for the next profile's prediction, with its sum over the layers
        uint4* hp = reinterpret_cast<uint4*>(pb.hprev + (size_t)big * D1_BINS + tid * 16u);
#pragma unroll
        for (int k = 0; k < 4; ++k) hp[k] = make_uint4(c[4 * k], c[4 * k + 1], c[4 * k + 2], c[4 * k + 3]);
    }
    uint32_t ctot;
    const uint32_t cex = block_exclusive_scan<uint32_t>(csum, su, &ctot);
    const double sex = block_exclusive_scan<double>(ssum, sd, nullptr);
    {
        uint32_t run_c = cex;
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
    }
    for (uint32_t b = tid; b < D1_BINS; b += 256) glutc[b] = (uint8_t)NO_SLOT;
    __syncthreads();
    // the sum over the layers: neighbouring lanes add to neighbouring bins (a lane adding its own sixteen bins
    // touched 64 cache lines per instruction, and the additions of all layers queue up on the same lines)
    for (uint32_t b = tid; b < D1_BINS; b += 256) {
        const uint32_t cb = cnt[b];
        if (cb) atomicAdd(&pb.gprev[b], (unsigned long long)cb);
    }

    const uint32_t spill_cnt = st.spill_bin >= D1_BINS ? 0u
                             : (st.spill_bin == 0u ? ctot : above[st.spill_bin - 1u]);
    const bool spill_valid = pb.spill_over[big] == 0u;
    if (tid < J) {
        const uint32_t K = Ktab[(size_t)li * J + tid];
        uint32_t bin = 0xFFFFFFFFu;
        if (K != 0u && K < L.n) {
            uint32_t lo = 0, hi = D1_BINS - 1;
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (above[mid] < K) hi = mid; else lo = mid + 1;
            }
            bin = lo;
            pb.tgt_r[(size_t)li * J + tid] = K - above[bin];
            pb.tgt_above1[(size_t)li * J + tid] = above[bin];
            pb.tgt_below[(size_t)li * J + tid] = below[bin];
            if (lut[bin] == NO_SLOT && !(spill_valid && bin >= st.spill_bin)) atomicOr(&sh_redo, 1u);
        }
        tbin[tid] = bin;
    }
    __syncthreads();
    // Slots for the boundary bins, by the first wave: lane j holds candidate j.  Candidates ascend in
    // K, so their boundary bins never ascend and equal bins are adjacent: a run of equal bins starts
    // where the bin differs from the lane before, and its number among the runs is a prefix count.
    uint32_t bin = 0xFFFFFFFFu, pslot = NO_SLOT;
    bool valid = false, newrun = false;
    uint64_t heads_c = 0;
    if (tid < 64) {
        if (tid < J) bin = tbin[tid];
        valid = bin != 0xFFFFFFFFu;
        if (valid) pslot = lut[bin];                       // slot fixed before the pass, if any
        const uint32_t prevbin = __shfl_up(bin, 1, 64);
        newrun = valid && (tid == 0 || prevbin != bin);
        heads_c = ballot(newrun && pslot == NO_SLOT);      // runs that need a slot filled from the candidates
        if (tid == 0 && (uint32_t)__popcll(heads_c) > SLOT_STRIDE - PRE_SLOTS) sh_redo = 1u;
    }
    __syncthreads();
    const bool redo = sh_redo != 0u;
    if (redo) {
        // exact slots for every boundary bin; their digit-2 counts are recounted by a full pass
        for (uint32_t b = tid; b < D1_BINS; b += 256) glut[b] = (uint8_t)NO_SLOT;
        uint32_t* c2 = pb.cnt2 + (size_t)big * SLOT_STRIDE * D2_BINS;
        unsigned long long* s2 = reinterpret_cast<unsigned long long*>(pb.sq2) + (size_t)big * SLOT_STRIDE * D2_BINS;
        for (uint32_t e = tid; e < PRE_SLOTS * D2_BINS; e += 256) { c2[e] = 0u; s2[e] = 0ull; }
        __syncthreads();
    }
    if (tid < 64) {
        const uint64_t upto = (2ull << tid) - 1ull;        // this lane and the lanes before it
        const uint64_t heads_all = ballot(newrun);
        uint32_t slot = NO_SLOT;
        if (redo) {
            if (valid) slot = (uint32_t)__popcll(heads_all & upto) - 1u;
            if (newrun) {
                glut[bin] = (uint8_t)slot;
                pb.slot_bin[(size_t)big * SLOT_STRIDE + slot] = bin;
            }
        } else if (valid) {
            if (pslot != NO_SLOT) {
                slot = pslot;
            } else {
                slot = PRE_SLOTS + (uint32_t)__popcll(heads_c & upto) - 1u;
                if (newrun) {
                    glutc[bin] = (uint8_t)slot;
                    pb.slot_bin[(size_t)big * SLOT_STRIDE + slot] = bin;
                }
            }
        }
        if (tid < J) pb.tgt_slot[(size_t)li * J + tid] = slot;
        if (tid == 0) {
            if (redo) atomicAdd(&pb.diag[3], 1u);
            const uint32_t nd = redo ? (uint32_t)__popcll(heads_all) : st.nslots_d;
            st.nslots_d = nd; st.nslots_t = redo ? 0u : (uint32_t)__popcll(heads_c); st.redo = redo ? 1u : 0u;
            st.spill_cnt = spill_cnt; st.spill_valid = spill_valid ? 1u : 0u;
            pb.state[big] = st;
            pb.nslots[big] = nd;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Digit-2 histograms of the slots PRE_SLOTS.. from the candidate buffer.  Four lanes per chunk: the kernel is bound
// by how many loads its waves keep in flight (eight per lane here), not by their number.
__global__ __launch_bounds__(256) void k_hist2c(ProfileBuffers pb) {
    constexpr uint32_t S = SUB_HIST;
    const SubGroup g = sub_group<S>();
    const uint32_t chunk = blockIdx.x * (256u / S) + threadIdx.x / S;
    if (chunk >= pb.nchunks_total) return;
    // what the chunk index alone addresses is fetched together; it says where the chunk's candidates are, so the
    // layer's state and the first rounds' candidates are asked for together as well
    const uint32_t big = pb.chunk_big[chunk];
    const uint32_t first = pb.chunk_first[chunk];
    const uint32_t cnt = pb.rec_cnt[chunk];
    const uint32_t start = pb.rec_start[chunk];
    materialise(big); materialise(first); materialise(cnt); materialise(start);
    if (cnt == 0u) return;
    const uint64_t base = region_start(first, big) + start;
    const LayerState st = pb.state[big];
    const uint8_t* lutc = pb.lutc + (size_t)big * D1_BINS;
    uint32_t* c2 = pb.cnt2 + (size_t)big * SLOT_STRIDE * D2_BINS;
    unsigned long long* s2 = reinterpret_cast<unsigned long long*>(pb.sq2) + (size_t)big * SLOT_STRIDE * D2_BINS;
    // Eight rounds at a time: their keys are loaded together, then their slots.  Positions past the
    // chunk's last candidate read that last candidate again (always a valid address) and are dropped.
    constexpr int AHEAD = 8;
    for (uint32_t k0 = g.sub; k0 < cnt; k0 += AHEAD * S) {
        uint32_t key[AHEAD], slot[AHEAD];
#pragma unroll
        for (int t = 0; t < AHEAD; ++t)
            key[t] = key_of(pb.tmp_x[base + min(k0 + (uint32_t)t * S, cnt - 1u)]);
        if (st.redo || st.nslots_t == 0u) return;       // (a layer without such slots: its candidates were asked for in vain)
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) slot[t] = (uint32_t)lutc[key[t] >> D1_SHIFT];
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) {
            if (slot[t] == NO_SLOT || k0 + (uint32_t)t * S >= cnt) continue;
            const uint32_t bin = key[t] >> D1_SHIFT;
            const uint32_t e = slot[t] * D2_BINS + ((key[t] >> D2_SHIFT) & (D2_BINS - 1));
            const unsigned long long s = bin ? (unsigned long long)sq_coarse(key[t]) : sq_exact(key[t]);
            atomicAdd(&c2[e], 1u);
            if (s) atomicAdd(&s2[e], s);
        }
    }
}

}  // namespace kimad
