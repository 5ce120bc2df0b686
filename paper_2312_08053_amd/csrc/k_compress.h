// Selection, compaction and estimator update.
//
// Computes, per layer, the support of TopK_K(x) for x = g - h (paper Section 2.2), writes the
// (index, value) payload that Algorithm 1's worker uploads, and applies h <- h + TopK(x)
// (Section 3.3, Eq. EF21-2).  Equal magnitudes are kept in order of lower index.
//
// Tiled layers: one streaming pass writes every entry whose 19-bit key prefix is >= the layer's
// threshold prefix into a candidate buffer (in index order inside each 1024-element chunk) and
// histograms the last 12 key bits of the entries whose prefix is equal.  Four small kernels then
// fix the exact threshold key and tie quota, count survivors per chunk, scan the chunks in index
// order and write payload and estimator.
#pragma once
#include "common.h"
#include <hip/hip_fp16.h>
#include "k_profile.h"   // LDS sort helpers shared with the small-layer profile

namespace kimad {

struct CompressBuffers {
    const LayerDesc* layers;
    const uint32_t* chunk_layer;  // tile -> layer (a tile holds tile_elems / CHUNK chunks)
    const uint32_t* big_layer;
    const uint32_t* small_layer;
    uint32_t tile_elems;
    uint32_t L, B, J;
    const uint32_t* Ktab;         // [L][J] grid sizes
    // threshold cache written by the profile scans
    const uint32_t* sel_prefix;
    const uint32_t* sel_above;
    const uint32_t* sel_amb;
    // per big layer
    SelRec* sel;                  // [B]
    uint32_t* cursor;             // [B] candidates reserved so far
    uint32_t* hist3;              // [B][4096] last-digit histogram of the ambiguous entries
    uint32_t* tau;                // [B] exact threshold key
    uint32_t* quota;              // [B] entries equal to tau that are kept (lowest indices)
    // per chunk
    uint32_t* rec_start;          // start inside the layer's candidate region
    uint32_t* rec_cnt;            // candidates written
    uint32_t* rec_amb;            // of which ambiguous
    uint32_t* c_gt;               // candidates above tau
    uint32_t* c_eq;               // candidates equal to tau
    uint32_t* o_base;             // first payload slot of the chunk inside the layer
    uint32_t* o_allow;            // ties this chunk may keep
    const uint32_t* chunk_first;  // chunk -> first chunk of its layer (with the big index: where its region starts)
    const uint32_t* cblk_big;     // block of 1024 chunks -> big index
    // candidate buffer
    uint32_t* tmp_idx;
    float* tmp_x;
    uint32_t* ncompact;       // layers whose selection needs the streaming compaction pass
    uint32_t* fresh;          // 1 while the profile's cache describes the current g - h (see ProfileBuffers)
    const LayerState* state;      // fused-profile state (spill range) per big layer
    // outputs
    const uint64_t* K;
    const uint64_t* offsets;
    uint32_t* idx_out;
    float* val_out;               // fp32 values, or binary16 bit patterns (uint16) when value_f16 is set
    uint32_t value_f16;
    uint64_t capacity_pairs;
    uint64_t tmp_total;           // entries of the candidate buffer (all regions)
    int32_t* status;
};

// A kept value as it travels in half precision: binary16, round to nearest even, saturated to +-65504 (never
// infinite), NaN kept.  Returns the bit pattern; *decoded gets the fp32 value the receiver will add.
__device__ __forceinline__ uint16_t value_to_f16(float x, float* decoded) {
    const float c = x != x ? x : fminf(fmaxf(x, -65504.f), 65504.f);
    const __half hv = __float2half_rn(c);
    *decoded = __half2float(hv);
    return __half_as_ushort(hv);
}

// Payload slot o gets value x; returns what the estimator must add: x itself, or its half-precision image.
__device__ __forceinline__ float emit_value(const CompressBuffers& cb, uint64_t o, float x) {
    if (cb.value_f16) {
        float dec;
        reinterpret_cast<uint16_t*>(cb.val_out)[o] = value_to_f16(x, &dec);
        return dec;
    }
    cb.val_out[o] = x;
    return x;
}

// ---------------------------------------------------------------------------------------------
// Per layer: turn K[i] into a selection record using the profile's threshold cache.
// One workgroup; thread b handles big layer b (looping).
__global__ __launch_bounds__(256) void k_lookup(CompressBuffers cb, int32_t err_offgrid, int32_t err_offsets,
                                                int32_t err_stale, uint32_t use_candidates) {
    __shared__ int bad;
    __shared__ uint32_t need_pass;
    const uint32_t tid = threadIdx.x;
    // Thresholds may be reused only if a profile wrote them for the g - h that is there now: the compression
    // itself changes h, so a second call without a new profile in between is refused (status err_stale).
    const bool stale = use_candidates && *cb.fresh != 1u;
    if (tid == 0) { bad = stale ? 3 : 0; need_pass = 0u; }
    __syncthreads();
    // validate offsets / K for every layer
    for (uint32_t i = tid; i < cb.L; i += 256) {
        const uint64_t K = cb.K[i], off = cb.offsets[i];
        if (K > cb.layers[i].n || off > cb.capacity_pairs || K > cb.capacity_pairs - off) atomicMax(&bad, 1);
    }
    __syncthreads();
    const bool offsets_bad = bad == 1;
    __syncthreads();
    for (uint32_t b = tid; b < cb.B; b += 256) {
        SelRec r;
        r.mode = SEL_NONE; r.prefix = 0; r.above = 0; r.amb = 0; r.cap = 0; r.K = 0;
        const uint32_t li = cb.big_layer[b];
        const uint32_t n = cb.layers[li].n;
        r.tmp_base = cb.layers[li].tmp0;
        r.h = cb.layers[li].h;
        r.dst = cb.offsets[li];
        if (!offsets_bad && !stale) {
            const uint32_t K = (uint32_t)cb.K[li];
            r.K = K;
            if (K == 0u) {
                r.mode = SEL_NONE;
            } else if (K == n) {
                r.mode = SEL_DIRECT; r.above = n;        // everything is kept: no candidates, no threshold
            } else {
                // the row of grid sizes is read eight entries at a time (a look-up that stops at the
                // first hit would wait for one load per entry)
                int found = -1;
                for (uint32_t j0 = 0; j0 < cb.J && found < 0; j0 += 8) {
                    uint32_t kt[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) kt[u] = cb.Ktab[(size_t)li * cb.J + min(j0 + (uint32_t)u, cb.J - 1u)];
#pragma unroll
                    for (int u = 7; u >= 0; --u)
                        if (j0 + (uint32_t)u < cb.J && kt[u] == K) found = (int)(j0 + (uint32_t)u);
                }
                if (found < 0) {
                    atomicMax(&bad, 2);
                } else {
                    const size_t t = (size_t)li * cb.J + found;
                    r.prefix = cb.sel_prefix[t];
                    r.above = cb.sel_above[t];
                    r.amb = cb.sel_amb[t];
                    r.cap = cb.layers[li].tmp_cap;
                    const LayerState st = cb.state[b];
                    // every entry at or above the threshold prefix already sits in the candidate buffer
                    const bool in_spill = use_candidates && st.spill_valid && st.spill_bin < D1_BINS &&
                                          r.prefix >= (st.spill_bin << D2_BITS);
                    // The compaction pass writes what lies at or above the threshold prefix into the region; its
                    // waves reserve space in blocks and leave a block's tail unused when the next chunk does not
                    // fit (less than the chunk needs, so at most as much again), and every wave its last block
                    // of a tile.  What would not fit is served from g and h directly.
                    const uint64_t need = 2ull * ((uint64_t)r.above + r.amb) + 4ull * SPILL_BLOCK * cb.layers[li].ntiles;
                    r.mode = in_spill ? SEL_CAND : need <= r.cap ? SEL_PREFIX : SEL_DIRECT;
                }
            }
        }
        cb.sel[b] = r;
        // the classic pass reserves its candidates from zero; the spilled ones keep their records
        if (r.mode != SEL_CAND) cb.cursor[b] = 0u;
        if (r.mode == SEL_PREFIX || r.mode == SEL_DIRECT) atomicAdd(&need_pass, 1u);
    }
    __syncthreads();
    if (tid == 0) *cb.ncompact = bad ? 0u : need_pass;
    if (bad) {
        // refuse the whole call: nothing is written by the later kernels
        for (uint32_t b = tid; b < cb.B; b += 256) { cb.sel[b].mode = SEL_NONE; cb.sel[b].cap = 0; cb.sel[b].K = 0; }
        if (tid == 0) *cb.status = stale ? err_stale : offsets_bad ? err_offsets : err_offgrid;
    } else if (tid == 0) {
        *cb.status = 0;
    }
    // From here on the cache no longer describes g - h (the estimator is about to change, or a selection from
    // scratch has overwritten the cache); a refused call that reuses the profile leaves both as they were.
    if (tid == 0 && (!use_candidates || !bad)) *cb.fresh = 0u;
}

// ---------------------------------------------------------------------------------------------
// Streaming compaction pass (layers whose threshold lies below the spilled range, or all layers
// when no fused profile preceded).  One wave per chunk; a workgroup of 4 waves walks the chunks
// of one tile.  Each lane holds 4 quads (16 elements); positions come from ballots, so
// the candidates of a chunk are written in index order at a range reserved with one atomic.
// Tiles are taken in a grid-stride loop; *cb.ncompact (set by k_lookup) is the number of layers that
// need this pass, so that after a single-pass profile, when the candidates serve every layer, a
// small grid leaves after one load.
// (Workgroups `block` of `nblocks` of the launch that also histograms the spilled candidates: k_candidates.)
__device__ __forceinline__ void compact_tiles(const CompressBuffers& cb, uint32_t ntiles, int32_t err_internal,
                                              uint32_t block, uint32_t nblocks) {
    if (*cb.ncompact == 0u) return;
    const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
    const uint32_t chunks_per_tile = cb.tile_elems / CHUNK;
    for (uint32_t tile = block; tile < ntiles; tile += nblocks) {
    const uint32_t li = cb.chunk_layer[tile];
    const LayerDesc L = cb.layers[li];
    const SelRec S = cb.sel[L.big];
    const uint32_t tile_in_layer = tile - L.tile0;
    uint32_t* hist3 = cb.hist3 + (size_t)L.big * D3_BINS;
    // layers served from the spilled candidates (or with K = 0) need no pass over g, h
    if (S.mode == SEL_NONE || S.mode == SEL_CAND) continue;
    WaveAlloc wa{0u, 0u};

    for (uint32_t cc = wave; cc < chunks_per_tile; cc += 4) {
        const uint32_t chunk_in_layer = tile_in_layer * chunks_per_tile + cc;
        if (chunk_in_layer >= L.nchunks) break;
        const uint32_t chunk = L.chunk0 + chunk_in_layer;
        const uint32_t vbase = chunk_in_layer * CHUNK;
        Quad q[NQ];
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) load_quad(L, vbase + u * 256u + lane * 4u, q[u]);

        // flags: bit c of sel[u] = candidate, of amb[u] = ambiguous
        uint32_t selm[NQ], ambm[NQ];
        uint32_t mine_amb = 0;
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) {
            selm[u] = 0; ambm[u] = 0;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t key = q[u].key[c];
                if (key == KEY_INVALID) continue;
                const uint32_t p = key >> D2_SHIFT;
                const bool all = S.mode == SEL_DIRECT && S.amb == 0u;
                const bool sure = all || p > S.prefix;
                const bool amb = !all && p == S.prefix;
                if (sure || amb) selm[u] |= 1u << c;
                if (amb) { ambm[u] |= 1u << c; ++mine_amb; }
            }
        }
        // wave totals and the exclusive prefix of the lanes' counts, per quad row
        uint32_t total = 0, total_amb = 0;
        uint32_t rowbase[NQ];                   // candidates in earlier rows + earlier lanes of this row
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) {
            const uint32_t cnt = __popc(selm[u]);
            // exclusive prefix over lanes of a small integer: three ballots on its bits
            const uint64_t b0 = ballot(cnt & 1u), b1 = ballot(cnt & 2u), b2 = ballot(cnt & 4u);
            const uint32_t ex = mbcnt(b0) + 2u * mbcnt(b1) + 4u * mbcnt(b2);
            rowbase[u] = total + ex;
            total += __popcll(b0) + 2u * __popcll(b1) + 4u * __popcll(b2);
        }
        {
            uint32_t a = mine_amb;
#pragma unroll
            for (int d = 32; d > 0; d >>= 1) a += __shfl_xor(a, d, 64);
            total_amb = a;
        }
        const bool direct = S.mode == SEL_DIRECT;   // counted only: the later kernels read g and h again
        uint32_t start = 0;
        if (total && !direct) start = wave_reserve(wa, total, &cb.cursor[L.big]);
        // k_lookup sends a layer here only if its region holds every chunk's block; should a reservation
        // still not fit, drop it, never write out of bounds, and report it.
        const uint32_t written = direct ? total : start >= S.cap ? 0u : min(total, S.cap - start);
        if (written != total && lane == 0) atomicMin(cb.status, err_internal);
        if (lane == 0) { cb.rec_start[chunk] = start; cb.rec_cnt[chunk] = written; cb.rec_amb[chunk] = total_amb; }
        if (total == 0) continue;
        const uint64_t base = S.tmp_base + start;
        if (!direct) {
#pragma unroll
        for (int u = 0; u < (int)NQ; ++u) {
            uint32_t pos = rowbase[u];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (selm[u] & (1u << c)) {
                    if ((uint64_t)start + pos < S.cap) {
                        const uint64_t o = base + pos;
                        cb.tmp_idx[o] = vbase + u * 256u + lane * 4u + c - L.mis;
                        cb.tmp_x[o] = q[u].g[c] - q[u].h[c];
                    }
                    ++pos;
                }
            }
        }
        }
        if (total_amb) {
#pragma unroll
            for (int u = 0; u < (int)NQ; ++u) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const bool a = (ambm[u] >> c) & 1u;
                    const uint64_t am = ballot(a);
                    if (am == 0) continue;
                    const uint32_t low = q[u].key[c] & (D3_BINS - 1);
                    // one atomic per wave when every ambiguous lane holds the same key (zeros, constants)
                    const uint32_t first = __shfl(low, __ffsll((long long)am) - 1, 64);
                    const bool uniform = ballot(a && low != first) == 0;
                    if (uniform) {
                        if (lane == (uint32_t)(__ffsll((long long)am) - 1)) atomicAdd(&hist3[first], (uint32_t)__popcll(am));
                    } else if (a) {
                        atomicAdd(&hist3[low], 1u);
                    }
                }
            }
        }
    }
    }
}

// ---------------------------------------------------------------------------------------------
// Last-digit histogram of the spilled candidates that share the threshold prefix (layers in
// SEL_CAND mode).  Four lanes per chunk, eight rounds of candidates per memory round trip.
__device__ __forceinline__ void hist3_candidates(const CompressBuffers& cb, uint32_t nchunks_total,
                                                 const uint32_t* chunk_big, uint32_t block) {
    constexpr uint32_t S = SUB_HIST;
    const SubGroup g = sub_group<S>();
    const uint32_t chunk = block * (256u / S) + threadIdx.x / S;
    uint32_t cnt = 0, prefix = 0;
    uint64_t base = 0;
    uint32_t* hist3 = cb.hist3;
    bool is_cand = false;
    if (chunk < nchunks_total) {
        // what the chunk index alone addresses goes out together, then the layer's record
        const uint32_t b = chunk_big[chunk], first = cb.chunk_first[chunk];
        const uint32_t n_rec = cb.rec_cnt[chunk], start = cb.rec_start[chunk];
        materialise(b); materialise(first); materialise(n_rec); materialise(start);
        // where the candidates are follows from the above: they are asked for together with the layer's record
        // (of a layer in another mode in vain: its chunks count as empty)
        base = region_start(first, b) + start;
        // (the compaction half of this launch may be rewriting the records of a layer in another mode: whatever
        // is read of them, nothing is asked for outside the buffer)
        cnt = base + n_rec <= cb.tmp_total ? n_rec : 0u;
        const SelRec S = cb.sel[b];
        is_cand = S.mode == SEL_CAND;
        prefix = S.prefix;
        hist3 = cb.hist3 + (size_t)b * D3_BINS;
    }
    const uint32_t cmax = wave_max_over_groups<S>(cnt);
    uint32_t n_above = 0, n_amb = 0;            // of this chunk: threshold prefix exceeded / shared
    // one round: one candidate of the chunk per lane of its group
    auto round = [&](bool in, uint32_t key) {
        in = in && is_cand;
        const bool a = in && (key >> D2_SHIFT) == prefix;
        const bool hi = in && (key >> D2_SHIFT) > prefix;
        const uint32_t am = ballot_sub<S>(g, a);
        n_above += __popc(ballot_sub<S>(g, hi));
        n_amb += __popc(am);
        if (am == 0) return;
        // one atomic per group when all its matching lanes hold the same key (zeros, constants)
        const uint32_t first = (uint32_t)__ffs((int)am) - 1u;
        const uint32_t k0v = __shfl(key, g.shift + first, 64);
        const bool uniform = ballot_sub<S>(g, a && key != k0v) == 0;
        if (uniform) {
            if (g.sub == first) atomicAdd(&hist3[key & (D3_BINS - 1)], (uint32_t)__popc(am));
        } else if (a) {
            atomicAdd(&hist3[key & (D3_BINS - 1)], 1u);
        }
    };
    // the first eight rounds' loads go out together (positions past the chunk's last candidate read entry 0
    // of the buffer, always a valid address, and are dropped; a chunk without candidates has no valid start)
    // (and so on, eight rounds per memory round trip: a layer that spills an eighth has 32 rounds a chunk)
    constexpr int AHEAD = 8;
    for (uint32_t k0 = 0; k0 < cmax; k0 += AHEAD * S) {
        float px[AHEAD];
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) {
            const uint32_t k = k0 + (uint32_t)t * S + g.sub;
            px[t] = cb.tmp_x[k < cnt ? base + k : 0ull];
        }
#pragma unroll
        for (int t = 0; t < AHEAD; ++t)
            if (k0 + (uint32_t)t * S < cmax) round(k0 + (uint32_t)t * S + g.sub < cnt, key_of(px[t]));
    }
    // A chunk without an entry in the threshold's prefix bin (nearly all of them) is settled here:
    // every entry above the prefix is above the threshold, none equals it.  The others are counted
    // again once the threshold key is known.
    if (is_cand && g.sub == 0) { cb.c_gt[chunk] = n_above; cb.c_eq[chunk] = 0u; cb.rec_amb[chunk] = n_amb; }
}

// One launch for both sources of candidates: the first `hist_blocks` workgroups histogram the last
// digit of the spilled candidates (layers in SEL_CAND mode), the others run the streaming compaction
// for the layers that need it (none after a single-pass profile whose spilled range serves every
// layer: they leave after one load).  The two touch different layers.
__global__ __launch_bounds__(256) void k_candidates(CompressBuffers cb, uint32_t nchunks_total, const uint32_t* chunk_big,
                                                    uint32_t hist_blocks, uint32_t ntiles, int32_t err_internal) {
    if (blockIdx.x < hist_blocks) hist3_candidates(cb, nchunks_total, chunk_big, blockIdx.x);
    else compact_tiles(cb, ntiles, err_internal, blockIdx.x - hist_blocks, gridDim.x - hist_blocks);
}

// ---------------------------------------------------------------------------------------------
// Exact threshold key and tie quota per big layer from the last-digit histogram.
__global__ __launch_bounds__(256) void k_resolve(CompressBuffers cb) {
    __shared__ uint32_t su[16];
    __shared__ uint32_t res[2];
    const uint32_t b = blockIdx.x, tid = threadIdx.x;
    const SelRec S = cb.sel[b];
    // The histogram is left at zero for the next call, whatever the mode: this kernel is its only reader.
    uint4* h4 = reinterpret_cast<uint4*>(cb.hist3 + (size_t)b * D3_BINS + tid * 16u);
    if (S.mode != SEL_PREFIX && S.mode != SEL_CAND && !(S.mode == SEL_DIRECT && S.amb != 0u)) {
        if (tid == 0) { cb.tau[b] = 0u; cb.quota[b] = 0u; }   // everything or nothing: decided by the mode alone
#pragma unroll
        for (int k = 0; k < 4; ++k) h4[k] = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    const uint32_t need = S.K - S.above;           // 1..amb entries to take from the ambiguous ones
    // thread t owns digits 16t..16t+15; we need, from the top, the digit where the running count reaches `need`
    uint32_t c[16], sum = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const uint4 v = h4[k];
        c[4 * k] = v.x; c[4 * k + 1] = v.y; c[4 * k + 2] = v.z; c[4 * k + 3] = v.w;
        h4[k] = make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) sum += c[k];
    uint32_t tot;
    const uint32_t ex = block_exclusive_scan<uint32_t>(sum, su, &tot);
    // entries in digits above this thread's range
    uint32_t above = tot - ex - sum;
    if (tid == 0) { res[0] = 0xFFFFFFFFu; res[1] = 0; }
    __syncthreads();
    if (above < need && above + sum >= need) {
#pragma unroll
        for (int k = 15; k >= 0; --k) {
            if (above + c[k] >= need) { res[0] = tid * 16u + k; res[1] = need - above; break; }
            above += c[k];
        }
    }
    __syncthreads();
    if (tid == 0) {
        if (res[0] == 0xFFFFFFFFu) {               // histogram does not cover the quota (stale cache): keep all ambiguous
            cb.tau[b] = S.prefix << D2_SHIFT; cb.quota[b] = 0xFFFFFFFFu;
        } else {
            cb.tau[b] = (S.prefix << D2_SHIFT) | res[0];
            cb.quota[b] = res[1];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Per chunk: how many candidates lie above tau and how many equal it.  Four lanes per chunk.
__global__ __launch_bounds__(256) void k_chunk_count(CompressBuffers cb, uint32_t nchunks_total,
                                                     const uint32_t* chunk_big) {
    constexpr uint32_t S = SUB_COUNT;
    const SubGroup g = sub_group<S>();
    const uint32_t chunk = blockIdx.x * (256u / S) + threadIdx.x / S;
    const bool live = chunk < nchunks_total;
    uint32_t cnt = 0, tau = 0, total = 0;
    uint64_t base = 0;
    bool settled = false;
    // a chunk of a layer that is served from g and h: its 1024 positions take the place of its candidates
    bool direct = false;
    const float* gL = nullptr;
    const float* hL = nullptr;
    uint32_t vb = 0, mis = 0, nL = 0;
    if (live) {
        // what the chunk index alone addresses goes out together, then the layer's record
        const uint32_t b = chunk_big[chunk], first = cb.chunk_first[chunk];
        const uint32_t amb = cb.rec_amb[chunk], start = cb.rec_start[chunk];
        total = cb.rec_cnt[chunk];
        materialise(b); materialise(first); materialise(amb); materialise(start); materialise(total);
        const SelRec S = cb.sel[b];
        const uint32_t t = cb.tau[b];
        // Only chunks with entries in the threshold's prefix bin are read again.  Of the others, those
        // of the classic pass hold nothing below the threshold prefix and pass whole; those of the
        // spilled candidates were counted by k_hist3c.
        if ((S.mode == SEL_CAND || S.mode == SEL_PREFIX) && amb != 0u) {
            cnt = total;
            tau = t;
            base = region_start(first, b) + start;
        }
        settled = S.mode == SEL_CAND && cnt == 0u;      // counted by k_hist3c
        if (S.mode == SEL_DIRECT && amb != 0u) {
            const LayerDesc L = cb.layers[cb.big_layer[b]];
            direct = true; cnt = CHUNK; tau = t;
            gL = L.g; hL = L.h; vb = (chunk - L.chunk0) * CHUNK; mis = L.mis; nL = L.n;
        }
    }
    uint32_t gt = 0, eq = 0;
    if (direct) {
        for (uint32_t k = g.sub; k < CHUNK; k += S) {
            const uint32_t v = vb + k, e = v - mis;
            if (v >= mis && e < nL) {
                const uint32_t key = key_of(gload(gL + e) - gload(hL + e));
                gt += key > tau;
                eq += key == tau;
            }
        }
    } else {
        for (uint32_t k = g.sub; k < cnt; k += S) {
            const uint32_t key = key_of(cb.tmp_x[base + k]);
            gt += key > tau;
            eq += key == tau;
        }
    }
#pragma unroll
    for (int d = S / 2; d > 0; d >>= 1) { gt += __shfl_xor(gt, d, 64); eq += __shfl_xor(eq, d, 64); }
    if (cnt == 0) { gt = total; eq = 0; }
    if (live && !settled && g.sub == 0) { cb.c_gt[chunk] = gt; cb.c_eq[chunk] = eq; }
}

// ---------------------------------------------------------------------------------------------
// Payload position and tie allowance of every chunk.  One workgroup per block of 1024 chunks, one
// thread per chunk.  Ties are granted to the lowest indices first, so all chunks before this
// block together keep min(their ties, quota) of them: the block's starting point follows from two
// sums over the earlier chunks of the layer, which every workgroup takes for itself (no atomics,
// no serial pass over the layer).
__global__ __launch_bounds__(1024) void k_chunk_bases(CompressBuffers cb) {
    __shared__ uint32_t su[16];
    const uint32_t blk = blockIdx.x, tid = threadIdx.x;
    const uint32_t b = cb.cblk_big[blk];
    const uint32_t li = cb.big_layer[b];
    const LayerDesc L = cb.layers[li];
    const uint32_t quota = cb.quota[b];
    const uint32_t kb = blk - L.cblk0;              // this block's number inside the layer
    uint32_t pg = 0, pe = 0;
    {
        // kb * CBLOCK is a multiple of 1024: every thread takes kb entries, sixteen loads of each table at a time (the
        // last block of the largest layer has the most to add up and sets the kernel's duration: few round trips)
        const uint32_t* pgt = cb.c_gt + L.chunk0 + tid;
        const uint32_t* peq = cb.c_eq + L.chunk0 + tid;
        for (uint32_t k = 0; k < kb; k += 16u) {
            uint32_t a[16], e[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const bool in = k + (uint32_t)u < kb;
                const size_t o = (size_t)(in ? k + (uint32_t)u : 0u) * 1024u;
                a[u] = pgt[o]; e[u] = peq[o];
                if (!in) { a[u] = 0u; e[u] = 0u; }
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) { pg += a[u]; pe += e[u]; }
        }
    }
    uint32_t gt_before, eq_before0;
    (void)block_exclusive_scan<uint32_t>(pg, su, &gt_before);
    (void)block_exclusive_scan<uint32_t>(pe, su, &eq_before0);
    const uint32_t out_before = gt_before + min(eq_before0, quota);
    const uint32_t c = kb * CBLOCK + tid;
    const bool ok = c < L.nchunks;
    const uint32_t gt = ok ? cb.c_gt[L.chunk0 + c] : 0u;
    const uint32_t eq = ok ? cb.c_eq[L.chunk0 + c] : 0u;
    const uint32_t eq_before = eq_before0 + block_exclusive_scan<uint32_t>(eq, su, nullptr);
    const uint32_t allow = eq_before < quota ? min(eq, quota - eq_before) : 0u;
    const uint32_t ob = out_before + block_exclusive_scan<uint32_t>(gt + allow, su, nullptr);
    if (ok) { cb.o_base[L.chunk0 + c] = ob; cb.o_allow[L.chunk0 + c] = allow; }
}

// ---------------------------------------------------------------------------------------------
// Per chunk (sixteen lanes each): write the surviving candidates as payload and update the estimator.
__global__ __launch_bounds__(256) void k_finalize(CompressBuffers cb, uint32_t nchunks_total,
                                                  const uint32_t* chunk_big) {
    const SubGroup g = sub_group();
    const uint32_t chunk = blockIdx.x * CHUNKS_PER_WG + threadIdx.x / SUB;
    uint32_t cnt = 0, tau = 0, allow = 0, room = 0, out_run = 0, eq_run = 0;
    uint64_t src = 0, dst = 0;
    bool filter = false;
    float* h = nullptr;
    // a chunk of a layer that is served from g and h: its 1024 positions take the place of its candidates
    bool direct = false;
    const float* gL = nullptr;
    uint32_t vb = 0, mis = 0, nL = 0;
    if (chunk < nchunks_total) {
        // everything indexed by the chunk is fetched at once; one more round trip brings the layer's record
        const uint32_t b = chunk_big[chunk], first = cb.chunk_first[chunk];
        const uint32_t keepn = cb.c_gt[chunk];
        const uint32_t n_rec = cb.rec_cnt[chunk], start = cb.rec_start[chunk], amb = cb.rec_amb[chunk];
        allow = cb.o_allow[chunk];
        out_run = cb.o_base[chunk];
        materialise(b); materialise(first); materialise(keepn); materialise(n_rec); materialise(start); materialise(amb);
        materialise(allow); materialise(out_run);
        // most chunks keep nothing (the candidates are several times the payload): not read at all
        if (keepn + allow != 0u) {
            // every field of the record is valid whatever the mode; SEL_NONE only empties the chunk.
            // (Kept free of a nested branch on the mode: with one, the generated code left dst undefined
            // for SEL_CAND lanes.)
            const SelRec S = cb.sel[b];
            tau = cb.tau[b];
            cnt = S.mode != SEL_NONE ? n_rec : 0u;
            h = S.h;
            filter = S.mode == SEL_CAND || (S.mode == SEL_PREFIX && amb != 0u);
            src = region_start(first, b) + start;
            dst = S.dst;
            room = S.K;                            // payload slots of this layer
            if (S.mode == SEL_DIRECT) {
                const LayerDesc L = cb.layers[cb.big_layer[b]];
                direct = true; cnt = CHUNK; filter = S.amb != 0u;      // amb == 0: every entry is kept
                gL = L.g; vb = (chunk - L.chunk0) * CHUNK; mis = L.mis; nL = L.n;
            }
        }
    }
    // entry k of the chunk: a candidate (index, x), or position k of the chunk itself
    auto fetch = [&](uint32_t k, uint32_t& idx, float& x) -> bool {
        if (direct) {
            const uint32_t v = vb + k, e = v - mis;
            const bool in = k < cnt && v >= mis && e < nL;
            const uint32_t at = in ? e : 0u;
            idx = at;
            x = gload(gL + at) - gload(h + at);
            return in;
        }
        const bool in = k < cnt;
        const uint64_t at = in ? src + k : 0ull;
        idx = cb.tmp_idx[at]; x = cb.tmp_x[at];
        return in;
    };
    const uint32_t cmax = wave_max_over_groups(cnt);
    // one round: sixteen candidates of the chunk, in index order: which are kept, and where they go
    auto round = [&](bool in, float x, uint32_t& pos) -> bool {
        const uint32_t key = key_of(x);
        const bool iseq = in && filter && key == tau;
        const uint32_t eqm = ballot_sub(g, iseq);
        const bool keep = in && (!filter || key > tau || (iseq && eq_run + rank_sub(g, eqm) < allow));
        eq_run += __popc(eqm);
        const uint32_t km = ballot_sub(g, keep);
        pos = out_run + rank_sub(g, km);
        out_run += __popc(km);
        return keep && pos < room;
    };
    // A chunk rarely holds more than 64 candidates: the loads of the first four rounds go out together,
    // so the wave pays one memory round trip for them instead of four; likewise the estimator entries of what the
    // four rounds keep are read together, then written (the entries of a chunk are distinct elements).
    constexpr int AHEAD = 4;
    // (positions past the chunk's last entry read entry 0 of the buffer or the layer, a valid address, and are dropped)
    for (uint32_t k0 = 0; k0 < cmax; k0 += AHEAD * SUB) {
        uint32_t pidx[AHEAD], pos[AHEAD];
        float px[AHEAD], ph[AHEAD];
        bool pin[AHEAD], keep[AHEAD];
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) pin[t] = fetch(k0 + (uint32_t)t * SUB + g.sub, pidx[t], px[t]);
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) {
            keep[t] = false; pos[t] = 0u;
            if (k0 + (uint32_t)t * SUB < cmax) keep[t] = round(pin[t], px[t], pos[t]);
        }
        // the estimator is read here: candidates carry (index, x) only
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) ph[t] = keep[t] ? gload(h + pidx[t]) : 0.0f;
#pragma unroll
        for (int t = 0; t < AHEAD; ++t) {
            if (keep[t]) {
                const uint64_t o = dst + pos[t];
                cb.idx_out[o] = pidx[t];
                const float add = emit_value(cb, o, px[t]);
                gstore(h + pidx[t], ph[t] + add);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Small layers: sort in LDS, mark the first K of the order, emit in index order.
__global__ __launch_bounds__(SMALL_THREADS) void k_small_compress(CompressBuffers cb) {
    __shared__ unsigned long long a[SMALL_MAX];
    __shared__ uint32_t flag[SMALL_MAX / 32];
    __shared__ uint32_t su[16];
    __shared__ int bad;
    const uint32_t tid = threadIdx.x;
    const uint32_t li = cb.small_layer[blockIdx.x];
    const LayerDesc L = cb.layers[li];
    // the lookup kernel refuses the whole call through the status word; small layers re-check
    // their own slice so that nothing is written out of bounds
    const uint64_t K64 = cb.K[li], off = cb.offsets[li];
    if (tid == 0) bad = (*cb.status != 0);
    __syncthreads();
    if (bad || K64 == 0 || K64 > L.n || off > cb.capacity_pairs || K64 > cb.capacity_pairs - off) return;
    const uint32_t K = (uint32_t)K64;
    const uint32_t P = next_pow2(L.n < 2 ? 2 : L.n);
    load_sorted_small(L, a, P);
    bitonic_sort_lds<SMALL_THREADS>(a, P);
    for (uint32_t w = tid; w < SMALL_MAX / 32; w += SMALL_THREADS) flag[w] = 0u;
    __syncthreads();
    for (uint32_t rk = tid; rk < K; rk += SMALL_THREADS) {
        const uint32_t idx = (uint32_t)a[rk];
        atomicOr(&flag[idx >> 5], 1u << (idx & 31));
    }
    __syncthreads();
    // emit in index order: thread t owns indices [t*per, (t+1)*per), per a multiple of 32 or the whole word range
    const uint32_t words = (L.n + 31) / 32;
    const uint32_t wper = (words + SMALL_THREADS - 1) / SMALL_THREADS;
    uint32_t mine = 0;
    for (uint32_t w = tid * wper; w < min(words, (tid + 1) * wper); ++w) mine += __popc(flag[w]);
    uint32_t pos = block_exclusive_scan<uint32_t>(mine, su, nullptr);
    for (uint32_t w = tid * wper; w < min(words, (tid + 1) * wper); ++w) {
        uint32_t f = flag[w];
        while (f) {
            const uint32_t bit = __ffs(f) - 1;
            f &= f - 1;
            const uint32_t idx = w * 32 + bit;
            const float g = gload(L.g + idx), hv = gload(L.h + idx);
            const float x = g - hv;
            cb.idx_out[off + pos] = idx;
            const float add = emit_value(cb, off + pos, x);
            gstore(L.h + idx, hv + add);
            ++pos;
        }
    }
}

}  // namespace kimad
