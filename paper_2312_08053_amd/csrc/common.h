// Shared definitions for the gfx950 kernels: layouts, radix digits, loaders, wave primitives.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kimad {

// ---- radix decomposition of the 31-bit magnitude key -------------------------------------
// key = bits(x) & 0x7fffffff.  digit 1 = key[30:19] (8 exponent + 4 mantissa bits), digit 2 =
// key[18:12], digit 3 = key[11:0].  Every element of one digit-1 bin shares its exponent field,
// which lets squares be summed exactly as integers relative to that exponent.
constexpr uint32_t D1_BITS = 12, D2_BITS = 7, D3_BITS = 12;
constexpr uint32_t D1_BINS = 1u << D1_BITS;   // 4096
constexpr uint32_t D2_BINS = 1u << D2_BITS;   // 128
constexpr uint32_t D3_BINS = 1u << D3_BITS;   // 4096
constexpr uint32_t D1_SHIFT = 19, D2_SHIFT = 12;
constexpr uint32_t MAX_SLOTS = 64;            // distinct boundary bins per layer (<= J)
constexpr uint32_t NO_SLOT = 0xFF;
constexpr uint32_t KIMAD_MAX_J_CONST = 64;   // must equal KIMAD_MAX_J of the public header
constexpr uint32_t KEY_INVALID = 0xFFFFFFFFu; // marks lanes outside the layer

constexpr uint32_t SMALL_MAX = 8192;          // layers up to this size are sorted whole in LDS
constexpr uint32_t CHUNK = 1024;              // elements one wave compacts at a time (4 quads per lane)
constexpr uint32_t NQ = CHUNK / 256;          // quads per lane and chunk
constexpr uint32_t CBLOCK = 1024;             // chunks per chunk block (one workgroup scans one block)
constexpr uint32_t PRE_SLOTS = 108;           // digit-2 slots the single-pass profile can hold in LDS
constexpr uint32_t SLOT_STRIDE = PRE_SLOTS + 64;  // slots per layer in the global digit-2 tables: 0..PRE_SLOTS-1 fixed
                                              // before a pass, PRE_SLOTS.. found after it (filled from candidates)
// LDS entry of a slot in the single-pass profile: [count:20 | sum of (significand^2 >> 24):44]
constexpr uint32_t PK_SHIFT = 24;
constexpr uint64_t PK_ONE = 1ull << 44;
constexpr uint64_t PK_MASK = PK_ONE - 1;
constexpr uint32_t PK_MAX_CHUNKS = 1023;      // 1023 * 1024 entries < 2^20: the count field cannot overflow
constexpr uint32_t SQ_SHIFT = 16;             // squares of 24-bit significands are kept >> 16
constexpr uint64_t CNT_ONE = 1ull << 48;      // packed LDS entry: [count:16 | sum of squares:48]
constexpr uint64_t SQ_MASK = CNT_ONE - 1;

// selection modes of a layer in the compaction pass
// (SEL_DIRECT: what lies at or above the threshold prefix does not fit the layer's candidate region, or
// everything is kept: counted, and later written out, straight from g and h.  amb == 0 then means K == n.)
enum : uint32_t { SEL_NONE = 0, SEL_PREFIX = 1, SEL_ALL = 2, SEL_CAND = 3, SEL_DIRECT = 4 };

struct LayerDesc {
    const float* g;
    float* h;
    uint32_t n;        // elements
    uint32_t mis;      // (address of g / 4) & 3: virtual index v = element + mis is 16-byte aligned at v % 4 == 0
    uint32_t hvec;     // h has the same misalignment, so it can be read with 16-byte loads too
    int32_t big;       // index among the tiled ("big") layers, -1 for a small layer
    uint32_t tile0;    // first tile of this layer in the tile list
    uint32_t ntiles;
    uint32_t chunk0;   // first chunk of this layer in the chunk list
    uint32_t nchunks;
    uint32_t sstride;  // the sampling pre-pass reads one chunk out of every sstride
    uint32_t cblk0;    // first block of 1024 chunks of this layer in the chunk-block list
    uint64_t tmp0;     // start of this layer's region in the candidate buffer
    uint32_t tmp_cap;  // entries the region holds
    uint32_t pad;
};

// Per big layer, state of the fused single-pass profile.
struct LayerState {
    uint32_t spill_bin;    // entries whose digit-1 bin is >= spill_bin were written to the candidate buffer
    uint32_t nslots_d;     // boundary-bin slots fixed before the pass (predicted, or exact after a redo)
    uint32_t nslots_t;     // slots PRE_SLOTS.. assigned after the pass and filled from the candidates
    uint32_t redo;         // prediction missed: digit 2 is recounted by a full pass over this layer
    uint32_t spill_cnt;    // entries in the candidate region
    uint32_t spill_valid;  // the region holds every entry with bin >= spill_bin, in index order per chunk
    uint32_t slot_lo;      // single-pass profile: the predicted slots 0..nslots_d-1 are the bins slot_lo, slot_lo+1, ...
    uint32_t pad;
};

// Per big layer, what the compaction pass needs.
struct SelRec {
    uint32_t mode;     // SEL_*
    uint32_t prefix;   // 19-bit key prefix of the threshold (digit1 | digit2)
    uint32_t above;    // entries whose prefix is greater (certainly selected)
    uint32_t amb;      // entries whose prefix is equal (decided by digit 3)
    uint64_t tmp_base; // start of this layer's region in the candidate buffer
    uint32_t cap;      // candidates this layer may write
    uint32_t K;
    float* h;          // the layer's estimator
    uint64_t dst;      // first payload slot of the layer
};

// ---- global-memory accessors ----------------------------------------------------------------
// Layer pointers come out of a table in memory, so the compiler only knows them as generic
// ("flat") pointers; flat accesses count against the LDS counter as well and serialise with the
// LDS atomics.  They always point to device memory: say so.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const float gc_float;
typedef __attribute__((address_space(1))) float g_float;
typedef __attribute__((address_space(1))) const f32x4 gc_f32x4;

__device__ __forceinline__ float gload(const float* p) { return *reinterpret_cast<gc_float*>((uintptr_t)p); }
__device__ __forceinline__ float4 gload4(const float* p) {
    const f32x4 v = *reinterpret_cast<gc_f32x4*>((uintptr_t)p);
    return make_float4(v.x, v.y, v.z, v.w);
}
// The same for data that is read once and not again soon (a streaming pass over g and h): the
// nontemporal hint keeps such lines from displacing everything else in the L2, and a plain read of
// 1 GB runs about a tenth faster with it on this machine (6.8 instead of 6.1 TB/s).
__device__ __forceinline__ float4 gload4_stream(const float* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<gc_f32x4*>((uintptr_t)p));
    return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void gstore(float* p, float v) { *reinterpret_cast<g_float*>((uintptr_t)p) = v; }
typedef __attribute__((address_space(1))) f32x4 g_f32x4;
__device__ __forceinline__ void gstore4(float* p, float4 v) {
    f32x4 t;
    t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    *reinterpret_cast<g_f32x4*>((uintptr_t)p) = t;
}

// ---- small device helpers ----------------------------------------------------------------
// Makes the compiler hold a loaded value in a register here.  Placed after a group of independent
// loads and before the first branch on one of them, it keeps the loads together in front of the
// branch: one memory round trip instead of one per load.
__device__ __forceinline__ void materialise(uint32_t v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

__device__ __forceinline__ uint32_t mbcnt(uint64_t mask) {
    // number of set bits of mask below the calling lane
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

__device__ __forceinline__ uint64_t ballot(bool p) { return __ballot(p); }

// Orders one wave's LDS accesses: what its lanes wrote before is what its lanes read after (the hardware runs a
// wave's LDS instructions in order; this keeps the compiler from moving them across).
__device__ __forceinline__ void wave_sync_lds() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ uint32_t key_of(float x) { return __float_as_uint(x) & 0x7FFFFFFFu; }

// Integer square of the significand, truncated to 32 bits.  For bin 0 (denormals below 2^-130
// and zeros) callers use sq_exact() instead.  Exponent 255 (Inf/NaN) contributes a NaN count.
__device__ __forceinline__ uint32_t sq_fixed(uint32_t key) {
    uint32_t e = key >> 23, m = key & 0x7FFFFFu;
    uint32_t m24 = e ? (m | 0x800000u) : m;
    uint64_t sq = (uint64_t)m24 * (uint64_t)m24;
    uint32_t c = (uint32_t)(sq >> SQ_SHIFT);
    return e == 255u ? (m != 0u ? 1u : 0u) : c;
}
// The same square in the units of sq_fixed(), but as the single-pass profile knows it: the low 24
// bits of the square dropped and replaced by their midpoint.  Every source of a digit-2 table of
// that profile (the pass itself, the candidate buffer, the recount of a mispredicted layer) uses
// this form, so the table's bits do not depend on which of them filled a slot.
__device__ __forceinline__ uint32_t sq_coarse(uint32_t key) {
    uint32_t e = key >> 23, m = key & 0x7FFFFFu;
    uint32_t m24 = e ? (m | 0x800000u) : m;
    uint64_t sq = (uint64_t)m24 * (uint64_t)m24;
    uint32_t c = ((uint32_t)(sq >> PK_SHIFT) << (PK_SHIFT - SQ_SHIFT)) + (1u << (PK_SHIFT - SQ_SHIFT - 1));
    return e == 255u ? (m != 0u ? 1u : 0u) : c;
}
__device__ __forceinline__ uint64_t sq_exact(uint32_t key) {   // key < 2^19
    return (uint64_t)key * (uint64_t)key;
}

// Value of one unit of a digit-1 bin's integer sum of squares, as a double.
__device__ __forceinline__ double bin_scale(uint32_t bin1) {
    uint32_t e = bin1 >> 4;
    if (bin1 == 0u) return __longlong_as_double((int64_t)(1023 - 298) << 52);           // 2^-298
    int ex = 2 * ((int)(e ? e : 1u) - 150) + (int)SQ_SHIFT;
    return __longlong_as_double((int64_t)(1023 + ex) << 52);
}
__device__ __forceinline__ double sq_to_double(uint32_t bin1, uint64_t s, uint32_t cnt) {
    // Exponent 255: s counts NaNs.  Any NaN makes the sum NaN, otherwise any entry makes it Inf.
    if ((bin1 >> 4) == 255u) {
        if (s) return __longlong_as_double(0x7FF8000000000000ll);
        return cnt ? __longlong_as_double(0x7FF0000000000000ll) : 0.0;
    }
    return (double)s * bin_scale(bin1);
}

// Four consecutive virtual positions v .. v+3 of a layer (v % 4 == 0).  Lanes outside the layer
// get KEY_INVALID.  16-byte loads are used when the quad is entirely inside.
struct Quad {
    float g[4], h[4];
    uint32_t key[4];
};

__device__ __forceinline__ void load_quad(const LayerDesc& L, uint32_t v, Quad& q) {
    const uint32_t lo = L.mis, hi = L.mis + L.n;
    if (v >= lo && v + 4u <= hi) {
        const uint32_t e = v - lo;
        const float4 G = gload4(L.g + e);
        q.g[0] = G.x; q.g[1] = G.y; q.g[2] = G.z; q.g[3] = G.w;
        if (L.hvec) {
            const float4 H = gload4(L.h + e);
            q.h[0] = H.x; q.h[1] = H.y; q.h[2] = H.z; q.h[3] = H.w;
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) q.h[c] = gload(L.h + e + c);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) q.key[c] = key_of(q.g[c] - q.h[c]);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint32_t vv = v + c;
            if (vv >= lo && vv < hi) {
                q.g[c] = gload(L.g + (vv - lo));
                q.h[c] = gload(L.h + (vv - lo));
                q.key[c] = key_of(q.g[c] - q.h[c]);
            } else {
                q.g[c] = 0.f; q.h[c] = 0.f; q.key[c] = KEY_INVALID;
            }
        }
    }
}

// All quads of one chunk for one wave: lane l gets positions vbase + u*256 + 4l .. +3 as raw g, h
// values; bit 4u+c of `valid` tells whether position c of quad u lies inside the layer.  Interior
// chunks of layers whose h shares g's alignment take straight 16-byte loads with no per-lane checks.
struct QuadGH {
    float g[4], h[4];
};

template <int N>
__device__ __forceinline__ void load_chunk(const LayerDesc& L, uint32_t vbase, QuadGH (&q)[N], uint32_t& valid) {
    const uint32_t lane = lane_id();
    if (L.hvec && vbase >= L.mis && vbase + (uint32_t)N * 256u <= L.mis + L.n) {
        const float* gp = L.g + (vbase - L.mis) + 4u * lane;
        const float* hp = L.h + (vbase - L.mis) + 4u * lane;
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const float4 G = gload4_stream(gp + u * 256), H = gload4_stream(hp + u * 256);
            q[u].g[0] = G.x; q[u].g[1] = G.y; q[u].g[2] = G.z; q[u].g[3] = G.w;
            q[u].h[0] = H.x; q[u].h[1] = H.y; q[u].h[2] = H.z; q[u].h[3] = H.w;
        }
        valid = (N >= 8) ? 0xFFFFFFFFu : ((1u << (4 * N)) - 1u);
    } else {
        valid = 0u;
#pragma unroll
        for (int u = 0; u < N; ++u) {
            Quad t;
            load_quad(L, vbase + u * 256u + lane * 4u, t);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                q[u].g[c] = t.g[c]; q[u].h[c] = t.h[c];
                if (t.key[c] != KEY_INVALID) valid |= 1u << (4 * u + c);
            }
        }
    }
}

// Space for a wave's candidates.  Waves take blocks of SPILL_BLOCK entries (or exactly what a
// chunk needs, if more) from the layer's cursor with one returning atomic per block, instead of
// one per chunk: thousands of waves adding to the same address serialise.  Unused tails of blocks
// are never referenced: chunk records delimit what is valid.
constexpr uint32_t SPILL_BLOCK = 512;
// A layer's region of the candidate buffer holds REGION_PER_CHUNK entries per chunk of the layer plus
// REGION_SLACK: 21/128 of the layer.  The single-pass profile spills at most an eighth of a layer into it
// (each workgroup into the slice that belongs to its chunks), the compaction pass whatever lies at or above a
// threshold prefix if that fits; whatever does not fit is served from g and h directly.
constexpr uint32_t REGION_PER_CHUNK = 168;        // a multiple of the 8 entries space is handed out in
constexpr uint32_t REGION_SLACK = 2048;
// The regions of the tiled layers follow one another in the candidate buffer, so a layer's region starts where its
// first chunk and its number among the tiled layers say: a kernel that walks chunks knows where a chunk's candidates
// are from what the chunk's index addresses, without reading the layer's record first.
__host__ __device__ inline uint64_t region_start(uint32_t first_chunk, uint32_t big) {
    return (uint64_t)first_chunk * REGION_PER_CHUNK + (uint64_t)big * REGION_SLACK;
}
struct WaveAlloc { uint32_t base, left; };

__device__ __forceinline__ uint32_t wave_reserve(WaveAlloc& wa, uint32_t total, uint32_t* cursor) {
    if (total > wa.left) {
        const uint32_t want = total > SPILL_BLOCK ? total : SPILL_BLOCK;
        uint32_t b = 0;
        if (lane_id() == 0) b = atomicAdd(cursor, want);
        wa.base = __shfl(b, 0, 64);
        wa.left = want;
    }
    const uint32_t start = wa.base;
    wa.base += total;
    wa.left -= total;
    return start;
}

// Kernels that walk the candidates of chunks give a group of lanes to a chunk, several chunks to a wave: 16 lanes
// where a lane writes per candidate kept (a chunk holds ~20 candidates at a 2 % spill), 4 lanes where the
// candidates are only counted or histogrammed: those kernels are bound by the loads their short-lived waves keep in
// flight, and most lanes of a wider group ask for nothing (measured: 16 -> 8 -> 4 lanes faster each time, 2 slower).
// Ballots are wave-wide; these helpers cut out a group's part.
constexpr uint32_t SUB = 16;                  // lanes per chunk
constexpr uint32_t SUB_COUNT = 4;             // the same where candidates are only counted
constexpr uint32_t SUB_HIST = 4;              // and where every candidate is looked at once for a histogram: eight rounds'
                                              // loads per lane and memory round trip, sixteen chunks to a wave
constexpr uint32_t CHUNKS_PER_WG = 256 / SUB; // chunks a 256-thread workgroup handles
struct SubGroup {
    uint32_t sub;   // lane inside the group
    uint32_t shift; // first lane of the group
};
template <uint32_t S = SUB>
__device__ __forceinline__ SubGroup sub_group() {
    SubGroup g;
    g.sub = threadIdx.x & (S - 1);
    g.shift = (threadIdx.x & 63u) & ~(S - 1);
    return g;
}
template <uint32_t S = SUB>
__device__ __forceinline__ uint32_t ballot_sub(const SubGroup& g, bool p) { return (uint32_t)(ballot(p) >> g.shift) & ((1u << S) - 1u); }
__device__ __forceinline__ uint32_t rank_sub(const SubGroup& g, uint32_t m) { return __popc(m & ((1u << g.sub) - 1u)); }
// largest value over the groups of the wave (loop bounds must be wave-uniform)
template <uint32_t S = SUB>
__device__ __forceinline__ uint32_t wave_max_over_groups(uint32_t v) {
    static_assert(S == 4 || S == 8 || S == 16, "groups of 4, 8 or 16 lanes");
    if (S <= 4) v = max(v, (uint32_t)__shfl_xor(v, 4, 64));
    if (S <= 8) v = max(v, (uint32_t)__shfl_xor(v, 8, 64));
    v = max(v, (uint32_t)__shfl_xor(v, 16, 64));
    v = max(v, (uint32_t)__shfl_xor(v, 32, 64));
    return v;
}

// Block-wide exclusive scan over one value per thread (any block size that is a multiple of 64,
// up to 1024).  `scratch` needs 16 entries.  Returns the exclusive prefix; *total gets the sum.
// Inclusive add-scan of a 32-bit value over the 64 lanes with DPP shifts: no LDS traffic and six
// vector instructions (the shuffle version costs twelve plus six LDS permutes).  Lanes without a
// source keep their value.  A DPP operand must not be read within two cycles of the vector
// instruction that wrote it; the compiler does not know that this assembly reads through DPP, so
// the waits are written out, before the first step as well.
__device__ __forceinline__ uint32_t wave_scan_add_u32(uint32_t v) {
    asm("s_nop 1\n\t"
        "v_add_u32_dpp %0, %0, %0 row_shr:1 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_u32_dpp %0, %0, %0 row_shr:2 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_u32_dpp %0, %0, %0 row_shr:4 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_u32_dpp %0, %0, %0 row_shr:8 row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_u32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\t"
        "v_add_u32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf"
        : "+v"(v));
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        T o = __shfl_up(v, d, 64);
        if ((int)lane_id() >= d) v += o;
    }
    return v;
}

// (32-bit integers take the DPP scan, and the exclusive prefix by subtraction, which is exact for them)
__device__ __forceinline__ void wave_scan_pair(uint32_t v, uint32_t& inc, uint32_t& exc) {
    inc = wave_scan_add_u32(v);
    exc = inc - v;
}
template <typename T>
__device__ __forceinline__ void wave_scan_pair(T v, T& inc, T& exc) {
    inc = wave_inclusive_scan(v);
    // exclusive prefix taken from the neighbouring lane: subtracting v back out would cancel
    // catastrophically for floating-point sums whose terms grow along the scan
    exc = __shfl_up(inc, 1, 64);
    if (lane_id() == 0) exc = 0;
}

template <typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, T* scratch, T* total) {
    const uint32_t w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    T inc, exc;
    wave_scan_pair(v, inc, exc);
    if (lane_id() == 63) scratch[w] = inc;
    __syncthreads();
    T base = 0, tot = 0;
    for (uint32_t i = 0; i < nw; ++i) {
        T s = scratch[i];
        if (i < w) base += s;
        tot += s;
    }
    __syncthreads();
    if (total) *total = tot;
    return base + exc;
}

}  // namespace kimad
