// C ABI of the library: argument checks, workspace layout, kernel launches.
// Declarations and the contract of every entry point are in include/kimad.h.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/kimad.h"
#include "common.h"
#include "k_profile.h"
#include "k_fused.h"
#include "k_compress.h"
#include "k_alloc.h"
#include "k_alloc_band.h"
#include "k_server.h"
#include "k_selftest.h"

static_assert(kimad::KIMAD_MAX_J_CONST == KIMAD_MAX_J, "J limit mismatch");

namespace {

using namespace kimad;

constexpr uint64_t ALIGN = 256;
// A table entry is accepted from the two histogram levels when its rigorous error bound is
// below this fraction of the entry; otherwise the exact last-digit pass recomputes it.
constexpr double CERT_TOL = 4e-6;
constexpr double SLOT_WIDEN = 1.2e-7;      // half width (relative) of the midpoint form of a single-pass slot's squares

inline uint64_t align_up(uint64_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Byte offsets of every array inside the workspace.
struct Layout {
    uint32_t L = 0, J = 0, B = 0, S = 0;
    uint32_t tile_elems = 0, ntiles = 0, nchunks = 0, nswg = 0, ncblk = 0;
    uint64_t dp_cells = 0, tmp_cap = 0, sum_kmax = 0;
    // static tables
    uint64_t layers, ktab, tile_layer, chunk_big, chunk_first, big_layer, small_layer;
    // zeroed before every profile
    uint64_t swg_layer, swg_first, state, lutc;
    uint64_t fresh = 0, hprev = 0, gprev = 0;
    uint64_t zero1_begin, cnt1, sq1, cnt2, sq2, diag, layer_flag, shist, ghist, cursor, spill_over, zero1_end;
    uint64_t cprev = 0;
    uint64_t big_tmp0, parts, wg_part0, big_part0, big_nparts, zero1_mid;
    uint32_t main_wgs = 256, chunks_per_wg = 1, nparts = 0;
    uint64_t pool_prefix, pool_big, pool_t0, pool_cnt, pool_hist, tgt_unsel, tgt_base;
    uint32_t pool_cap = 1;
    uint64_t lut1, nslots, slot_bin, slot_cnt, slot_sq;
    uint64_t tgt_slot, tgt_r, tgt_above1, tgt_below, sel_prefix, sel_above, sel_amb;
    // compress
    uint64_t ksel, sel, zero2_begin, hist3, zero2_end, tau, quota, cblk_big;
    uint64_t rec_start, rec_cnt, rec_amb, c_gt, c_eq, o_base, o_allow;
    uint64_t tmp_idx, tmp_x;
    // allocation
    uint64_t ncompact;
    uint64_t row0, row1, choice, dp_flags, dl_wall, dl_w, dl_jj, dl_e, dl_n, dl_bad, rows_g;
    uint64_t dense_E, dense_Kcost, dense_Kout;
    uint64_t band_lo, band_hi, band_info, live_off, live_e, live_before, live_w, live_jj;
    uint64_t rstride = 0;            // cells per stored DP row (LDS-resident recurrence only)
    uint64_t total = 0;
};

struct HostLayer {
    uint32_t n, mis, hvec;
    int32_t big;
    uint32_t tile0, ntiles, chunk0, nchunks;
    uint32_t sstride, sgroups, swg0, nswg;   // sampling: stride in chunks, sampled groups, workgroups
    uint32_t cblk0, ncblk;                   // blocks of 1024 chunks
    uint64_t tmp0;                           // region start in the candidate buffer
    uint32_t tmp_cap;                        // entries of the region
};

uint32_t pick_tile_elems(uint64_t d_big) {
    // aim at >= 8 tiles per compute unit on large inputs, keep tiles within the 16-bit LDS counters
    uint64_t t = 32768;
    while (t > 2048 && d_big / t < 256ull * 8ull) t >>= 1;
    return (uint32_t)t;
}

uint32_t grid_size_K(double r, uint64_t n) {
    double k = std::ceil(r * (double)n);
    if (k < 1.0) k = 1.0;
    if (k > (double)n) k = (double)n;
    return (uint32_t)k;
}

// Shapes only: misalignment is taken as the worst case (3) so that the layout does not depend on
// pointer values and kimad_workspace_bytes can be called before the tensors exist.
// Workgroups of the streaming pass: one per compute unit of the current device (256 if no device
// answers, as when only the workspace size is asked for on a machine without one), at most 1024,
// and at most cfg.max_workgroups.
uint32_t stream_workgroups(const kimad_config_t& cfg) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) {
        (void)hipGetLastError();
        cus = 256;
    }
    uint32_t w = (uint32_t)std::min(cus, 1024);
    if (cfg.max_workgroups) w = std::min(w, cfg.max_workgroups);
    return w;
}

// The parts of the streaming pass: workgroup w walks chunks [w * per, (w + 1) * per) and starts a new
// histogram at every layer boundary and after PK_MAX_CHUNKS chunks, exactly as k_main does.
struct PartTables {
    std::vector<uint32_t> wg_part0, big_part0, big_nparts;
};
uint32_t plan_parts(const std::vector<HostLayer>& hl, uint32_t B, uint32_t nchunks, uint32_t wgs, uint32_t per,
                    PartTables* out) {
    std::vector<uint32_t> c0(B ? B : 1), c1(B ? B : 1);
    for (const HostLayer& h : hl)
        if (h.big >= 0) { c0[h.big] = h.chunk0; c1[h.big] = h.chunk0 + h.nchunks; }
    if (out) { out->wg_part0.assign(wgs, 0); out->big_part0.assign(B ? B : 1, 0); out->big_nparts.assign(B ? B : 1, 0); }
    uint32_t part = 0, b = 0;
    for (uint32_t w = 0; w < wgs; ++w) {
        uint64_t cur = (uint64_t)w * per;
        const uint64_t c_end = std::min<uint64_t>(nchunks, cur + per);
        if (out) out->wg_part0[w] = part;
        while (cur < c_end) {
            while (cur >= c1[b]) ++b;
            const uint64_t seg_end = std::min<uint64_t>(std::min<uint64_t>(c_end, c1[b]), cur + PK_MAX_CHUNKS);
            if (out) { if (out->big_nparts[b]++ == 0) out->big_part0[b] = part; }
            ++part;
            cur = seg_end;
        }
    }
    return part;
}

int make_layout(const uint64_t* n, uint32_t L, uint32_t J, const kimad_config_t& cfg, Layout& lo,
                std::vector<HostLayer>* hl_out, PartTables* parts_out = nullptr) {
    std::vector<HostLayer> hl_local;
    std::vector<HostLayer>* hl = hl_out ? hl_out : &hl_local;
    if (!n || L == 0 || L > 65535 || J == 0 || J > KIMAD_MAX_J) return KIMAD_ERR_INVALID_ARG;
    lo.L = L; lo.J = J;
    uint64_t d_big = 0, d_all = 0;
    uint32_t B = 0, S = 0;
    for (uint32_t i = 0; i < L; ++i) {
        if (n[i] == 0 || n[i] > KIMAD_MAX_N) return KIMAD_ERR_INVALID_ARG;
        d_all += n[i];
        if (n[i] > SMALL_MAX) { d_big += n[i]; ++B; } else ++S;
    }
    lo.B = B; lo.S = S;
    lo.tile_elems = pick_tile_elems(d_big);
    uint64_t nt = 0, nc = 0, tmp_run = 0;
    uint32_t nsw = 0, ncblk = 0;
    hl->resize(L);
    int32_t bi = 0;
    for (uint32_t i = 0; i < L; ++i) {
        HostLayer h{};
        h.n = (uint32_t)n[i];
        h.big = -1;
        if (n[i] > SMALL_MAX) {
            const uint64_t span = n[i] + 3;
            h.big = bi++;
            h.tile0 = (uint32_t)nt; h.ntiles = (uint32_t)((span + lo.tile_elems - 1) / lo.tile_elems);
            h.chunk0 = (uint32_t)nc; h.nchunks = (uint32_t)((span + CHUNK - 1) / CHUNK);
            nt += h.ntiles; nc += h.nchunks;
            // sample one chunk in every `sstride`, keeping at least ~64 sampled chunks per layer
            h.sstride = std::max<uint32_t>(1, std::min<uint32_t>(16, h.nchunks / 64));
            h.sgroups = (h.nchunks + h.sstride - 1) / h.sstride;
            h.swg0 = nsw; h.nswg = (h.sgroups + SAMPLE_GROUPS_PER_WG - 1) / SAMPLE_GROUPS_PER_WG;
            nsw += h.nswg;
            h.tmp0 = region_start(h.chunk0, (uint32_t)h.big); h.tmp_cap = h.nchunks * REGION_PER_CHUNK + REGION_SLACK;
            tmp_run = h.tmp0 + h.tmp_cap;                 // the regions follow one another: region_start says where
            h.cblk0 = ncblk; h.ncblk = (h.nchunks + CBLOCK - 1) / CBLOCK; ncblk += h.ncblk;
        }
        (*hl)[i] = h;
    }
    lo.nswg = nsw;
    lo.ncblk = ncblk;
    if (nt > 0x7FFFFFFFull || nc > 0xFFFFFFFFull) return KIMAD_ERR_INVALID_ARG;
    lo.ntiles = (uint32_t)nt; lo.nchunks = (uint32_t)nc;
    lo.sum_kmax = d_all;                                  // the last grid ratio may be 1
    const uint32_t pair = cfg.pair_bytes ? cfg.pair_bytes : 8u;
    if (cfg.cost_units_D) {
        lo.dp_cells = std::min<uint64_t>(cfg.cost_units_D, d_all) + 1;
    } else {
        uint64_t pmax = cfg.max_budget_bytes ? cfg.max_budget_bytes / pair : d_all;
        lo.dp_cells = std::min<uint64_t>(pmax, d_all) + 1;
    }
    // (the winners' table of the allocation is L rows of dp_cells bytes: with the exact cost axis and no
    // budget limit that is L * d bytes, 18 GB for a 124M-element model: refused rather than asked of the caller)
    if ((uint64_t)L * align_up(lo.dp_cells) > (4ull << 30)) return KIMAD_ERR_TABLES_TOO_LARGE;
    lo.tmp_cap = tmp_run;                                 // one region per tiled layer
    // a workgroup of the streaming pass writes its histograms out whole (140 KB a part): on small sets fewer
    // workgroups with at least 16 chunks each do less of that than one per compute unit would
    lo.main_wgs = std::max<uint32_t>(1, std::min<uint32_t>(stream_workgroups(cfg), (lo.nchunks + 15) / 16));
    lo.chunks_per_wg = std::max<uint32_t>(1, (lo.nchunks + lo.main_wgs - 1) / lo.main_wgs);
    lo.nparts = plan_parts(*hl, B, lo.nchunks, lo.main_wgs, lo.chunks_per_wg, parts_out);

    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { uint64_t o = off; off = align_up(off + bytes); return o; };
    const uint64_t LJ = (uint64_t)L * J;
    lo.layers = take(sizeof(LayerDesc) * (uint64_t)L);
    lo.ktab = take(4 * LJ);
    lo.tile_layer = take(4ull * (nt ? nt : 1));
    lo.chunk_big = take(4ull * (nc ? nc : 1));
    lo.chunk_first = take(4ull * (nc ? nc : 1));
    lo.big_layer = take(4ull * (B ? B : 1));
    lo.big_tmp0 = take(8ull * (B ? B : 1));
    lo.wg_part0 = take(4ull * lo.main_wgs);
    lo.big_part0 = take(4ull * (B ? B : 1));
    lo.big_nparts = take(4ull * (B ? B : 1));
    // (the exact pass's pool of last-digit histograms lives in the same memory: the parts are dead once
    // k_reduce_parts has run, and a pool entry is cleared by the workgroup that takes it)
    lo.pool_cap = (uint32_t)std::min<uint64_t>(std::max<uint64_t>((uint64_t)B * J, 1), POOL_LIMIT);
    lo.parts = take(std::max<uint64_t>(8ull * PART_STRIDE * (lo.nparts ? lo.nparts : 1), 4ull * lo.pool_cap * D3_BINS));
    lo.pool_hist = lo.parts;
    lo.small_layer = take(4ull * (S ? S : 1));
    lo.swg_layer = take(4ull * (nsw ? nsw : 1));
    lo.swg_first = take(4ull * (nsw ? nsw : 1));
    lo.state = take(sizeof(LayerState) * (uint64_t)(B ? B : 1));
    lo.lutc = take(1ull * B * D1_BINS);
    lo.zero1_begin = off;
    lo.cnt1 = take(4ull * B * D1_BINS);
    lo.sq1 = take(8ull * B * D1_BINS);
    lo.cnt2 = take(4ull * B * SLOT_STRIDE * D2_BINS);
    lo.sq2 = take(8ull * B * SLOT_STRIDE * D2_BINS);
    lo.zero1_mid = off;                                   // the single-pass profile writes the tables above whole
    lo.diag = take(16);
    lo.fresh = take(16);
    lo.layer_flag = take(4ull * (B ? B : 1));
    lo.shist = take(4ull * B * D1_BINS);
    lo.ghist = take(8ull * D1_BINS);
    lo.cursor = take(4ull * (B ? B : 1));
    lo.spill_over = take(4ull * (B ? B : 1));
    lo.rec_cnt = take(4ull * (nc ? nc : 1));              // chunk records start out as "nothing spilled"
    lo.zero1_end = off;
    lo.hprev = take(4ull * B * D1_BINS);
    lo.gprev = take(8ull * D1_BINS);
    lo.pool_prefix = take(4ull * lo.pool_cap);
    lo.pool_big = take(4ull * lo.pool_cap);
    lo.pool_t0 = take(4ull * lo.pool_cap);
    lo.pool_cnt = take(4ull * lo.pool_cap);
    lo.tgt_unsel = take(4 * LJ);
    lo.tgt_base = take(8 * LJ);
    lo.lut1 = take(1ull * B * D1_BINS);
    lo.nslots = take(4ull * (B ? B : 1));
    lo.slot_cnt = take(4ull * (B ? B : 1) * SLOT_STRIDE);
    lo.slot_sq = take(8ull * (B ? B : 1) * SLOT_STRIDE);
    lo.slot_bin = take(4ull * B * SLOT_STRIDE);
    lo.tgt_slot = take(4 * LJ);
    lo.tgt_r = take(4 * LJ);
    lo.tgt_above1 = take(4 * LJ);
    lo.tgt_below = take(8 * LJ);
    lo.sel_prefix = take(4 * LJ);
    lo.sel_above = take(4 * LJ);
    lo.sel_amb = take(4 * LJ);
    lo.ksel = take(4ull * L);
    lo.sel = take(sizeof(SelRec) * (uint64_t)(B ? B : 1));
    lo.zero2_begin = off;
    lo.hist3 = take(4ull * B * D3_BINS);
    lo.zero2_end = off;
    lo.cblk_big = take(4ull * (ncblk ? ncblk : 1));
    lo.tau = take(4ull * (B ? B : 1));
    lo.quota = take(4ull * (B ? B : 1));
    const uint64_t ncb = 4ull * (nc ? nc : 1);
    lo.rec_start = take(ncb); lo.rec_amb = take(ncb);
    lo.c_gt = take(ncb); lo.c_eq = take(ncb); lo.o_base = take(ncb); lo.o_allow = take(ncb);
    lo.tmp_idx = take(4 * lo.tmp_cap); lo.tmp_x = take(4 * lo.tmp_cap);
    lo.row0 = take(8 * lo.dp_cells);
    lo.row1 = take(8 * lo.dp_cells);
    lo.choice = take((uint64_t)L * align_up(lo.dp_cells));
    lo.cprev = take(2ull * L * align_up(std::min<uint64_t>(lo.dp_cells, DP_PAD_WIDE)));
    lo.dp_flags = take(16);
    lo.ncompact = take(16);
    lo.dl_wall = take(4 * LJ); lo.dl_w = take(4 * LJ); lo.dl_jj = take(4 * LJ); lo.dl_e = take(16 * LJ); lo.dl_n = take(4ull * L);
    lo.dl_bad = take(4ull * L);
    lo.dense_E = take(8 * LJ); lo.dense_Kcost = take(4 * LJ); lo.dense_Kout = take(4 * LJ);
    lo.band_lo = take(4ull * (L + 1)); lo.band_hi = take(4ull * (L + 1));
    lo.band_info = take(64);
    lo.live_off = take(4ull * (L + 1)); lo.live_e = take(8 * LJ); lo.live_before = take(8 * LJ);
    lo.live_w = take(4 * LJ); lo.live_jj = take(4 * LJ);
    {
        // a stored row holds a whole number of the forward kernel's 512-thread sweeps (2, 4 or 6 cells per thread)
        const uint64_t cells = std::min<uint64_t>(lo.dp_cells, DP_PAD_WIDE);
        lo.rstride = 512ull * (cells <= 1024 ? 2 : cells <= 2048 ? 4 : cells <= DP_PAD ? 6 : 9);
    }
    lo.rows_g = take(8ull * (L + 1) * lo.rstride);
    lo.total = off;
    return KIMAD_OK;
}

kimad_config_t normalise(const kimad_config_t* cfg) {
    kimad_config_t c{};
    if (cfg) c = *cfg;
    if (c.pair_bytes == 0) c.pair_bytes = c.value_format == KIMAD_VALUES_F16 ? 6 : 8;
    return c;
}

constexpr uint64_t BAND_AUTO_CELLS = 1537;  // rows from this many cost cells on take the banded recurrence by themselves
constexpr uint32_t FALLBACK_GRID = 1024;   // workgroups of a pass that usually has nothing to do

__global__ __launch_bounds__(256) void k_zero16(uint4* p, uint64_t n16) {
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

__global__ __launch_bounds__(64) void k_fill_i32(int32_t* p, uint32_t n, int32_t v) {
    for (uint32_t i = threadIdx.x; i < n; i += 64u) p[i] = v;
}

// Entries of an ascending index list that fall into each layer's range of the flat buffer: two bisections a layer.
__global__ __launch_bounds__(256) void k_layer_counts(const uint32_t* __restrict__ idx, uint64_t pairs,
                                                      const uint64_t* __restrict__ layer_start, uint32_t L, uint64_t* counts) {
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i >= L) return;
    auto first_at_or_above = [&](uint64_t pos) {      // number of entries below position pos
        uint64_t lo = 0, hi = pairs;
        while (lo < hi) {
            const uint64_t mid = (lo + hi) >> 1;
            if ((uint64_t)idx[mid] < pos) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    counts[i] = first_at_or_above(layer_start[i + 1]) - first_at_or_above(layer_start[i]);
}

__global__ __launch_bounds__(256) void k_make_ksel(const uint64_t* K, const kimad::LayerDesc* layers, uint32_t L,
                                                   uint32_t* ksel) {
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    if (i < L) {
        const uint64_t k = K[i];
        ksel[i] = k > layers[i].n ? layers[i].n : (uint32_t)k;
    }
}

}  // namespace

struct kimad_plan {
    Layout lo;
    kimad_config_t cfg;
    std::vector<HostLayer> hl;
    std::vector<uint32_t> ktab;      // host copy of K_ij
    std::vector<uint32_t> kmax;      // K_{i,J-1}
    char* ws = nullptr;
    int device = 0;
    uint32_t main_wgs = 256;         // persistent workgroups of the fused pass (one per compute unit)
    uint32_t chunks_per_wg = 0;
    kimad::ProfileBuffers pb;
    kimad::CompressBuffers cb;
    // optional per-kernel timing (events recorded after every launch)
    bool timing = false;
    std::vector<hipEvent_t> ev;
    std::vector<const char*> ev_name;
    uint32_t ev_n = 0;
    // The small layers (one workgroup each) do not depend on the tiled layers: their kernels run on a
    // side stream, forked from and joined back into the caller's stream with events, so that they
    // overlap the short kernels of the tiled path instead of standing in line with them.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    // The single-pass profile predicts from the exact histogram its previous run on this plan left behind, once
    // there is one (stream order makes it visible).
    bool hist_valid = false;
    ~kimad_plan() {
        for (hipEvent_t e : ev) (void)hipEventDestroy(e);
        if (ev_fork) (void)hipEventDestroy(ev_fork);
        if (ev_join) (void)hipEventDestroy(ev_join);
        if (side) (void)hipStreamDestroy(side);
    }
};

namespace {

template <typename T> T* at(kimad_plan* p, uint64_t off) { return reinterpret_cast<T*>(p->ws + off); }

constexpr uint32_t MAX_EVENTS = 1024;

// Stream for work that may overlap what follows on `s`: the side stream, made to wait for
// everything enqueued on `s` so far.  With per-kernel timing on (or if anything fails) it is `s`
// itself, i.e. plain in-order execution.
hipStream_t fork_side(kimad_plan* p, hipStream_t s) {
    if (p->timing || !p->side) return s;
    if (hipEventRecord(p->ev_fork, s) != hipSuccess) return s;
    if (hipStreamWaitEvent(p->side, p->ev_fork, 0) != hipSuccess) return s;
    return p->side;
}
int join_side(kimad_plan* p, hipStream_t s, hipStream_t used) {
    if (used == s) return KIMAD_OK;
    if (hipEventRecord(p->ev_join, used) != hipSuccess) return KIMAD_ERR_HIP;
    if (hipStreamWaitEvent(s, p->ev_join, 0) != hipSuccess) return KIMAD_ERR_HIP;
    return KIMAD_OK;
}

// With timing on, an event follows every launch; the interval between consecutive events is
// that kernel's duration on the stream.
void mark(kimad_plan* p, hipStream_t s, const char* name) {
    if (!p->timing || p->ev_n >= MAX_EVENTS) return;
    if (hipEventRecord(p->ev[p->ev_n], s) == hipSuccess) p->ev_name[p->ev_n++] = name;
}

#define KLAUNCH(p, s, name, kern, grid, block, ...)                    \
    do {                                                               \
        hipLaunchKernelGGL(kern, grid, block, 0, s, __VA_ARGS__);      \
        if (hipGetLastError() != hipSuccess) return KIMAD_ERR_HIP;     \
        mark(p, s, name);                                              \
    } while (0)

int zero_range(kimad_plan* p, uint64_t begin, uint64_t end, hipStream_t s) {
    const uint64_t n16 = (end - begin) / 16;
    if (n16 == 0) return KIMAD_OK;
    const uint32_t blocks = (uint32_t)std::min<uint64_t>((n16 + 255) / 256, 2048);
    KLAUNCH(p, s, "k_zero16", k_zero16, dim3(blocks), dim3(256), at<uint4>(p, begin), n16);
    return KIMAD_OK;
}

// Histogram passes + scans for a target table (the plan's grid, or one K per layer).
// mark_fresh: the targets are the plan's grid, i.e. this is kimad_profile (see ProfileBuffers::fresh).
// clear: the tables the passes add into (and the profile's "fresh" word) are cleared here; a caller that has
// already cleared them, before it let other kernels of the same call start on the side stream, passes false.
int run_select_passes(kimad_plan* p, const uint32_t* ktab_dev, uint32_t J, double* err_table, hipStream_t s,
                      uint32_t mark_fresh = 0u, bool clear = true) {
    const Layout& lo = p->lo;
    int rc = clear ? zero_range(p, lo.zero1_begin, lo.zero1_end, s) : KIMAD_OK;
    if (rc) return rc;
    if (lo.B) {
        KLAUNCH(p, s, "k_hist1", k_hist1, dim3(lo.ntiles), dim3(256), p->pb);
        KLAUNCH(p, s, "k_scan1", k_scan1, dim3(lo.B), dim3(256), p->pb, ktab_dev, J);
        KLAUNCH(p, s, "k_hist2", k_hist2, dim3(lo.ntiles), dim3(512), p->pb, lo.ntiles, (const uint32_t*)nullptr, 0u);
        KLAUNCH(p, s, "k_scan2", k_scan2, dim3(lo.B), dim3(SCAN2_THREADS), p->pb, ktab_dev, J, err_table, CERT_TOL, 0.0);
        if (err_table) {
            // exact last-digit pass for the entries scan 2 could not certify (usually none)
            KLAUNCH(p, s, "k_hist3p", k_hist3p, dim3(lo.ntiles), dim3(256), p->pb, lo.ntiles);
            KLAUNCH(p, s, "k_scan3p", k_scan3p, dim3(std::min(lo.pool_cap, POOL_GRID)), dim3(256), p->pb, err_table,
                    mark_fresh);
        }
    }
    return KIMAD_OK;
}

// Single-pass profile: sample, predict, one streaming pass, candidate-fed digit-2 slots, and the
// classic recount only for layers whose prediction missed.
// Small layers (one workgroup each, LDS-heavy) go to the side stream once the streaming pass is
// enqueued on `s`: they then run beside the scans that follow it, which occupy a few dozen
// workgroups, instead of taking compute units from the persistent grid of the streaming pass.
// *side gets the stream they were put on (to be joined by the caller).
int launch_small_profile(kimad_plan* p, double* err_table, hipStream_t s, hipStream_t* side,
                         const uint32_t* ktab_dev = nullptr, uint32_t J = 0) {
    const Layout& lo = p->lo;
    if (!lo.S) return KIMAD_OK;
    *side = fork_side(p, s);
    const uint32_t mark_fresh = ktab_dev ? 0u : 1u;       // other targets than the grid do not make a profile to reuse
    KLAUNCH(p, *side, "k_small_profile", k_small_profile, dim3(lo.S), dim3(SMALL_THREADS), p->pb,
            ktab_dev ? ktab_dev : (const uint32_t*)at<uint32_t>(p, lo.ktab), ktab_dev ? J : lo.J, err_table, mark_fresh);
    return KIMAD_OK;
}

int run_fused_profile(kimad_plan* p, double* err_table, uint64_t budget_pairs, hipStream_t s, hipStream_t* side) {
    const Layout& lo = p->lo;
    const uint32_t* ktab = at<uint32_t>(p, lo.ktab);
    if (!lo.B) {
        int rc0 = zero_range(p, lo.zero1_mid, lo.zero1_end, s);
        if (rc0) return rc0;
        return launch_small_profile(p, err_table, s, side);
    }
    int rc = KIMAD_OK;
    if (p->hist_valid && !(p->cfg.flags & KIMAD_CFG_SAMPLE_ALWAYS)) {
        // prediction from the previous profile's exact histogram: no sampling pass, no clearing launch
        KLAUNCH(p, s, "k_predict", k_predict, dim3(lo.B), dim3(256), p->pb, ktab, lo.J, (unsigned long long)budget_pairs,
                (const uint32_t*)p->pb.hprev, (const unsigned long long*)p->pb.gprev, 1u);
    } else {
        rc = zero_range(p, lo.zero1_mid, lo.zero1_end, s);   // the histogram tables are written whole by k_reduce_parts
        if (rc) return rc;
        KLAUNCH(p, s, "k_sample", k_sample, dim3(lo.nswg), dim3(SAMPLE_THREADS), p->pb);
        KLAUNCH(p, s, "k_predict", k_predict, dim3(lo.B), dim3(256), p->pb, ktab, lo.J, (unsigned long long)budget_pairs,
                (const uint32_t*)p->pb.shist, (const unsigned long long*)p->pb.ghist, 0u);
    }
    p->hist_valid = true;
    KLAUNCH(p, s, "k_main", k_main, dim3(p->main_wgs), dim3(FUSED_THREADS), p->pb, p->chunks_per_wg);
    KLAUNCH(p, s, "k_reduce_parts", k_reduce_parts, dim3((LAYER_ENTRIES + REDUCE_ENTRIES - 1) / REDUCE_ENTRIES, lo.B), dim3(256), p->pb);
    rc = launch_small_profile(p, err_table, s, side);
    if (rc) return rc;
    KLAUNCH(p, s, "k_scan1x", k_scan1x, dim3(lo.B), dim3(256), p->pb, ktab, lo.J);
    KLAUNCH(p, s, "k_hist2c", k_hist2c, dim3((lo.nchunks + 256u / SUB_HIST - 1) / (256u / SUB_HIST)), dim3(256), p->pb);
    // fallbacks that normally find nothing to do: small grids
    KLAUNCH(p, s, "k_hist2", k_hist2, dim3(std::min<uint32_t>(lo.ntiles, FALLBACK_GRID)), dim3(512), p->pb, lo.ntiles,
            (const uint32_t*)(at<uint32_t>(p, lo.diag) + 3), 1u);   // layers marked redo only
    KLAUNCH(p, s, "k_scan2", k_scan2, dim3(lo.B), dim3(SCAN2_THREADS), p->pb, ktab, lo.J, err_table, CERT_TOL, SLOT_WIDEN);
    KLAUNCH(p, s, "k_hist3p", k_hist3p, dim3(std::min<uint32_t>(lo.ntiles, FALLBACK_GRID)), dim3(256), p->pb, lo.ntiles);
    KLAUNCH(p, s, "k_scan3p", k_scan3p, dim3(std::min(lo.pool_cap, POOL_GRID)), dim3(256), p->pb, err_table, 1u);
    return KIMAD_OK;
}

// ---- allocation: the same kernels on two homes of their tables ----------------------------------
// Device memory the allocation's kernels work in besides their inputs and outputs.
struct AllocScratch {
    double* row0; double* row1;          // per-layer-launch path only
    uint8_t* choice; uint16_t* cprev;    // [L][pitch]
    uint32_t* flags;                     // 16 bytes
    DpLists dl;
    BandBuffers band;
    double* dense_E; uint32_t* dense_Kcost; uint32_t* dense_Kout;   // [L][J] each: the tables as the dense fallback sees them
    double* rows_g;                      // [(L + 1)][rstride]
    uint32_t rstride;
    uint64_t max_cells;                  // longest row (capacity + 1) the tables hold
};

// Table memory for callers that cannot allocate (kimad_allocate_static): one array per device, inside the
// loaded code object.  Host code never passes the array's name to a kernel: it is a host-side stand-in,
// not a device address; the address of each device's copy is looked up once and kept.
constexpr uint64_t STATIC_SCRATCH_BYTES = 4096ull * 1024ull;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[MAX_DEVICES] = {};

// Address of the current device's copy of `scratch`, or nullptr on a HIP error.
unsigned char* static_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { (void)hipGetLastError(); return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return nullptr; }
        g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
    }
    return g_scratch_ptr[dev];
}

int enqueue_allocate(kimad_plan* p, const AllocScratch& ws, const double* err_table, uint64_t budget_bytes,
                     int32_t* j_out, uint64_t* K_out, uint64_t* offsets_out, int32_t* status_out, hipStream_t s) {
    const Layout& lo = p->lo;
    const uint64_t P = budget_bytes / p->cfg.pair_bytes;
    const uint64_t D = p->cfg.cost_units_D;
    const uint64_t unit = (D == 0 || P <= D) ? 1 : (P + D - 1) / D;
    uint64_t cap = P / unit;
    // Costs above the dearest allocation are unreachable (+inf for ever): cutting the rows there
    // changes no finite cell and so neither the least total nor the smallest cost attaining it.
    const bool dense = (p->cfg.flags & KIMAD_CFG_DENSE_FALLBACK) != 0;
    uint64_t wmax = 0;
    for (uint32_t i = 0; i < lo.L; ++i) {
        uint64_t dearest = p->kmax[i];
        const uint64_t n = p->hl[i].n, pb = p->cfg.pair_bytes;
        if (dense && dearest * pb >= n * 4) dearest = (n * 4 + pb - 1) / pb;   // (costs ascend with j up to the break-even, and no grid point costs more than the dense size)
        wmax += (dearest + unit - 1) / unit;
    }
    if (cap > wmax) cap = wmax;
    if (cap + 1 > ws.max_cells) return KIMAD_ERR_INVALID_ARG;   // budget beyond what the tables were sized for

    AllocBuffers ab;
    ab.E = err_table; ab.Ktab = at<uint32_t>(p, lo.ktab); ab.Kout = ab.Ktab; ab.L = lo.L; ab.J = lo.J;
    ab.unit = unit; ab.cap = (uint32_t)cap;
    ab.row0 = ws.row0; ab.row1 = ws.row1;
    ab.choice = ws.choice; ab.cprev = ws.cprev; ab.stride = align_up(cap + 1);   // row pitch: <= align_up(max_cells)
    ab.j_out = j_out; ab.K_out = K_out; ab.offsets_out = offsets_out; ab.status = status_out;
    ab.flags = ws.flags;
    mark(p, s, "begin");
    if (dense) {
        KLAUNCH(p, s, "k_dense_view", k_dense_view, dim3((lo.L * lo.J + 255) / 256), dim3(256), err_table, ab.Ktab,
                (const LayerDesc*)at<LayerDesc>(p, lo.layers), lo.L, lo.J, p->cfg.pair_bytes, ws.dense_E, ws.dense_Kcost,
                ws.dense_Kout);
        ab.E = ws.dense_E; ab.Ktab = ws.dense_Kcost; ab.Kout = ws.dense_Kout;
    }
    const uint32_t cell_blocks = (uint32_t)((cap + 1 + 255) / 256);
    if (cap + 1 <= DP_PAD_WIDE) {
        const DpLists& dl = ws.dl;
        double* rows_g = ws.rows_g;
        const uint32_t rstride = ws.rstride;
        KLAUNCH(p, s, "k_dp_prep", k_dp_prep, dim3(lo.L), dim3(64), ab, dl);
        const bool band = (p->cfg.flags & KIMAD_CFG_BAND_DP) || cap + 1 >= BAND_AUTO_CELLS;
        if (lo.L <= BAND_MAX_L && band && !(p->cfg.flags & KIMAD_CFG_FULL_DP)) {
            // the recurrence inside the band of cells that Lagrangian bounds leave (same result, a fraction of the cells)
            KLAUNCH(p, s, "k_dp_bounds", k_dp_bounds, dim3(1), dim3(BOUNDS_THREADS), ab, dl, ws.band);
            KLAUNCH(p, s, "k_dp_banded", k_dp_banded, dim3(1), dim3(BANDED_THREADS), ab, ws.band, (const uint32_t*)dl.bad,
                    (int32_t)KIMAD_ERR_INFEASIBLE, (int32_t)KIMAD_ERR_NONFINITE);
            return KIMAD_OK;
        }
        // 512 threads: two waves per SIMD leave each thread the registers for two trips in flight
        const uint32_t cpt = (uint32_t)((cap + 1 + 511) / 512);
        if (cpt <= 2) {
            KLAUNCH(p, s, "k_dp_forward", (k_dp_forward<512, 2>), dim3(1), dim3(512), ab, (const uint32_t*)dl.w,
                    (const double*)dl.e, (const uint32_t*)dl.n, rows_g, rstride);
        } else if (cpt <= 4) {
            KLAUNCH(p, s, "k_dp_forward", (k_dp_forward<512, 4>), dim3(1), dim3(512), ab, (const uint32_t*)dl.w,
                    (const double*)dl.e, (const uint32_t*)dl.n, rows_g, rstride);
        } else if (cpt <= 6) {
            KLAUNCH(p, s, "k_dp_forward", (k_dp_forward<512, 6>), dim3(1), dim3(512), ab, (const uint32_t*)dl.w,
                    (const double*)dl.e, (const uint32_t*)dl.n, rows_g, rstride);
        } else {
            KLAUNCH(p, s, "k_dp_forward", (k_dp_forward<512, 9, DP_PAD_WIDE, DP_LIST_CAP_WIDE>), dim3(1), dim3(512), ab,
                    (const uint32_t*)dl.w, (const double*)dl.e, (const uint32_t*)dl.n, rows_g, rstride);
        }
        KLAUNCH(p, s, "k_dp_choice", k_dp_choice, dim3(cell_blocks, lo.L), dim3(256), ab, dl, (const double*)rows_g, rstride);
        KLAUNCH(p, s, "k_dp_walk", k_dp_walk, dim3(1), dim3(1024), ab, (const double*)(rows_g + (size_t)lo.L * rstride),
                (const uint32_t*)dl.bad, (int32_t)KIMAD_ERR_INFEASIBLE, (int32_t)KIMAD_ERR_NONFINITE);
    } else {
        // (clears with a kernel, not hipMemsetAsync: the call may be recorded into a graph)
        KLAUNCH(p, s, "k_zero16", k_zero16, dim3(1), dim3(256), reinterpret_cast<uint4*>(ws.flags), (uint64_t)1);
        KLAUNCH(p, s, "k_dp_init", k_dp_init, dim3(std::min<uint32_t>(cell_blocks, 1024)), dim3(256), ab);
        double* rows[2] = {ab.row0, ab.row1};
        for (uint32_t i = 0; i < lo.L; ++i) {
            KLAUNCH(p, s, "k_dp_layer", k_dp_layer, dim3(cell_blocks), dim3(256), ab, i, rows[i & 1], rows[(i + 1) & 1]);
        }
        KLAUNCH(p, s, "k_dp_final", k_dp_final, dim3(1), dim3(1024), ab, (const double*)rows[lo.L & 1],
                (int32_t)KIMAD_ERR_INFEASIBLE, (int32_t)KIMAD_ERR_NONFINITE);
    }
    return KIMAD_OK;
}

}  // namespace

extern "C" {

int kimad_workspace_bytes(const uint64_t* n, uint32_t L, uint32_t J, const kimad_config_t* cfg, uint64_t* bytes_out) {
    if (!bytes_out) return KIMAD_ERR_INVALID_ARG;
    Layout lo;
    const int rc = make_layout(n, L, J, normalise(cfg), lo, nullptr);
    if (rc) return rc;
    *bytes_out = lo.total;
    return KIMAD_OK;
}

int kimad_plan_create(const kimad_layer_t* layers, uint32_t L, const double* ratios, uint32_t J,
                      const kimad_config_t* cfg, void* workspace, uint64_t workspace_bytes, void* stream,
                      kimad_plan_t** plan_out) {
    if (!layers || !ratios || !workspace || !plan_out) return KIMAD_ERR_INVALID_ARG;
    if (L == 0 || L > 65535 || J == 0 || J > KIMAD_MAX_J) return KIMAD_ERR_INVALID_ARG;
    if (cfg && cfg->value_format > KIMAD_VALUES_F16) return KIMAD_ERR_INVALID_ARG;
    if (((uintptr_t)workspace) % ALIGN) return KIMAD_ERR_INVALID_ARG;
    for (uint32_t j = 0; j < J; ++j) {
        if (!(ratios[j] > 0.0) || !(ratios[j] <= 1.0)) return KIMAD_ERR_INVALID_ARG;
        if (j && !(ratios[j] > ratios[j - 1])) return KIMAD_ERR_INVALID_ARG;
    }
    std::vector<uint64_t> n(L);
    for (uint32_t i = 0; i < L; ++i) {
        if (!layers[i].g || !layers[i].h) return KIMAD_ERR_INVALID_ARG;
        if (((uintptr_t)layers[i].g) % 4 || ((uintptr_t)layers[i].h) % 4) return KIMAD_ERR_INVALID_ARG;
        n[i] = layers[i].n;
    }
    kimad_plan* p = new (std::nothrow) kimad_plan();
    if (!p) return KIMAD_ERR_INVALID_ARG;
    p->cfg = normalise(cfg);
    PartTables pt;
    int rc = make_layout(n.data(), L, J, p->cfg, p->lo, &p->hl, &pt);
    if (rc) { delete p; return rc; }
    if (workspace_bytes < p->lo.total) { delete p; return KIMAD_ERR_WORKSPACE_TOO_SMALL; }
    p->ws = static_cast<char*>(workspace);
    if (hipGetDevice(&p->device) != hipSuccess) { delete p; return KIMAD_ERR_HIP; }
    (void)static_scratch_of_current_device();   // set-up: the address of this device's fixed tables is known from here on
    const Layout& lo = p->lo;

    // host tables
    std::vector<LayerDesc> ld(L);
    std::vector<uint32_t> tile_layer(lo.ntiles ? lo.ntiles : 1), chunk_big(lo.nchunks ? lo.nchunks : 1);
    std::vector<uint32_t> chunk_first(lo.nchunks ? lo.nchunks : 1);
    std::vector<uint32_t> big_layer(lo.B ? lo.B : 1), small_layer(lo.S ? lo.S : 1);
    std::vector<uint64_t> big_tmp0(lo.B ? lo.B : 1);
    std::vector<uint32_t> swg_layer(lo.nswg ? lo.nswg : 1), swg_first(lo.nswg ? lo.nswg : 1);
    std::vector<uint32_t> cblk_big(lo.ncblk ? lo.ncblk : 1);
    p->ktab.resize((size_t)L * J);
    p->kmax.resize(L);
    uint32_t si = 0;
    for (uint32_t i = 0; i < L; ++i) {
        HostLayer& h = p->hl[i];
        h.mis = (uint32_t)((((uintptr_t)layers[i].g) / 4) & 3u);
        h.hvec = ((((uintptr_t)layers[i].h) / 4) & 3u) == h.mis;
        LayerDesc& d = ld[i];
        d.g = layers[i].g; d.h = layers[i].h; d.n = h.n; d.mis = h.mis; d.hvec = h.hvec; d.big = h.big;
        if (h.big >= 0) {
            // Tiles and chunks are reserved for the worst misalignment; positions past the end of
            // the layer load nothing.
            for (uint32_t t = 0; t < h.ntiles; ++t) tile_layer[h.tile0 + t] = i;
            for (uint32_t c = 0; c < h.nchunks; ++c) { chunk_big[h.chunk0 + c] = (uint32_t)h.big; chunk_first[h.chunk0 + c] = h.chunk0; }
            d.tile0 = h.tile0; d.ntiles = h.ntiles; d.chunk0 = h.chunk0; d.nchunks = h.nchunks;
            d.sstride = h.sstride; d.cblk0 = h.cblk0; d.tmp0 = h.tmp0; d.tmp_cap = h.tmp_cap; d.pad = 0;
            for (uint32_t k = 0; k < h.ncblk; ++k) cblk_big[h.cblk0 + k] = (uint32_t)h.big;
            for (uint32_t w = 0; w < h.nswg; ++w) {
                swg_layer[h.swg0 + w] = i;
                swg_first[h.swg0 + w] = w * SAMPLE_GROUPS_PER_WG;
            }
            big_layer[h.big] = i;
            big_tmp0[h.big] = h.tmp0;
        } else {
            d.tile0 = d.ntiles = d.chunk0 = d.nchunks = 0;
            d.sstride = 1; d.cblk0 = 0; d.tmp0 = 0; d.tmp_cap = 0; d.pad = 0;
            small_layer[si++] = i;
        }
        for (uint32_t j = 0; j < J; ++j) p->ktab[(size_t)i * J + j] = grid_size_K(ratios[j], h.n);
        p->kmax[i] = p->ktab[(size_t)i * J + J - 1];
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto up = [&](uint64_t off, const void* src, size_t bytes) {
        return hipMemcpyAsync(p->ws + off, src, bytes, hipMemcpyHostToDevice, s) == hipSuccess;
    };
    bool ok = up(lo.layers, ld.data(), sizeof(LayerDesc) * L) && up(lo.ktab, p->ktab.data(), 4ull * L * J) &&
              up(lo.tile_layer, tile_layer.data(), 4ull * tile_layer.size()) &&
              up(lo.chunk_big, chunk_big.data(), 4ull * chunk_big.size()) &&
              up(lo.chunk_first, chunk_first.data(), 4ull * chunk_first.size()) &&
              up(lo.big_layer, big_layer.data(), 4ull * big_layer.size()) &&
              up(lo.big_tmp0, big_tmp0.data(), 8ull * big_tmp0.size()) &&
              up(lo.wg_part0, pt.wg_part0.data(), 4ull * pt.wg_part0.size()) &&
              up(lo.big_part0, pt.big_part0.data(), 4ull * pt.big_part0.size()) &&
              up(lo.big_nparts, pt.big_nparts.data(), 4ull * pt.big_nparts.size()) &&
              up(lo.small_layer, small_layer.data(), 4ull * small_layer.size()) &&
              up(lo.swg_layer, swg_layer.data(), 4ull * swg_layer.size()) &&
              up(lo.swg_first, swg_first.data(), 4ull * swg_first.size()) &&
              up(lo.cblk_big, cblk_big.data(), 4ull * cblk_big.size());
    ok = ok && hipStreamSynchronize(s) == hipSuccess;     // host vectors go out of scope below
    if (!ok) { delete p; return KIMAD_ERR_HIP; }

    ProfileBuffers& pb = p->pb;
    pb.layers = at<LayerDesc>(p, lo.layers);
    pb.tile_layer = at<uint32_t>(p, lo.tile_layer);
    pb.big_layer = at<uint32_t>(p, lo.big_layer);
    pb.small_layer = at<uint32_t>(p, lo.small_layer);
    pb.tile_elems = lo.tile_elems;
    pb.cnt1 = at<uint32_t>(p, lo.cnt1); pb.sq1 = at<uint64_t>(p, lo.sq1);
    pb.lut1 = at<uint8_t>(p, lo.lut1); pb.nslots = at<uint32_t>(p, lo.nslots); pb.slot_bin = at<uint32_t>(p, lo.slot_bin);
    pb.slot_cnt = at<uint32_t>(p, lo.slot_cnt); pb.slot_sq = at<uint64_t>(p, lo.slot_sq);
    pb.cnt2 = at<uint32_t>(p, lo.cnt2); pb.sq2 = at<uint64_t>(p, lo.sq2);
    pb.tgt_slot = at<uint32_t>(p, lo.tgt_slot); pb.tgt_r = at<uint32_t>(p, lo.tgt_r);
    pb.tgt_above1 = at<uint32_t>(p, lo.tgt_above1); pb.tgt_below = at<double>(p, lo.tgt_below);
    pb.sel_prefix = at<uint32_t>(p, lo.sel_prefix); pb.sel_above = at<uint32_t>(p, lo.sel_above);
    pb.sel_amb = at<uint32_t>(p, lo.sel_amb); pb.diag = at<uint32_t>(p, lo.diag);
    pb.fresh = at<uint32_t>(p, lo.fresh);
    pb.hprev = at<uint32_t>(p, lo.hprev); pb.gprev = at<unsigned long long>(p, lo.gprev);
    pb.layer_flag = at<uint32_t>(p, lo.layer_flag);
    pb.pool_prefix = at<uint32_t>(p, lo.pool_prefix); pb.pool_big = at<uint32_t>(p, lo.pool_big);
    pb.pool_t0 = at<uint32_t>(p, lo.pool_t0); pb.pool_cnt = at<uint32_t>(p, lo.pool_cnt);
    pb.pool_hist = at<uint32_t>(p, lo.pool_hist); pb.pool_cap = lo.pool_cap;
    pb.tgt_unsel = at<uint32_t>(p, lo.tgt_unsel); pb.tgt_base = at<double>(p, lo.tgt_base);
    pb.state = at<LayerState>(p, lo.state); pb.big_tmp0 = at<uint64_t>(p, lo.big_tmp0);
    pb.parts = at<unsigned long long>(p, lo.parts); pb.wg_part0 = at<uint32_t>(p, lo.wg_part0);
    pb.big_part0 = at<uint32_t>(p, lo.big_part0); pb.big_nparts = at<uint32_t>(p, lo.big_nparts);
    pb.chunk_big = at<uint32_t>(p, lo.chunk_big); pb.chunk_first = at<uint32_t>(p, lo.chunk_first); pb.nchunks_total = lo.nchunks;
    pb.swg_layer = at<uint32_t>(p, lo.swg_layer); pb.swg_first = at<uint32_t>(p, lo.swg_first);
    pb.shist = at<uint32_t>(p, lo.shist); pb.ghist = at<unsigned long long>(p, lo.ghist);
    pb.lutc = at<uint8_t>(p, lo.lutc); pb.cursor = at<uint32_t>(p, lo.cursor);
    pb.spill_over = at<uint32_t>(p, lo.spill_over);
    pb.rec_start = at<uint32_t>(p, lo.rec_start); pb.rec_cnt = at<uint32_t>(p, lo.rec_cnt);
    pb.tmp_idx = at<uint32_t>(p, lo.tmp_idx); pb.tmp_x = at<float>(p, lo.tmp_x);
    p->main_wgs = lo.main_wgs;
    p->chunks_per_wg = lo.chunks_per_wg;
    // Layer states start as "nothing spilled, nothing cached".
    if (hipMemsetAsync(p->ws + lo.state, 0, sizeof(LayerState) * (uint64_t)(lo.B ? lo.B : 1), s) != hipSuccess ||
        hipMemsetAsync(p->ws + lo.zero2_begin, 0, lo.zero2_end - lo.zero2_begin, s) != hipSuccess ||
        hipMemsetAsync(p->ws + lo.band_info, 0, 64, s) != hipSuccess ||
        hipMemsetAsync(p->ws + lo.fresh, 0, 16, s) != hipSuccess ||
        hipMemsetAsync(p->ws + lo.gprev, 0, 8ull * D1_BINS, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) { delete p; return KIMAD_ERR_HIP; }

    CompressBuffers& cb = p->cb;
    cb.layers = pb.layers; cb.chunk_layer = pb.tile_layer; cb.big_layer = pb.big_layer; cb.small_layer = pb.small_layer;
    cb.tile_elems = lo.tile_elems; cb.L = L; cb.B = lo.B; cb.J = J;
    cb.Ktab = at<uint32_t>(p, lo.ktab);
    cb.sel_prefix = pb.sel_prefix; cb.sel_above = pb.sel_above; cb.sel_amb = pb.sel_amb;
    cb.sel = at<SelRec>(p, lo.sel); cb.cursor = pb.cursor; cb.hist3 = at<uint32_t>(p, lo.hist3);
    cb.tau = at<uint32_t>(p, lo.tau); cb.quota = at<uint32_t>(p, lo.quota);
    cb.rec_start = at<uint32_t>(p, lo.rec_start); cb.rec_cnt = at<uint32_t>(p, lo.rec_cnt);
    cb.chunk_first = at<uint32_t>(p, lo.chunk_first); cb.tmp_total = lo.tmp_cap;
    cb.rec_amb = at<uint32_t>(p, lo.rec_amb); cb.c_gt = at<uint32_t>(p, lo.c_gt); cb.c_eq = at<uint32_t>(p, lo.c_eq);
    cb.o_base = at<uint32_t>(p, lo.o_base); cb.o_allow = at<uint32_t>(p, lo.o_allow);
    cb.cblk_big = at<uint32_t>(p, lo.cblk_big);
    cb.tmp_idx = at<uint32_t>(p, lo.tmp_idx); cb.tmp_x = at<float>(p, lo.tmp_x);
    cb.ncompact = at<uint32_t>(p, lo.ncompact);
    cb.fresh = pb.fresh;
    cb.state = pb.state;
    cb.K = nullptr; cb.offsets = nullptr; cb.idx_out = nullptr; cb.val_out = nullptr; cb.capacity_pairs = 0;
    cb.value_f16 = 0;
    cb.status = nullptr;
    if (lo.S && lo.B) {
        // default priority; without the side stream everything simply runs in order on the caller's stream
        if (hipStreamCreateWithFlags(&p->side, hipStreamNonBlocking) != hipSuccess) p->side = nullptr;
        if (p->side && (hipEventCreateWithFlags(&p->ev_fork, hipEventDisableTiming) != hipSuccess ||
                        hipEventCreateWithFlags(&p->ev_join, hipEventDisableTiming) != hipSuccess)) {
            (void)hipStreamDestroy(p->side);
            p->side = nullptr;
        }
    }
    *plan_out = p;
    return KIMAD_OK;
}

int kimad_plan_destroy(kimad_plan_t* plan) {
    delete plan;
    return KIMAD_OK;
}

int kimad_plan_grid_sizes(const kimad_plan_t* plan, uint64_t* K_table_out) {
    if (!plan || !K_table_out) return KIMAD_ERR_INVALID_ARG;
    for (size_t t = 0; t < plan->ktab.size(); ++t) K_table_out[t] = plan->ktab[t];
    return KIMAD_OK;
}

int kimad_profile(kimad_plan_t* p, double* err_table, uint64_t budget_hint_bytes, void* stream) {
    if (!p || !err_table) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Layout& lo = p->lo;
    mark(p, s, "begin");
    hipStream_t ss = s;
    int rc;
    if (p->cfg.flags & KIMAD_CFG_CLASSIC_PROFILE) {
        // (the clearing comes before the fork: the small layers' kernel on the side stream marks the profile as
        // fresh, and in a plan without tiled layers nothing marks it again)
        rc = zero_range(p, lo.zero1_begin, lo.zero1_end, s);
        if (!rc) rc = launch_small_profile(p, err_table, s, &ss);
        if (!rc) rc = run_select_passes(p, at<uint32_t>(p, lo.ktab), lo.J, err_table, s, 1u, false);
    } else {
        rc = run_fused_profile(p, err_table, budget_hint_bytes / p->cfg.pair_bytes, s, &ss);
    }
    const int rj = join_side(p, s, ss);       // always join, also after an error
    return rc ? rc : rj;
}

int kimad_allocate(kimad_plan_t* p, const double* err_table, uint64_t budget_bytes, int32_t* j_out, uint64_t* K_out,
                   uint64_t* offsets_out, int32_t* status_out, void* stream) {
    if (!p || !err_table || !j_out || !K_out || !offsets_out || !status_out) return KIMAD_ERR_INVALID_ARG;
    const Layout& lo = p->lo;
    AllocScratch ws;
    ws.row0 = at<double>(p, lo.row0); ws.row1 = at<double>(p, lo.row1);
    ws.choice = at<uint8_t>(p, lo.choice); ws.cprev = at<uint16_t>(p, lo.cprev);
    ws.flags = at<uint32_t>(p, lo.dp_flags);
    ws.dl.wall = at<uint32_t>(p, lo.dl_wall); ws.dl.w = at<uint32_t>(p, lo.dl_w); ws.dl.jj = at<uint32_t>(p, lo.dl_jj);
    ws.dl.e = at<double>(p, lo.dl_e); ws.dl.n = at<uint32_t>(p, lo.dl_n); ws.dl.bad = at<uint32_t>(p, lo.dl_bad);
    ws.dense_E = at<double>(p, lo.dense_E); ws.dense_Kcost = at<uint32_t>(p, lo.dense_Kcost);
    ws.dense_Kout = at<uint32_t>(p, lo.dense_Kout);
    ws.band.lo = at<uint32_t>(p, lo.band_lo); ws.band.hi = at<uint32_t>(p, lo.band_hi);
    ws.band.info = at<uint32_t>(p, lo.band_info);
    ws.band.live_off = at<uint32_t>(p, lo.live_off); ws.band.live_e = at<double>(p, lo.live_e);
    ws.band.live_before = at<double>(p, lo.live_before); ws.band.live_w = at<uint32_t>(p, lo.live_w);
    ws.band.live_jj = at<uint32_t>(p, lo.live_jj);
    ws.rows_g = at<double>(p, lo.rows_g);
    ws.rstride = (uint32_t)lo.rstride;
    ws.max_cells = lo.dp_cells;
    return enqueue_allocate(p, ws, err_table, budget_bytes, j_out, K_out, offsets_out, status_out,
                            static_cast<hipStream_t>(stream));
}

int kimad_allocate_static(kimad_plan_t* p, const double* err_table, uint64_t budget_bytes, int32_t* j_out,
                          uint64_t* K_out, uint64_t* offsets_out, int32_t* status_out, void* stream) {
    if (!p || !err_table || !j_out || !K_out || !offsets_out || !status_out) return KIMAD_ERR_INVALID_ARG;
    const Layout& lo = p->lo;
    if (lo.L > KIMAD_STATIC_MAX_L) return KIMAD_ERR_STATIC_LIMIT;
    unsigned char* base = static_scratch_of_current_device();
    if (!base) return KIMAD_ERR_HIP;
    // Fixed carving of the array for the largest case it admits (KIMAD_STATIC_MAX_L layers, KIMAD_MAX_J
    // ratios, rows of KIMAD_STATIC_MAX_CELLS cost cells), so the offsets do not depend on the plan.
    constexpr uint64_t LJ = (uint64_t)KIMAD_STATIC_MAX_L * KIMAD_MAX_J;
    constexpr uint64_t CELLS = KIMAD_STATIC_MAX_CELLS;
    uint64_t off = 0;
    auto take = [&](uint64_t bytes) { unsigned char* q = base + off; off = align_up(off + bytes); return q; };
    AllocScratch ws;
    ws.row0 = nullptr; ws.row1 = nullptr;                       // only the per-layer-launch path uses them
    ws.choice = reinterpret_cast<uint8_t*>(take((uint64_t)KIMAD_STATIC_MAX_L * CELLS));
    ws.cprev = reinterpret_cast<uint16_t*>(take(2ull * KIMAD_STATIC_MAX_L * CELLS));
    ws.flags = reinterpret_cast<uint32_t*>(take(16));
    ws.dl.wall = reinterpret_cast<uint32_t*>(take(4 * LJ)); ws.dl.w = reinterpret_cast<uint32_t*>(take(4 * LJ));
    ws.dl.jj = reinterpret_cast<uint32_t*>(take(4 * LJ)); ws.dl.e = reinterpret_cast<double*>(take(16 * LJ));
    ws.dl.n = reinterpret_cast<uint32_t*>(take(4ull * KIMAD_STATIC_MAX_L));
    ws.dl.bad = reinterpret_cast<uint32_t*>(take(4ull * KIMAD_STATIC_MAX_L));
    ws.dense_E = reinterpret_cast<double*>(take(8 * LJ)); ws.dense_Kcost = reinterpret_cast<uint32_t*>(take(4 * LJ));
    ws.dense_Kout = reinterpret_cast<uint32_t*>(take(4 * LJ));
    ws.band.lo = reinterpret_cast<uint32_t*>(take(4ull * (KIMAD_STATIC_MAX_L + 1)));
    ws.band.hi = reinterpret_cast<uint32_t*>(take(4ull * (KIMAD_STATIC_MAX_L + 1)));
    ws.band.info = reinterpret_cast<uint32_t*>(take(64));
    ws.band.live_off = reinterpret_cast<uint32_t*>(take(4ull * (KIMAD_STATIC_MAX_L + 1)));
    ws.band.live_e = reinterpret_cast<double*>(take(8 * LJ)); ws.band.live_before = reinterpret_cast<double*>(take(8 * LJ));
    ws.band.live_w = reinterpret_cast<uint32_t*>(take(4 * LJ)); ws.band.live_jj = reinterpret_cast<uint32_t*>(take(4 * LJ));
    ws.rows_g = reinterpret_cast<double*>(take(8ull * (KIMAD_STATIC_MAX_L + 1) * CELLS));
    ws.rstride = (uint32_t)CELLS;
    ws.max_cells = CELLS;
    static_assert(KIMAD_STATIC_MAX_CELLS == 1024, "a stored row is two sweeps of the forward kernel's 512 threads");
    if (off > STATIC_SCRATCH_BYTES) return KIMAD_ERR_INTERNAL;
    const int rc = enqueue_allocate(p, ws, err_table, budget_bytes, j_out, K_out, offsets_out, status_out,
                                    static_cast<hipStream_t>(stream));
    return rc == KIMAD_ERR_INVALID_ARG ? KIMAD_ERR_STATIC_LIMIT : rc;   // the one argument left to reject: rows too long
}

int kimad_compress_ef(kimad_plan_t* p, const uint64_t* K, const uint64_t* offsets, uint32_t* idx_out, void* val_out,
                      uint64_t capacity_pairs, uint32_t flags, int32_t* status_out, void* stream) {
    if (!p || !K || !offsets || !idx_out || !val_out || !status_out) return KIMAD_ERR_INVALID_ARG;
    if (flags & ~KIMAD_REUSE_PROFILE) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Layout& lo = p->lo;
    CompressBuffers cb = p->cb;
    cb.K = K; cb.offsets = offsets; cb.idx_out = idx_out; cb.val_out = static_cast<float*>(val_out);
    cb.value_f16 = p->cfg.value_format == KIMAD_VALUES_F16 ? 1u : 0u;
    cb.capacity_pairs = capacity_pairs; cb.status = status_out;
    mark(p, s, "begin");
    if (!(flags & KIMAD_REUSE_PROFILE)) {
        // select from scratch: the two histogram passes with one target per layer
        uint32_t* ksel = at<uint32_t>(p, lo.ksel);
        KLAUNCH(p, s, "k_make_ksel", k_make_ksel, dim3((lo.L + 255) / 256), dim3(256), K, cb.layers, lo.L, ksel);
        int rc = run_select_passes(p, ksel, 1, nullptr, s);
        if (rc) return rc;
        cb.Ktab = ksel;
        cb.J = 1;
    }
    // (the last-digit histograms are zero here: k_resolve clears what it has read)
    KLAUNCH(p, s, "k_lookup", k_lookup, dim3(1), dim3(256), cb, (int32_t)KIMAD_ERR_OFFGRID,
            (int32_t)KIMAD_ERR_BAD_OFFSETS, (int32_t)KIMAD_ERR_STALE_PROFILE,
            (uint32_t)((flags & KIMAD_REUSE_PROFILE) ? 1u : 0u));
    hipStream_t ss = s;
    if (lo.S) {
        ss = fork_side(p, s);                 // after the lookup: the small layers read its verdict
        KLAUNCH(p, ss, "k_small_compress", k_small_compress, dim3(lo.S), dim3(SMALL_THREADS), cb);
    }
    if (lo.B) {
        const uint32_t* chunk_big = at<uint32_t>(p, lo.chunk_big);
        const uint32_t cblocks = (lo.nchunks + CHUNKS_PER_WG - 1) / CHUNKS_PER_WG;
        const uint32_t nblocks = (lo.nchunks + 256u / SUB_COUNT - 1) / (256u / SUB_COUNT);   // where candidates are only counted
        const uint32_t hblocks = (lo.nchunks + 256u / SUB_HIST - 1) / (256u / SUB_HIST);      // and where they are histogrammed
        KLAUNCH(p, s, "k_candidates", k_candidates, dim3(hblocks + std::min<uint32_t>(lo.ntiles, 4u * FALLBACK_GRID)), dim3(256), cb,
                lo.nchunks, chunk_big, hblocks, lo.ntiles, (int32_t)KIMAD_ERR_INTERNAL);
        KLAUNCH(p, s, "k_resolve", k_resolve, dim3(lo.B), dim3(256), cb);
        KLAUNCH(p, s, "k_chunk_count", k_chunk_count, dim3(nblocks), dim3(256), cb, lo.nchunks, chunk_big);
        KLAUNCH(p, s, "k_chunk_bases", k_chunk_bases, dim3(lo.ncblk), dim3(1024), cb);
        KLAUNCH(p, s, "k_finalize", k_finalize, dim3(cblocks), dim3(256), cb, lo.nchunks, chunk_big);
    }
    return join_side(p, s, ss);
}

int kimad_step(kimad_plan_t* p, uint64_t budget_bytes, double* err_table, int32_t* j_out, uint64_t* K_out,
               uint64_t* offsets_out, uint32_t* idx_out, void* val_out, uint64_t capacity_pairs, int32_t* status_out,
               void* stream) {
    if (!status_out) return KIMAD_ERR_INVALID_ARG;
    int rc = kimad_profile(p, err_table, budget_bytes, stream);
    if (rc) return rc;
    rc = kimad_allocate(p, err_table, budget_bytes, j_out, K_out, offsets_out, status_out, stream);
    if (rc) return rc;
    // On an allocation failure K and offsets are zero-filled, so the compression writes nothing.
    return kimad_compress_ef(p, K_out, offsets_out, idx_out, val_out, capacity_pairs, KIMAD_REUSE_PROFILE,
                             status_out + 1, stream);
}

int kimad_profile_diagnostics(kimad_plan_t* p, uint32_t* out4, void* stream) {
    if (!p || !out4) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(out4, p->ws + p->lo.diag, 16, hipMemcpyDeviceToHost, s) != hipSuccess) return KIMAD_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return KIMAD_ERR_HIP;
    return KIMAD_OK;
}

int kimad_allocate_diagnostics(kimad_plan_t* p, uint32_t* out4, void* stream) {
    if (!p || !out4) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(out4, p->ws + p->lo.band_info, 16, hipMemcpyDeviceToHost, s) != hipSuccess) return KIMAD_ERR_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return KIMAD_ERR_HIP;
    return KIMAD_OK;
}

#ifdef KIMAD_STAMPS
int kimad_debug_layout(const uint64_t* n, uint32_t L, uint32_t J, const kimad_config_t* cfg, uint64_t* out) {
    Layout lo;
    int rc = make_layout(n, L, J, *cfg, lo, nullptr);
    if (rc) return rc;
    out[0] = lo.parts; out[1] = lo.small_layer; out[2] = lo.state; out[3] = lo.cnt1; out[4] = lo.rec_cnt; out[5] = lo.hprev;
    out[6] = lo.pool_prefix; out[7] = lo.sel; out[8] = lo.hist3; out[9] = lo.rec_start; out[10] = lo.tmp_idx;
    out[11] = lo.tmp_x; out[12] = lo.row0; out[13] = lo.total;
    return 0;
}
int kimad_debug_band_info(kimad_plan_t* p, uint32_t* out16) {
    if (hipMemcpy(out16, p->ws + p->lo.band_info, 64, hipMemcpyDeviceToHost) != hipSuccess) return KIMAD_ERR_HIP;
    return KIMAD_OK;
}
#endif

int kimad_plan_set_timing(kimad_plan_t* p, int enable) {
    if (!p) return KIMAD_ERR_INVALID_ARG;
    if (enable && p->ev.empty()) {
        p->ev.resize(MAX_EVENTS);
        p->ev_name.assign(MAX_EVENTS, "");
        for (uint32_t k = 0; k < MAX_EVENTS; ++k)
            if (hipEventCreate(&p->ev[k]) != hipSuccess) { p->ev.resize(k); p->timing = false; return KIMAD_ERR_HIP; }
    }
    p->timing = enable != 0;
    p->ev_n = 0;
    return KIMAD_OK;
}

int kimad_plan_get_timings(kimad_plan_t* p, char* names, uint32_t names_bytes, float* ms, uint32_t max_entries,
                           uint32_t* count_out) {
    if (!p || !names || !ms || !count_out) return KIMAD_ERR_INVALID_ARG;
    uint32_t n = 0;
    size_t pos = 0;
    if (p->ev_n) {
        if (hipEventSynchronize(p->ev[p->ev_n - 1]) != hipSuccess) return KIMAD_ERR_HIP;
        for (uint32_t k = 1; k < p->ev_n && n < max_entries; ++k) {
            if (std::strcmp(p->ev_name[k], "begin") == 0) continue;   // gap between two calls
            float t = 0.f;
            if (hipEventElapsedTime(&t, p->ev[k - 1], p->ev[k]) != hipSuccess) return KIMAD_ERR_HIP;
            const size_t len = std::strlen(p->ev_name[k]);
            if (pos + len + 2 > names_bytes) break;
            std::memcpy(names + pos, p->ev_name[k], len);
            pos += len;
            names[pos++] = '\n';
            ms[n++] = t;
        }
    }
    if (names_bytes) names[pos < names_bytes ? pos : names_bytes - 1] = 0;
    *count_out = n;
    p->ev_n = 0;
    return KIMAD_OK;
}

int kimad_plan_layer_states(kimad_plan_t* p, uint32_t* out, uint32_t max_layers, uint32_t* count_out, void* stream) {
    if (!p || !out || !count_out) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t B = std::min<uint32_t>(p->lo.B, max_layers);
    std::vector<LayerState> st(B ? B : 1);
    std::vector<SelRec> sel(B ? B : 1);
    if (B) {
        if (hipMemcpyAsync(st.data(), p->ws + p->lo.state, sizeof(LayerState) * B, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipMemcpyAsync(sel.data(), p->ws + p->lo.sel, sizeof(SelRec) * B, hipMemcpyDeviceToHost, s) != hipSuccess ||
            hipStreamSynchronize(s) != hipSuccess) return KIMAD_ERR_HIP;
    }
    uint32_t b = 0;
    for (uint32_t i = 0; i < p->lo.L && b < B; ++i) {
        if (p->hl[i].big < 0) continue;
        uint32_t* o = out + 8 * (size_t)b;
        o[0] = i; o[1] = st[b].spill_bin; o[2] = st[b].nslots_d; o[3] = st[b].nslots_t;
        o[4] = st[b].redo; o[5] = st[b].spill_cnt; o[6] = st[b].spill_valid; o[7] = sel[b].mode;
        ++b;
    }
    *count_out = b;
    return KIMAD_OK;
}

int kimad_server_apply(const kimad_payload_t* payloads, float* const* u_hat, const double* weights, uint32_t M,
                       const uint64_t* layer_start, uint32_t L, uint64_t d, float* x, double gamma,
                       int32_t* status_out, void* stream) {
    static_assert(KIMAD_MAX_WORKERS == MAX_WORKERS, "header and kernel constants");
    if (!payloads || !u_hat || !weights || !layer_start || M == 0 || M > KIMAD_MAX_WORKERS || L == 0 || d == 0 ||
        !status_out)
        return KIMAD_ERR_INVALID_ARG;
    ServerArgs a{};
    bool vec_ok = x && (reinterpret_cast<uintptr_t>(x) % 16 == 0);
    for (uint32_t m = 0; m < M; ++m) {
        if (!payloads[m].idx || !payloads[m].val || !payloads[m].offsets || !u_hat[m]) return KIMAD_ERR_INVALID_ARG;
        if (payloads[m].value_format > KIMAD_VALUES_F16) return KIMAD_ERR_INVALID_ARG;
        a.u_hat[m] = u_hat[m]; a.w[m] = weights[m];
        vec_ok = vec_ok && (reinterpret_cast<uintptr_t>(u_hat[m]) % 16 == 0);
    }
    a.M = M; a.d = d;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_fill_i32, dim3(1), dim3(64), 0, s, status_out, M, 0);
    if (hipGetLastError() != hipSuccess) return KIMAD_ERR_HIP;
    // payload sizes live on the device: a fixed grid strides over whatever the worker sent
    for (uint32_t m = 0; m < M; ++m) {
        hipLaunchKernelGGL(k_server_decode, dim3(1024), dim3(256), 0, s, payloads[m].idx, payloads[m].val,
                           payloads[m].offsets, payloads[m].capacity_pairs, u_hat[m], layer_start, L, d,
                           status_out + m, (int32_t)KIMAD_ERR_BAD_PAYLOAD,
                           payloads[m].value_format == KIMAD_VALUES_F16 ? 1u : 0u);
        if (hipGetLastError() != hipSuccess) return KIMAD_ERR_HIP;
    }
    if (x) {
        const uint64_t work = (d + 3) / 4;
        // one quad per thread: measured 15 % faster here than a grid-stride loop over fewer blocks
        const uint32_t blocks = (uint32_t)std::min<uint64_t>((work + 255) / 256, 1ull << 22);
        hipLaunchKernelGGL(k_server_step, dim3(blocks), dim3(256), 0, s, a, x, gamma, vec_ok ? 1u : 0u);
        if (hipGetLastError() != hipSuccess) return KIMAD_ERR_HIP;
    }
    return KIMAD_OK;
}

int kimad_error_at(kimad_plan_t* p, const uint64_t* K, double* err_out, void* stream) {
    if (!p || !K || !err_out) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Layout& lo = p->lo;
    mark(p, s, "begin");
    uint32_t* ksel = at<uint32_t>(p, lo.ksel);
    KLAUNCH(p, s, "k_make_ksel", k_make_ksel, dim3((lo.L + 255) / 256), dim3(256), K, (const LayerDesc*)p->pb.layers, lo.L, ksel);
    hipStream_t ss = s;
    int rc = launch_small_profile(p, err_out, s, &ss, ksel, 1u);
    if (!rc) rc = run_select_passes(p, ksel, 1, err_out, s, 0u);   // overwrites the grid profile's cache (k_lookup sees it as gone)
    const int rj = join_side(p, s, ss);
    return rc ? rc : rj;
}

int kimad_uniform_sizes(const uint64_t* n, uint32_t L, uint64_t budget_bytes, uint32_t pair_bytes, uint64_t* K_out,
                        uint64_t* pairs_out) {
    if (!n || !K_out || L == 0) return KIMAD_ERR_INVALID_ARG;
    if (pair_bytes == 0) pair_bytes = 8;
    uint64_t d = 0;
    for (uint32_t i = 0; i < L; ++i) {
        if (n[i] == 0 || n[i] > KIMAD_MAX_N) return KIMAD_ERR_INVALID_ARG;
        d += n[i];
    }
    const uint64_t P = budget_bytes / pair_bytes;
    const double rho = std::min(1.0, (double)P / (double)d);
    for (uint32_t i = 0; i < L; ++i) K_out[i] = rho > 0.0 ? grid_size_K(rho, n[i]) : 0;
    if (pairs_out) *pairs_out = std::min(P, d);
    return KIMAD_OK;
}

int kimad_payload_layer_counts(const uint32_t* idx, uint64_t pairs, const uint64_t* layer_start, uint32_t L,
                               uint64_t* counts_out, void* stream) {
    if (!idx || !layer_start || !counts_out || L == 0) return KIMAD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(k_layer_counts, dim3((L + 255) / 256), dim3(256), 0, s, idx, pairs, layer_start, L, counts_out);
    return hipGetLastError() == hipSuccess ? KIMAD_OK : KIMAD_ERR_HIP;
}

int kimad_selftest_wave_primitives(const uint32_t* in_u32, const double* in_f64, uint32_t* out_u32, double* out_f64,
                                   void* stream) {
    if (!in_u32 || !in_f64 || !out_u32 || !out_f64) return KIMAD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_selftest_wave, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), in_u32, in_f64, out_u32,
                       out_f64);
    return hipGetLastError() == hipSuccess ? KIMAD_OK : KIMAD_ERR_HIP;
}

uint64_t kimad_budget_bytes(double bandwidth_bits_per_s, double t_seconds, double t_comp_seconds, double alpha,
                            uint64_t cap_bytes) {
    const double B = bandwidth_bits_per_s, t = t_seconds, tc = t_comp_seconds;
    if (!(B > 0.0) || !(t > tc) || !(alpha >= 0.0) || std::isinf(B) || std::isinf(t)) return 0;
    const double c_bits = B * (t - tc) / (1.0 + alpha);
    const double bytes = std::floor(c_bits / 8.0);
    uint64_t out = bytes >= 18446744073709551615.0 ? ~0ull : (uint64_t)bytes;
    if (cap_bytes && out > cap_bytes) out = cap_bytes;
    return out;
}

const char* kimad_strerror(int status) {
    switch (status) {
        case KIMAD_OK: return "ok";
        case KIMAD_ERR_INVALID_ARG: return "invalid argument";
        case KIMAD_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case KIMAD_ERR_HIP: return "HIP runtime error";
        case KIMAD_ERR_INFEASIBLE: return "budget below the cheapest allocation";
        case KIMAD_ERR_NONFINITE: return "error table holds a non-finite entry";
        case KIMAD_ERR_OFFGRID: return "K is not one of the layer's grid sizes";
        case KIMAD_ERR_INTERNAL: return "internal error: candidate region overflow";
        case KIMAD_ERR_BAD_OFFSETS: return "K/offsets do not fit the payload capacity";
        case KIMAD_ERR_STALE_PROFILE: return "KIMAD_REUSE_PROFILE without a profile of the current g - h";
        case KIMAD_ERR_BAD_PAYLOAD: return "payload offsets or indices do not fit the layers";
        case KIMAD_ERR_TABLES_TOO_LARGE: return "exact cost axis without a budget limit: the allocation's tables would exceed 4 GiB";
        case KIMAD_ERR_STATIC_LIMIT: return "too many layers or cost cells for the fixed tables of kimad_allocate_static";
        default: return "unknown status";
    }
}

const char* kimad_version(void) { return "kimad-gfx950 0.1"; }

}  // extern "C"
