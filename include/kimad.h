/*
 * kimad.h - C ABI of the MI355X (gfx950) library for one worker's Kimad+ compression step.
 *
 * The calls follow the worker side of the Kimad algorithm (paper Algorithm 1, lines
 * "Select compressor" and "Upload the compressed vector"), split at its natural seams:
 *
 *   kimad_profile      layer-wise compression-error table over a grid of candidate ratios
 *                      (Section 3.2, Eq. norm decomposition; the Errors matrix of Appendix C)
 *   kimad_allocate     budget-constrained choice of one grid point per layer
 *                      (Section 3.2, Eq. optimisation; the dynamic programme of Appendix C)
 *   kimad_compress_ef  per-layer TopK of x = g - h, sparse (index, value) payload, and the
 *                      estimator update h <- h + TopK(g - h)
 *                      (Section 2.2 TopK; Section 3.3 Eq. EF21-2; Algorithm 1 upload line)
 *
 * Notation: g = fresh update u (the gradient), h = estimator u_hat (error-feedback state),
 * x = g - h.  "Layer" = one parameter tensor.  Magnitudes are compared on the binary32 bit
 * pattern of x with the sign cleared; equal magnitudes keep the lower index first.
 *
 * Conventions
 *   - Every pointer is marked HOST or DEVICE.  The library never allocates or frees device
 *     memory: gradients, estimator, outputs and the workspace belong to the caller.
 *   - All GPU work is ordered with the given stream (a hipStream_t passed as void*; NULL is the
 *     default stream): it is enqueued there, except that kernels for layers of at most 8192
 *     entries run on a side stream of the plan between a fork and a join event on the given
 *     stream.  No call waits for the device except kimad_plan_create (synchronous uploads) and
 *     the diagnostics getters.  kimad_profile, kimad_allocate, kimad_compress_ef, kimad_step and
 *     kimad_server_apply may be recorded into a HIP graph by stream capture (per-kernel timing off): tables
 *     are cleared by kernels, and the recording holds the pointers and the budget of the recorded call.
 *   - Return value: 0 on success, a negative kimad_status otherwise (argument errors are found
 *     on the host before anything is enqueued).  Data-dependent outcomes (infeasible budget,
 *     non-finite table, a K that is not on the grid) are written to a DEVICE status word.
 *   - One plan must not be used from two streams at once: its workspace is shared state.
 */
#ifndef KIMAD_H
#define KIMAD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KIMAD_MAX_J 64u                 /* candidate ratios per layer */
#define KIMAD_MAX_N 0xFFF00000ull       /* elements per layer (indices are u32) */

typedef enum kimad_status {
    KIMAD_OK = 0,
    KIMAD_ERR_INVALID_ARG = -1,
    KIMAD_ERR_WORKSPACE_TOO_SMALL = -2,
    KIMAD_ERR_HIP = -4,
    KIMAD_ERR_INFEASIBLE = -6,          /* device status: budget below the cheapest allocation */
    KIMAD_ERR_NONFINITE = -7,           /* device status: error table holds Inf or NaN */
    KIMAD_ERR_OFFGRID = -8,             /* device status: KIMAD_REUSE_PROFILE given but K is not a grid size */
    KIMAD_ERR_INTERNAL = -9,            /* device status: an internal capacity bound was violated (a bug) */
    KIMAD_ERR_BAD_OFFSETS = -10,        /* device status: offsets/K do not fit capacity_pairs */
    KIMAD_ERR_STATIC_LIMIT = -11,       /* kimad_allocate_static: more layers or longer rows than its fixed tables hold */
    KIMAD_ERR_STALE_PROFILE = -12,      /* device status: KIMAD_REUSE_PROFILE, but no kimad_profile has run on this plan
                                           since the last kimad_compress_ef (which changed h) */
    KIMAD_ERR_BAD_PAYLOAD = -13,        /* device status of kimad_server_apply: offsets or indices do not fit the layers */
    KIMAD_ERR_TABLES_TOO_LARGE = -14    /* cost_units_D == 0 without a max_budget_bytes that keeps the allocation's
                                           tables (L rows of one byte per pair of the budget) within 4 GiB */
} kimad_status;

/* One layer: DEVICE pointers to n fp32 values each.  g is read-only; h is updated in place by
 * kimad_compress_ef only.  4-byte alignment suffices (16-byte alignment of both is fastest). */
typedef struct kimad_layer {
    const float* g;
    float* h;
    uint64_t n;                         /* 1 .. KIMAD_MAX_N */
} kimad_layer_t;

typedef struct kimad_config {
    uint32_t pair_bytes;                /* bytes charged per kept entry; 0 means 8 (u32 index + fp32 value) */
    uint32_t cost_units_D;              /* Appendix C discretisation factor D applied to the budget; 0 = exact
                                           (one cost cell per pair: set max_budget_bytes, see there) */
    uint64_t max_budget_bytes;          /* largest budget kimad_allocate will see; 0 = uncompressed size.
                                           Sizes the DP tables when cost_units_D == 0: the workspace then grows
                                           by L * max_budget_bytes / pair_bytes bytes, and a plan whose tables
                                           would pass 4 GiB is refused with KIMAD_ERR_TABLES_TOO_LARGE (the
                                           default of 0 does that for models beyond a few million elements:
                                           give the budget limit, or a factor such as the paper's 1000). */
    uint64_t flags;                     /* KIMAD_CFG_* */
    uint32_t max_workgroups;            /* workgroups (= compute units) the streaming pass of the profile may
                                           occupy; 0 = all of the device.  A smaller number leaves units to
                                           other work on the device and changes no result. */
    uint32_t value_format;              /* KIMAD_VALUES_F32 (0) or KIMAD_VALUES_F16: how kept values travel */
} kimad_config_t;

/* Payload values.  F32: the fp32 value x itself.  F16 (Section 2.2 names quantisation beside sparsification):
 * binary16, round to nearest even, saturated to +-65504, NaN kept; pair_bytes then defaults to 6, val_out holds
 * uint16 bit patterns, and worker and server both add the decoded value, h[idx] = fl32(h[idx] + fl32(q16(x))):
 * the two estimator copies stay equal and what the rounding lost stays in g - h for the next round.  The error
 * table remains that of TopK (the rounding of kept values, below 2^-22 of their energy, is not charged). */
#define KIMAD_VALUES_F32 0u
#define KIMAD_VALUES_F16 1u

#define KIMAD_CFG_CLASSIC_PROFILE 1ull  /* profile with two full passes over g, h instead of the sampled
                                           single pass (same results; for comparison and testing) */

#define KIMAD_CFG_SAMPLE_ALWAYS 16ull    /* profile: predict every call from a fresh sampling pass over 1/16 of g, h.  By
                                           default only a plan's first profile samples; later ones predict from the
                                           exact histogram the previous one left (gradients of successive rounds are
                                           distributed alike), which saves the sampling pass.  No result depends on
                                           the prediction: a layer it misses is recounted by a full pass. */
#define KIMAD_CFG_FULL_DP 2ull          /* allocation: always run the recurrence over whole rows of cost cells */
#define KIMAD_CFG_BAND_DP 4ull          /* allocation: always run it inside the band of cells that Lagrangian bounds
                                           leave.  Same results either way; by default rows of 1537 cells or more
                                           take the band (its cost hardly grows with the row), shorter ones the
                                           whole rows.  Rows that do not fit LDS (more than 4224 cells) and plans
                                           of more than 1024 layers always take whole rows. */

#define KIMAD_CFG_DENSE_FALLBACK 8ull    /* allocation: a layer never costs more than its bare values (4 n bytes).  A grid
                                           point at or beyond the break-even K * pair_bytes >= 4 n stands for sending
                                           the layer whole: error 0, K_out = n, charged ceil(4 n / pair_bytes) pairs
                                           (the levelling off at the uncompressed size in Section 4.2).  offsets_out
                                           remain the exclusive scan of K_out: size the payload buffers for it. */

/* flags of kimad_compress_ef */
#define KIMAD_REUSE_PROFILE 1u          /* every K[i] is one of layer i's grid sizes and g, h are unchanged
                                           since the last kimad_profile on this plan: reuse its thresholds.
                                           The plan remembers on the device whether a profile is still current: a
                                           kimad_compress_ef ends that (it changes h), so a second call with this
                                           flag and no kimad_profile in between is refused through status_out
                                           (KIMAD_ERR_STALE_PROFILE) and writes nothing.  Changes of g or h by the
                                           caller are not seen. */

typedef struct kimad_plan kimad_plan_t; /* host object; owns no device memory */

/* Bytes of DEVICE workspace a plan over these layer sizes needs.  n: HOST array of L sizes.
 * About a quarter of the bytes of g and h for large models: candidate space for a sixth of every layer above
 * 8192 entries (8 bytes an entry), histogram tables, chunk records and the allocation's rows (see
 * kimad_config_t::max_budget_bytes for the latter). */
int kimad_workspace_bytes(const uint64_t* n, uint32_t L, uint32_t J,
                          const kimad_config_t* cfg, uint64_t* bytes_out);

/* Build a plan: validates arguments, computes the candidate sizes
 *   K_ij = min(n_i, max(1, ceil(ratios[j] * n_i)))          (Section 3.2, the discrete set)
 * and uploads layer descriptors and tile maps into the workspace.
 *   layers   HOST array of L descriptors (device pointers inside)
 *   ratios   HOST array of J values, strictly ascending, each in (0, 1]
 *   workspace DEVICE, 256-byte aligned, at least kimad_workspace_bytes() bytes; the plan keeps
 *            using it until kimad_plan_destroy.
 * The plan stays valid while the layers' pointers and sizes stay the same. */
int kimad_plan_create(const kimad_layer_t* layers, uint32_t L,
                      const double* ratios, uint32_t J,
                      const kimad_config_t* cfg,
                      void* workspace, uint64_t workspace_bytes,
                      void* stream, kimad_plan_t** plan_out);
int kimad_plan_destroy(kimad_plan_t* plan);

/* HOST copy of the plan's candidate sizes, L*J row-major (for callers that want K_ij). */
int kimad_plan_grid_sizes(const kimad_plan_t* plan, uint64_t* K_table_out);

/* Error profile (Section 3.2, Eq. norm decomposition):
 *   err_table[i*J + j] = || x_i - TopK_{K_ij}(x_i) ||^2  = sum of squares of the entries dropped,
 * fp64, DEVICE, L*J row-major.  Exactly 0 where K_ij = n_i.  Pure: g and h are not modified.
 * Also records, inside the workspace, each candidate's selection threshold and the layer's
 * largest entries (index, x) for KIMAD_REUSE_PROFILE.
 *   budget_hint_bytes  the budget the following kimad_allocate will get, or 0 if unknown.  It only
 *                      sizes how many of the largest entries are kept for the compression; no
 *                      result depends on it.
 * Every entry is certified to 4e-6 relative or recomputed exactly from a last-digit histogram; the
 * plan holds min(L_big * J, 65536) such histograms, and an entry that finds none left is NaN (which
 * kimad_allocate reports as KIMAD_ERR_NONFINITE) rather than a loosely bounded value. */
int kimad_profile(kimad_plan_t* plan, double* err_table, uint64_t budget_hint_bytes, void* stream);

/* Allocation (Section 3.2 Eq. optimisation; Appendix C): choose j_i minimising
 * sum_i err_table[i][j_i] subject to sum_i K_{i j_i} * pair_bytes <= budget_bytes.
 *   P = floor(budget_bytes / pair_bytes); unit = 1 if D == 0 or P <= D else ceil(P / D);
 *   capacity = floor(P / unit); cost w_ij = ceil(K_ij / unit).
 * Rows are indexed by cost 0..capacity; candidates are tried in ascending j with strict "<";
 * the answer ends at the smallest cost attaining the least total.
 *   err_table   DEVICE, L*J fp64 (any table, e.g. kimad_profile's output)
 *   j_out       DEVICE int32[L]      chosen grid index per layer
 *   K_out       DEVICE uint64[L]     chosen size per layer
 *   offsets_out DEVICE uint64[L+1]   exclusive scan of K_out
 *   status_out  DEVICE int32[1]      KIMAD_OK, KIMAD_ERR_INFEASIBLE or KIMAD_ERR_NONFINITE
 * On a non-zero status the other outputs are zero-filled. */
int kimad_allocate(kimad_plan_t* plan, const double* err_table, uint64_t budget_bytes,
                   int32_t* j_out, uint64_t* K_out, uint64_t* offsets_out,
                   int32_t* status_out, void* stream);

/* kimad_allocate for callers that cannot allocate device memory or hand over a workspace at the point of
 * the call: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels, same results as kimad_allocate, but the dynamic programme's tables live in a
 * fixed array inside the library (4 MiB per device, held until the process ends) instead of the plan's
 * workspace; nothing is allocated or freed, by HIP or otherwise.  The plan supplies sizes, configuration and
 * the candidate sizes K_ij only.  Limits: at most KIMAD_STATIC_MAX_L layers and rows of at most
 * KIMAD_STATIC_MAX_CELLS cost cells (capacity + 1; a cost_units_D of up to 1023 always fits): beyond them
 * the call returns KIMAD_ERR_STATIC_LIMIT and enqueues nothing.  Every call on a device shares that device's
 * array, whatever the plan: calls that overlap on one device race, also with each other across streams. */
#define KIMAD_STATIC_MAX_L 256u
#define KIMAD_STATIC_MAX_CELLS 1024u
int kimad_allocate_static(kimad_plan_t* plan, const double* err_table, uint64_t budget_bytes,
                          int32_t* j_out, uint64_t* K_out, uint64_t* offsets_out,
                          int32_t* status_out, void* stream);

/* TopK selection, payload and estimator update (Section 2.2; Algorithm 1 upload line;
 * Section 3.3 Eq. EF21-2).  For each layer i with x = g_i - h_i (fp32):
 *   S_i = the K[i] entries of largest magnitude, equal magnitudes by lower index;
 *   idx_out[offsets[i] + r] = r-th smallest index in S_i (layer-local), val_out[...] = x[idx];
 *   h_i[idx] = fl32(h_i[idx] + x[idx]) for idx in S_i, all other entries untouched.
 *   K        DEVICE uint64[L], each 0..n_i
 *   offsets  DEVICE uint64[L+1], offsets[i] + K[i] <= capacity_pairs for every i
 *   idx_out  DEVICE uint32[capacity_pairs];  val_out DEVICE float[capacity_pairs]
 *   flags    0 (select from scratch: two extra passes over g, h) or KIMAD_REUSE_PROFILE
 *   status_out DEVICE int32[1] */
int kimad_compress_ef(kimad_plan_t* plan, const uint64_t* K, const uint64_t* offsets,
                      uint32_t* idx_out, void* val_out /* float[], or uint16[] with KIMAD_VALUES_F16 */,
                      uint64_t capacity_pairs, uint32_t flags, int32_t* status_out, void* stream);

/* profile -> allocate -> compress_ef(KIMAD_REUSE_PROFILE) on one stream: one worker's step. */
int kimad_step(kimad_plan_t* plan, uint64_t budget_bytes, double* err_table,
               int32_t* j_out, uint64_t* K_out, uint64_t* offsets_out,
               uint32_t* idx_out, void* val_out, uint64_t capacity_pairs,
               int32_t* status_out /* DEVICE int32[2]: allocate, compress */, void* stream);

/* Error of TopK at any sizes (Section 3.2, Eq. norm decomposition): err_out[i] = || x_i - TopK_{K[i]}(x_i) ||^2 for
 * K[i] in 0..n_i (DEVICE uint64[L] in, DEVICE double[L] out), with the accuracy of kimad_profile.  Two passes over
 * g and h; g and h are not modified.  It overwrites the thresholds of an earlier kimad_profile (a following
 * KIMAD_REUSE_PROFILE is refused).  This is what prices an allocation that is not on the grid, e.g. the baselines
 * of the paper's Section 4.3 below. */
int kimad_error_at(kimad_plan_t* plan, const uint64_t* K, double* err_out, void* stream);

/* Baseline allocators of Section 4.3, HOST arithmetic: "Kimad" without the layer-wise allocation gives every layer
 * the ratio rho = min(1, P / d), P = floor(budget_bytes / pair_bytes): K_out[i] = min(n_i, max(1, ceil(rho n_i)))
 * (0 everywhere if P = 0).  *pairs_out (optional) = min(P, d), the size of the whole-model TopK of the same budget.
 * n, K_out: HOST arrays of L. */
int kimad_uniform_sizes(const uint64_t* n, uint32_t L, uint64_t budget_bytes, uint32_t pair_bytes, uint64_t* K_out,
                        uint64_t* pairs_out);

/* Per-layer attribution of a selection made over the whole model (Section 4.3, "the optimal baseline ... with the
 * whole model information"): idx = the `pairs` ascending positions kept in the flat buffer (the payload of a
 * one-layer plan over it), layer_start = DEVICE uint64[L+1] element offsets of the layers; counts_out[i] (DEVICE
 * uint64[L]) = positions inside layer i.  With kimad_error_at on the per-layer plan this gives every layer's share
 * of the whole-model error. */
int kimad_payload_layer_counts(const uint32_t* idx, uint64_t pairs, const uint64_t* layer_start, uint32_t L,
                               uint64_t* counts_out, void* stream);

/* DEVICE diagnostics of the last kimad_profile on the plan, copied to HOST (synchronises the
 * stream): out[0] = table entries whose error bound exceeded the certified tolerance before the
 * exact last-digit pass ran, out[1] = entries that pass recomputed, out[2] = histograms it used,
 * out[3] = layers whose sampled prediction missed and were recounted by a full pass. */
int kimad_profile_diagnostics(kimad_plan_t* plan, uint32_t* out4, void* stream);

/* DEVICE diagnostics of the last kimad_allocate on the plan (rows that fit LDS only), copied to HOST
 * (synchronises the stream): out[0] = widest band of cost cells the recurrence visited in a row, out[1] = sum of
 * the bands' widths over the rows, out[2] = 1 if the bands were the whole rows (no bound could be used),
 * out[3] = upgrades the upper bound's greedy fill took.  All zero before the first allocation. */
int kimad_allocate_diagnostics(kimad_plan_t* plan, uint32_t* out4, void* stream);

/* Per-layer state of the last profile / compression, for benchmarks and tests (synchronises the
 * stream).  For each layer larger than 8192 entries, 8 words are written to `out` (HOST):
 * layer index, spill bin (entries at or above this digit-1 bin were kept as candidates; 4096 = none),
 * slots fixed before the pass, slots filled from the candidates, redo flag, candidates kept,
 * candidates valid (0 if the layer's candidate space ran out during the pass), selection mode of the last
 * kimad_compress_ef (0 none, 1 g and h read again into the candidate space, 3 from the profile's candidates,
 * 4 straight from g and h: everything is kept, or what had to be looked at did not fit the candidate space). */
int kimad_plan_layer_states(kimad_plan_t* plan, uint32_t* out, uint32_t max_layers, uint32_t* count_out,
                            void* stream);

/* Server side of a round (paper Algorithm 1, server lines "Aggregate all update estimators" and
 * "Updates the model"): for every worker m = 0..M-1 decode its payload into the server's copy
 * of its estimator,
 *     u_hat_m[layer_start[i] + idx] = fl32(u_hat_m[...] + val)   for the pairs of layer i,
 * which is the very addition the worker applied to its own estimator, so the two copies stay
 * equal bit for bit; then, if x is not NULL, step the model:
 *     x[t] = fl32( (double)x[t] - gamma * sum_m (double)weights[m] * (double)u_hat_m[t] ),
 * the sum in fp64 in worker order (the paper fixes no precision; this is the reading taken).
 *   payloads     HOST array[M] of {idx, val, offsets}: DEVICE pointers to one worker's payload as
 *                written by kimad_compress_ef (layer-local ascending indices; offsets uint64[L+1])
 *   u_hat        HOST array[M] of DEVICE float[d] buffers (flat: layer i at layer_start[i]), updated
 *                in place; the M buffers and x must not overlap
 *   weights      HOST double[M]
 *   M            1..KIMAD_MAX_WORKERS
 *   layer_start  DEVICE uint64[L+1], element offsets of the layers, layer_start[L] = d
 *   d            elements per flat buffer (HOST value of layer_start[L])
 *   x            DEVICE float[d] or NULL (aggregate only)
 *   status_out   DEVICE int32[M]: per worker KIMAD_OK, or KIMAD_ERR_BAD_PAYLOAD if its offsets are not a
 *                non-decreasing sequence from 0 to at most capacity_pairs, or layer_start is not non-decreasing
 *                up to d (then none of that worker's pairs is applied), or if some pair's index lies outside
 *                its layer (that pair is skipped, the others applied).  Nothing is ever written out of bounds.
 * Nothing is allocated; all work is enqueued on `stream`.
 * Returns KIMAD_ERR_INVALID_ARG for null pointers or M out of range. */
#define KIMAD_MAX_WORKERS 16
typedef struct kimad_payload {
    const uint32_t* idx;      /* DEVICE */
    const float* val;         /* DEVICE */
    const uint64_t* offsets;  /* DEVICE uint64[L+1] */
    uint64_t capacity_pairs;  /* entries the idx and val buffers hold */
    uint32_t value_format;    /* KIMAD_VALUES_F32, or KIMAD_VALUES_F16: val holds uint16 bit patterns */
    uint32_t pad;             /* 0 */
} kimad_payload_t;
int kimad_server_apply(const kimad_payload_t* payloads, float* const* u_hat, const double* weights,
                       uint32_t M, const uint64_t* layer_start, uint32_t L, uint64_t d,
                       float* x, double gamma, int32_t* status_out, void* stream);

/* Per-kernel timing (tracing aid for benchmarks).  With timing enabled the library records a
 * HIP event on the stream after every kernel it launches.  kimad_plan_get_timings waits for the
 * last recorded event, then writes one entry per launch since the last call: the kernel names,
 * newline-separated, into `names` (HOST, names_bytes long) and the durations in milliseconds
 * into `ms` (HOST, max_entries floats); *count_out = entries written.  At most 1024 launches are
 * kept between two calls. */
int kimad_plan_set_timing(kimad_plan_t* plan, int enable);
int kimad_plan_get_timings(kimad_plan_t* plan, char* names, uint32_t names_bytes, float* ms,
                           uint32_t max_entries, uint32_t* count_out);

/* Self-test of the kernels' wave-level building blocks that are written with DPP operands (the 64-lane prefix sum
 * of the streaming pass, the row-broadcast address and accumulate steps of the allocation's recurrence, the
 * group maxima of its bounds and the pair minima of its banded recurrence): one wave runs each on the given
 * per-lane inputs and writes every lane's result, for a test to compare with host-computed values.  All
 * pointers DEVICE:
 *   in_u32 uint32[128], in_f64 double[128], out_u32 uint32[64 + 1024 + 256], out_f64 double[1024 + 192 + 256];
 *   out_u32[lane]                          = in_u32[0] + ... + in_u32[lane]
 *   out_u32[64 + (4 k + u) * 64 + lane]    = in_u32[lane] + in_u32[64 + 16 (lane / 16) + 4 k + u]      k, u = 0..3
 *   out_f64[(4 k + u) * 64 + lane]         = in_f64[lane] + in_f64[64 + 16 (lane / 16) + 4 k + u]
 *   out_f64[1024 + 64 t + lane]            = max of in_f64 over the lane's aligned group of 2, 4, 8 lanes (t = 0, 1, 2)
 *   out_f64[1216 + 64 t + lane]            = min of in_f64 over the lane's aligned group of 2, 4, 8, 16 lanes (t = 0..3)
 *   out_u32[1088 + 64 t + lane]            = the smallest in_u32[64 + l] & 255 among the lanes l of that group that hold
 *                                            this minimum (the pair minimum of the banded recurrence) */
int kimad_selftest_wave_primitives(const uint32_t* in_u32, const double* in_f64, uint32_t* out_u32, double* out_f64,
                                   void* stream);

/* Compression budget of one round (Section 3.1, Eq. budget): the bytes that fit into the up-link share
 * of the time budget t at the monitored bandwidth.  The paper's time split t = c/B + T_comp + alpha c/B
 * gives c = B (t - T_comp) / (1 + alpha) bits (alpha = 1: the printed B (t - T_comp) / 2); the result is
 * floor(c / 8), at most cap_bytes if that is not 0 (the uncompressed size).  HOST arithmetic in fp64, no
 * device work.  Returns 0 for t <= T_comp and for a bandwidth or alpha that is negative, zero (bandwidth)
 * or not finite. */
uint64_t kimad_budget_bytes(double bandwidth_bits_per_s, double t_seconds, double t_comp_seconds, double alpha,
                            uint64_t cap_bytes);

const char* kimad_strerror(int status);
const char* kimad_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KIMAD_H */
