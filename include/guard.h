/*
 * guard.h -- C ABI of the online straggler detector's hot path on one MI355X.
 *
 * The library scores a dense telemetry tensor x[step][metric][rank] (fp32, rank
 * innermost) the way the paper's online monitor decides (Section 4.2, "Online
 * Monitoring Strategy"; nodes of 8 GPUs, Section 7.1):
 *
 *   gd_score_batch    every metric is judged relative to the peers of the same
 *                     job: per (step, metric) median and MAD over the ranks,
 *                     robust z, exceedance, the multi-signal rule with training
 *                     step time as the primary signal, and the 8-GPU node score;
 *   gd_update_window  a deviation only counts when it is sustained over
 *                     consecutive evaluations: k-of-W persistence per rank and
 *                     per node, kept as a ring of anomaly bits in device memory;
 *   gd_flags          the current fail-slow flags and counters;
 *   gd_topk_nodes     the k slowest nodes, ranked for the operator.
 *
 * Around that path: gd_severity (how much a flagged node slows the job: the tiered
 * response of Section 4.2), gd_sweep_score (scoring of single-node sweep results,
 * Section 5), and the ledger calls (persistence kept per indicator, ranking by the
 * score averaged over the window, recurrence of flag episodes as in Section 7).
 *
 * The paper states the decision in words only.  The estimators and constants
 * used here (median / MAD x 1.4826 / threshold 3.5 / k-of-W / scaled node sum)
 * are the defaults written into gd_config below.
 *
 * Conventions
 *   - Every pointer whose name starts with d_ is DEVICE memory owned by the
 *     caller (for instance a torch tensor).  The library never allocates, frees
 *     or keeps device memory, apart from remembering the state pointer given to
 *     gd_bind_state, which stays caller-owned and must outlive its use.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and is asynchronous: outputs are valid once the
 *     caller has synchronised that stream.  No call synchronises the device.
 *   - Arguments are validated on the host before anything is launched; a call
 *     that returns an error has launched nothing.  No exception crosses the ABI.
 *   - A NaN in the telemetry is a sample that did not arrive (see gd_score_batch).
 *     Infinities are unsupported input: the results of a column that holds one
 *     are unspecified.
 *   - A handle is not thread safe.  gd_score_batch is stateless; only
 *     gd_update_window writes the bound state; gd_flags / gd_topk_nodes /
 *     gd_severity read it; only gd_update_ledger writes the bound ledger.
 *   - The state is position independent: a byte copy of it, together with the
 *     number of steps consumed, is a checkpoint.
 */
#ifndef GUARD_H_
#define GUARD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gd_handle_s* gd_handle; /* host object; owns no device memory */

typedef enum {
    GD_OK = 0,
    GD_ERR_INVALID_ARG = 1,      /* NULL where a pointer is required, bad sizes          */
    GD_ERR_BAD_CONFIG = 2,       /* gd_config fails validation                           */
    GD_ERR_BUFFER_TOO_SMALL = 3, /* state buffer smaller than gd_state_bytes             */
    GD_ERR_UNSUPPORTED = 4,      /* valid but not built (e.g. gpus_per_node != 8)        */
    GD_ERR_HIP = 5               /* a HIP call failed; see gd_last_error                 */
} gd_status;

typedef enum { GD_NODE_SUM_SCALED = 0, GD_NODE_MAX = 1 } gd_node_agg;

#define GD_MAX_METRICS 8
#define GD_MAX_RANKS 65536
#define GD_MAX_WINDOW 1024

typedef struct gd_config {
    uint32_t struct_size;    /* = sizeof(gd_config)                                      */
    uint32_t n_ranks;        /* R: 8..65536, multiple of gpus_per_node                   */
    uint32_t gpus_per_node;  /* G: 8 (the node size of Section 7.1)                      */
    uint32_t n_metrics;      /* M: 1..8; metric m is bit m of every mask byte            */
    uint32_t primary_metric; /* the metric that must exceed (step time): default 0       */
    uint32_t min_signals;    /* metrics that must exceed together: default min(2, M)     */
    uint32_t window;         /* W: 1..1024 evaluations                                   */
    uint32_t persist_k;      /* k: 1..W anomalous evaluations inside the window          */
    uint32_t topk;           /* default k of gd_topk_nodes: min(64, N)                   */
    uint32_t node_agg;       /* gd_node_agg; default GD_NODE_SUM_SCALED                  */
    float z_threshold;       /* default 3.5; a score exceeds when it is strictly greater */
    float node_scale;        /* default 1/sqrt(G) = 0.35355338f; 1/G gives the mean      */
    float rel_floor;         /* default 1e-6 : scale >= rel_floor * |median|             */
    float abs_floor;         /* default 1e-30: scale >= abs_floor                        */
    int8_t direction[GD_MAX_METRICS]; /* +1 higher is worse, -1 lower is worse, 0 both   */
} gd_config;

/* Fill *cfg with the defaults above for the given shape (directions all +1). */
void gd_default_config(gd_config* cfg, uint32_t n_ranks, uint32_t n_metrics, uint32_t window,
                       uint32_t persist_k);

/* Validate *cfg and make a handle.  GD_ERR_BAD_CONFIG / GD_ERR_UNSUPPORTED on a
 * bad or unsupported configuration (then *out is NULL and gd_last_error(NULL)
 * describes the reason). */
gd_status gd_create(const gd_config* cfg, gd_handle* out);
gd_status gd_destroy(gd_handle h);

/* Bytes of window state for this configuration.  The caller allocates that many
 * bytes of device memory (256-byte aligned), fills them with zeros -- an
 * all-zero state is a fresh, empty window -- and binds them. */
size_t gd_state_bytes(gd_handle h);
gd_status gd_bind_state(gd_handle h, void* d_state, size_t state_bytes);

/*
 * Tuning of gd_score_batch for short batches (the streaming case of Section 4.2's
 * continuous monitoring: one evaluation per call).  A batch of at most max_steps
 * steps whose columns fit the chip side by side is scored with one workgroup per
 * (step, metric) column instead of one per run of steps; the results are the same
 * bit for bit, only the latency of a call differs.  0 switches this off.  The
 * default is GD_DEFAULT_STREAMING_STEPS.
 */
#define GD_DEFAULT_STREAMING_STEPS 4u
gd_status gd_set_streaming_steps(gd_handle h, uint32_t max_steps);

/*
 * (A tuning call, like the one above: no part of the paper's method and without
 * influence on any result.)
 * Where one-step calls of gd_score_batch may start looking: d_med and d_mad are device
 * arrays [n_metrics] holding the medians and MADs of a recent step -- normally the
 * previous call's own d_med and d_mad outputs, which may be the very buffers the next
 * call writes (each column reads its hint before it writes its result).  Telemetry
 * moves little from one step to the next, so the selection then starts from a narrow
 * bracket around the old median instead of sampling the column.  The arrays are read
 * by later gd_score_batch calls with T == 1 and must stay valid until replaced; NULL,
 * NULL switches the hints off.  Results never depend on the hints: a hint is only
 * trusted as far as the counting pass confirms it, so stale, wrong or uninitialised
 * contents cost time, not correctness.
 */
gd_status gd_set_streaming_hints(gd_handle h, const float* d_med, const float* d_mad);

/*
 * Score T steps (Section 4.2: peer-relative evaluation, multi-signal rule with
 * step time primary; Section 7.1: 8-GPU nodes).  With N = R/8, RW = ceil(R/64),
 * NW = ceil(N/64):
 *
 *   d_x            in   [T][M][R] f32
 *   d_med, d_mad   out  [T][M]    f32   median over ranks; median of |x - med|
 *   d_z            out  [T][M][R] f32   (x - med)/s, s = max(1.4826f*mad,
 *                                       rel_floor*|med|, abs_floor); may be NULL
 *   d_exceed_mask  out  [T][R]    u8    bit m: direction[m]*z > z_threshold
 *   d_rank_anom    out  [T][RW]   u64   bit r%64 of word r/64: primary bit set and
 *                                       popcount(mask) >= min_signals
 *   d_node_z       out  [T][N]    f32   node score of the primary metric:
 *                                       node_scale*(((z0+z1)+(z2+z3))+((z4+z5)+(z6+z7)))
 *                                       over the node's signed scores (or their max,
 *                                       a zero maximum reported as +0)
 *   d_node_mask    out  [T][N]    u8    bit m: node score of metric m > z_threshold
 *   d_node_anom    out  [T][NW]   u64   multi-signal rule applied to d_node_mask
 *
 * All arithmetic is IEEE fp32, one rounding per operation, -0 read as +0.
 * T == 0 is a valid no-op.  Every output except d_z is required.
 *
 * Missing samples: a NaN in d_x is a sample that did not arrive (polled telemetry
 * does not always answer, Section 7.1).  It is left out of its column's median and
 * MAD, which are taken over the samples present (the middle one of an odd number);
 * its z is 0, it never exceeds and it adds 0 to its node's score.  A column with
 * no sample present reports med = MAD = NaN and no exceedance.  Infinities remain
 * unsupported input (that column's results are unspecified).
 */
gd_status gd_score_batch(gd_handle h, const float* d_x, uint32_t T, float* d_med, float* d_mad,
                         float* d_z, uint8_t* d_exceed_mask, uint64_t* d_rank_anom,
                         float* d_node_z, uint8_t* d_node_mask, uint64_t* d_node_anom,
                         void* stream);

/*
 * Append T evaluations to the persistence windows of the bound state (Section
 * 4.2: only a deviation that lasts over successive evaluations counts; k of the
 * last W is this library's reading, the paper names no window).  For every rank
 * and node, at every appended step t = first_step_index .. first_step_index+T-1:
 * count = anomalous steps among the last W steps ending at t; the item is
 * flagged while count >= persist_k; the first flagged step is remembered.
 *
 *   d_rank_anom  in  [T][RW] u64, d_node_anom in [T][NW] u64  (from gd_score_batch)
 *   d_node_z     in  [T][N] f32; row T-1 becomes the "latest node score" used for
 *                ranking
 *   first_step_index  global index of the first appended step; calls must append
 *                consecutive steps starting from 0 on a zeroed state
 *                (first_step_index + T <= 2^31 - 1)
 */
gd_status gd_update_window(gd_handle h, const uint64_t* d_rank_anom, const uint64_t* d_node_anom,
                           const float* d_node_z, uint32_t T, uint64_t first_step_index,
                           void* stream);

/*
 * Read the current decision out of the state (Section 4.2: a node whose deviation has
 * lasted is flagged as fail-slow; the paper acts on nodes, Section 7.1, so a node also
 * reports whether one of its 8 GPUs is flagged).  Flags are instantaneous; the first
 * flagged step is kept besides (the paper is silent on a flag's lifetime).
 *   d_rank_flag  [R] u8   1 while count >= persist_k
 *   d_rank_count [R] u16  anomalous steps inside the current window
 *   d_rank_first [R] i32  first step at which the rank was flagged, -1 = never
 *   d_node_flag  [N] u8   bit 0: the node's own persistence flag;
 *                         bit 1: at least one of its 8 ranks is flagged
 *   d_node_count [N] u16, d_node_first [N] i32: as for ranks
 * Any of the six pointers may be NULL to skip that output.
 */
gd_status gd_flags(gd_handle h, uint8_t* d_rank_flag, uint16_t* d_rank_count,
                   int32_t* d_rank_first, uint8_t* d_node_flag, uint16_t* d_node_count,
                   int32_t* d_node_first, void* stream);

/*
 * The k slowest nodes.  The paper ranks nothing (a flagged node is simply handed to
 * mitigation, Section 4.2); the order is this library's: all N nodes ordered by (window count, high first; latest
 * primary node score, high first, -0 == +0; node index, low first).
 *   d_idx [k] i32  node indices in that order
 *   d_key [k] u64  count << 48 | order_key(score) << 16 | (0xFFFF - index), where
 *                  order_key maps fp32 to u32 preserving order; may be NULL
 * k == 0 selects the configured default; k > N is GD_ERR_INVALID_ARG.
 */
gd_status gd_topk_nodes(gd_handle h, uint32_t k, int32_t* d_idx, uint64_t* d_key, void* stream);

/*
 * Elastic membership (the paper is silent on ranks that join or leave a job; this is
 * the missing-sample rule of gd_score_batch applied to whole ranks): marks the ranks that take no part in a step as missing samples
 * of that step, in place, before gd_score_batch sees the batch.
 *   d_x      in/out [T][M][R] f32 device, 16-byte aligned
 *   d_active in     [T][ceil(R/64)] u64 device: bit r%64 of word r/64 set = rank r takes
 *                   part in step t
 * Where a bit is clear, x[t][m][r] becomes the quiet NaN 0x7FC00000 for every metric m
 * (a missing sample: see gd_score_batch); nothing else is written.  T == 0 is a no-op;
 * T above 65 535 per call is GD_ERR_INVALID_ARG.
 */
gd_status gd_apply_membership(gd_handle h, float* d_x, uint32_t T, const uint64_t* d_active, void* stream);

/*
 * Severity of the performance impact of the flagged nodes (Section 4.2, the
 * tiered response: no observable impact / a moderate, sustained slowdown of
 * about 10% / severe degradation of 20% or more).  Call after gd_update_window
 * has consumed the same T steps: a node counts as flagged when its own window
 * count or that of one of its 8 ranks has reached persist_k.  For a flagged node,
 * each of its 8 primary-metric samples of the last min(T, window) steps of d_x is
 * divided by that step's median d_med[t][primary] (the other way round when the
 * primary metric is lower-is-worse; whichever quotient is >= 1 when it is
 * two-sided; -0 reads as +0); the slowdown is the median of these quotients (the
 * two middle ones added, then halved) minus 1, every operation rounded to fp32.
 *   d_x   [T][M][R] device, the batch gd_score_batch scored
 *   d_med [T][M]    device, the medians it wrote
 *   d_node_slowdown [N] f32 device: the slowdown, 0 for a node that is not flagged
 *   d_node_tier     [N] u8  device: 0 not flagged; 1 slowdown < moderate;
 *                            2 moderate <= slowdown < severe; 3 slowdown >= severe
 * moderate > severe is GD_ERR_INVALID_ARG.  T == 0 reports tier 0 everywhere.
 * Missing samples (NaN) and steps whose median is NaN are left out of the quotients;
 * a flagged node with none left reports slowdown 0 in tier 1.  Zero medians or
 * samples and infinities give an unspecified slowdown for that node.
 */
gd_status gd_severity(gd_handle h, const float* d_x, uint32_t T, const float* d_med, float moderate,
                      float severe, float* d_node_slowdown, uint8_t* d_node_tier, void* stream);

/*
 * Scoring of single-node sweep results (Section 5, "Single-Node Sweep": sustained
 * throughput consistent across the GPUs of a node; pairwise intra-node bandwidth
 * connected and symmetric), for n_nodes nodes of 8 GPUs at once.  Independent of
 * the handle's configuration and state.
 *   d_flops [n_nodes][8]    f32 in   sustained throughput of each GPU
 *   d_bw    [n_nodes][8][8] f32 in   bandwidth from GPU i to GPU j; the diagonal is ignored
 *   d_gpu_shortfall [n_nodes][8] f32 out  (m8 - flops_g) / m8, m8 = median of the node's 8
 *                                         throughputs (the two middle ones added, then halved)
 *   d_gpu_mask  [n_nodes] u8  out  bit g: shortfall_g > tol_compute
 *   d_link_mask [n_nodes] u32 out  bit p for the pair i < j numbered row by row ((0,1), (0,2),
 *                                  ..., (6,7) = 27): with hi / lo the larger / smaller of
 *                                  bw[i][j] and bw[j][i] and m56 the median of the 56
 *                                  off-diagonal entries, (hi - lo) / hi > tol_sym or
 *                                  (m56 - lo) / m56 > tol_bw
 *   d_verdict   [n_nodes] u8  out  bit 0: some GPU bit set; bit 1: some link bit set
 * Every operation is rounded to fp32.  Non-finite or non-positive inputs give
 * unspecified results for that node (no fault).  n_nodes == 0 is a no-op.
 */
gd_status gd_sweep_score(gd_handle h, const float* d_flops, const float* d_bw, uint32_t n_nodes,
                         float tol_compute, float tol_sym, float tol_bw, float* d_gpu_shortfall,
                         uint8_t* d_gpu_mask, uint32_t* d_link_mask, uint8_t* d_verdict, void* stream);

/*
 * The ledger: bookkeeping beyond the default rule, in a buffer of its own.
 *
 *  - Persistence per indicator, the other reading of Section 4.2's rule that several
 *    indicators must deviate and keep deviating over successive evaluations:
 *    each metric keeps its own count of exceeding steps among the last `window`, a
 *    metric is sustained when that count has reached persist_k, and an item (a rank
 *    or a node) is flagged when the primary metric is sustained and at least
 *    min_signals metrics are.  (The default rule combines the metrics of each step
 *    first and persists the result.)
 *  - The primary node score summed over the window in integers,
 *    q = clamp(round-half-even(node_z * score_quant), -32768, 32767), NaN -> 0, for a
 *    ranking by the score averaged over the window rather than the latest one.
 *  - Recurrence (Section 7: a node sent to triage three times within a week is
 *    taken to be terminally bad): an episode starts at a step where the node's
 *    default-rule flag (its combined anomaly bit, k of W) rises; a node is terminal
 *    from the first step at which recur_limit episodes began within the last
 *    recur_horizon steps.
 */
typedef struct gd_ledger_config {
    uint32_t struct_size;    /* = sizeof(gd_ledger_config)                                   */
    float    score_quant;    /* finite, > 0; 64 keeps 1/64 of a score unit, range -512..512  */
    uint32_t recur_limit;    /* 1..8; the paper's clusters used 3                            */
    uint32_t reserved;       /* 0                                                            */
    uint64_t recur_horizon;  /* steps, >= 1: "a week" in evaluation steps                    */
} gd_ledger_config;

/* Fills c with score_quant 64, recur_limit 3, recur_horizon 604800 (a week of one-second steps). */
void gd_default_ledger_config(gd_ledger_config* c);

/* Bytes of the ledger for batches of at most max_T steps (0 for a null handle). */
size_t gd_ledger_bytes(gd_handle h, uint32_t max_T);

/*
 * Binds a caller-owned, 256-byte aligned device buffer of at least
 * gd_ledger_bytes(h, max_T) bytes.  All zero bytes are a fresh ledger; the bytes
 * are position-independent (a checkpoint is a copy).  The handle keeps cfg by value.
 */
gd_status gd_bind_ledger(gd_handle h, const gd_ledger_config* cfg, void* d_ledger, size_t bytes,
                         uint32_t max_T);

/*
 * Takes the T steps gd_score_batch just scored into the ledger.
 *   d_exceed_mask [T][R] u8 (4-byte aligned), d_node_mask [T][N] u8, d_node_z [T][N] f32:
 *                     its outputs, read only
 *   first_step_index: index of the batch's first step; batches must arrive in order
 *                     (each starting where the one before ended) and first_step_index + T
 *                     must stay below 2^31
 * Two kernels are enqueued on the stream; part of the ledger buffer serves as their work
 * area, so two calls on one ledger must not overlap.
 * T == 0 is GD_OK and does nothing; T > max_T is GD_ERR_INVALID_ARG.  Independent of
 * gd_update_window: either may be called without the other, in any order.
 */
gd_status gd_update_ledger(gd_handle h, const uint8_t* d_exceed_mask, const uint8_t* d_node_mask,
                           const float* d_node_z, uint32_t T, uint64_t first_step_index,
                           void* stream);

/*
 * gd_update_ledger for callers that cannot allocate device memory or hand over a work
 * area: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same results in the ledger, same two kernels; their work
 * area (the episode-start map and the staged counts) is a static device array inside
 * the library, gd_ledger_static_scratch_bytes() = 8 MiB per GPU, held from the first
 * call on that GPU until the process ends.  The call itself allocates nothing, here or
 * in any library it uses.  The ledger may therefore be bound with max_T = 1; T is
 * limited by the array instead: align256(T * ceil(N/64) * 8) + 16 R + 18 N (rounded up
 * to 256 per term) must not exceed it (T <= 7 024 at 65 536 ranks), else
 * GD_ERR_INVALID_ARG and nothing is launched.
 * Every call on one GPU, from any handle, shares that GPU's array: calls that could
 * overlap there (different streams, different threads) race; calls on one stream do
 * not.  Nothing in the array has to be cleared between calls.
 */
size_t gd_ledger_static_scratch_bytes(void);
gd_status gd_update_ledger_static(gd_handle h, const uint8_t* d_exceed_mask, const uint8_t* d_node_mask,
                                  const float* d_node_z, uint32_t T, uint64_t first_step_index,
                                  void* stream);

/*
 * Reads the ledger as of the last step taken in.  Every output is device memory
 * and may be NULL.
 *   d_rank_pmask [R] u8   bit m: metric m is sustained for the rank
 *   d_rank_pflag [R] u8   1 when the per-indicator rule flags the rank now
 *   d_rank_pfirst [R] i32 first step at which it did, -1 = never
 *   d_node_pmask, d_node_pflag, d_node_pfirst [N]: the same for nodes
 *   d_node_score_sum [N] i32  sum of q over the last min(steps so far, window) steps
 *   d_node_episodes [N] u8    episodes begun within the last recur_horizon steps,
 *                             saturating at recur_limit
 *   d_node_terminal_first [N] i32  first step at which the node was terminal, -1 = never
 */
gd_status gd_ledger_flags(gd_handle h, uint8_t* d_rank_pmask, uint8_t* d_rank_pflag,
                          int32_t* d_rank_pfirst, uint8_t* d_node_pmask, uint8_t* d_node_pflag,
                          int32_t* d_node_pfirst, int32_t* d_node_score_sum,
                          uint8_t* d_node_episodes, int32_t* d_node_terminal_first, void* stream);

/*
 * The k slowest nodes by (window count of the default rule as the ledger keeps it,
 * high first; windowed score sum, high first; node index, low first).
 *   d_idx [k] i32; d_key [k] u64 = count << 48 | (sum + 2^31) << 16 | (0xFFFF - index), or NULL
 * k == 0 selects the configured default; k > N is GD_ERR_INVALID_ARG.
 */
gd_status gd_topk_nodes_mean(gd_handle h, uint32_t k, int32_t* d_idx, uint64_t* d_key, void* stream);

/*
 * NOT part of the detector's contract -- a diagnostic for benchmarks, exported so that
 * the benchmark can time it through the same library: reads the first n_bytes (rounded down to a multiple of
 * 256 KiB) of d_x with the scoring kernel's own load pattern and does nothing else,
 * so that its duration next to gd_score_batch's gives the ceiling of a single pass
 * over the data on this chip.  d_x 16-byte aligned device memory; d_sink one u32 of
 * device memory that the call may write.
 */
gd_status gd_probe_read(gd_handle h, const float* d_x, uint64_t n_bytes, uint32_t* d_sink,
                        void* stream);

/* Text of the last error on this handle (or of the last failed gd_create when
 * h is NULL).  The pointer stays valid until the next call on the handle. */
const char* gd_last_error(gd_handle h);

#ifdef __cplusplus
}
#endif
#endif /* GUARD_H_ */
