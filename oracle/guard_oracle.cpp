// CPU oracle for the online straggler detector -- TEST INFRASTRUCTURE ONLY.
//
// This file is the plain, slow, obviously-correct statement of what the GPU
// library must compute.  Only the tests, the smoke check and the benchmark's
// CPU-baseline leg may call it; the product never does, and it shares no code
// with the HIP sources.
//
// What it follows.  The paper (Section 4.2, "Online Monitoring Strategy")
// fixes the shape of the decision and nothing else:
//   * every metric is judged relative to the peers of the same job, not
//     against absolute thresholds                       -> go_score (median,
//                                                          MAD, robust z)
//   * a node is flagged only when several indicators deviate, with training
//     step time as the primary one                      -> go_score (combine)
//   * and only when the deviation is sustained over consecutive evaluation
//     windows                                           -> go_window
//   * the unit acted upon is the 8-GPU node (Section 7.1) -> node scores,
//                                                          go_flags, go_topk
//   * the response to a flagged node depends on how much it slows the job
//     (none / about 10% / 20% or more)                  -> go_severity
//   * each indicator sustained on its own, then combined  -> go_metric_window
//   * ranking by the node score averaged over the window -> go_score_ring,
//                                                          go_topk_mean
//   * a node that keeps coming back to triage (three times within a week,
//     Section 7) is terminally bad                      -> go_recurrence
// The estimators and constants (median, MAD x 1.4826, threshold, k-of-W,
// scaled node sum, ranking key) are this repository's stated reading of those
// sentences; each function says which rule it implements.
//
// Arithmetic: IEEE fp32, round-to-nearest-even, one rounding per written
// operation (compile with -ffp-contract=off, no fast-math), denormals kept.
// Selection is done by sorting; windows are re-summed from scratch.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

struct go_config {
    uint32_t n_ranks;        // R, multiple of gpus_per_node
    uint32_t gpus_per_node;  // G
    uint32_t n_metrics;      // M in 1..8
    uint32_t primary_metric;
    uint32_t min_signals;
    uint32_t window;         // W
    uint32_t persist_k;      // k
    uint32_t node_agg;       // 0 = scaled sum, 1 = max
    float z_threshold;
    float node_scale;
    float rel_floor;
    float abs_floor;
    int8_t direction[8];     // +1, -1, or 0 (two-sided)
};

}  // extern "C"

namespace {

// Rule "order": values compare numerically; a negative zero is read as +0.
inline float canon(float v) { return v == 0.0f ? 0.0f : v; }

// Rule "median": sort; odd count -> the middle value; even count -> the two
// middle values added, then halved, each step rounded to fp32.
float median_by_sort(std::vector<float>& v) {
    std::sort(v.begin(), v.end());
    const size_t n = v.size();
    if (n & 1) return v[n / 2];
    float s = v[n / 2 - 1] + v[n / 2];
    return 0.5f * s;
}

// Rule "signed score": z' = z for direction +1, -z for -1, |z| for 0.
inline float signed_score(float z, int dir) {
    if (dir > 0) return z;
    if (dir < 0) return -z;
    return std::fabs(z);
}

inline bool near_threshold(float zs, float thr) {
    return std::fabs((double)zs - (double)thr) <= 1e-5 * std::fabs((double)thr);
}

// Order-preserving map fp32 -> u32 (larger float <=> larger integer).
inline uint32_t order_key(float f) {
    uint32_t b;
    std::memcpy(&b, &f, 4);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

}  // namespace

extern "C" {

// Threads the column-parallel loops will use (columns are independent).
int go_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// Limit the column-parallel loops to n threads (n >= 1), e.g. to time one core.
void go_set_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

// The median rule on its own (any count >= 1), after reading -0 as +0.
float go_median(const float* v, uint64_t n) {
    std::vector<float> w(n);
    for (uint64_t i = 0; i < n; ++i) w[i] = canon(v[i]);
    return median_by_sort(w);
}

// Score T steps of x[t][m][r].
//   med, mad        [T][M]
//   z               [T][M][R] or null        (unsigned robust z, before direction)
//   exceed_mask     [T][R]   bit m = metric m exceeds for that rank
//   rank_anom       [T][ceil(R/64)] bit (r%64) of word r/64
//   node_z          [T][N]   node score of the primary metric
//   node_mask       [T][N]   bit m = node score of metric m exceeds
//   node_anom       [T][ceil(N/64)]
//   node_z_all      [T][M][N] or null        (node score of every metric)
//   near            [2] or null: += number of rank / node comparisons whose score
//                   lies within 1e-5 (relative) of the threshold
void go_score(const go_config* c, const float* x, uint64_t T, float* med, float* mad, float* z,
              uint8_t* exceed_mask, uint64_t* rank_anom, float* node_z, uint8_t* node_mask,
              uint64_t* node_anom, float* node_z_all, uint64_t* near) {
    const size_t R = c->n_ranks, G = c->gpus_per_node, M = c->n_metrics, N = R / G;
    const size_t RW = (R + 63) / 64, NW = (N + 63) / 64;
    const float thr = c->z_threshold;
    uint64_t near_rank = 0, near_node = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : near_rank, near_node)
    for (int64_t t = 0; t < (int64_t)T; ++t) {
        std::vector<float> col(R), work(R), zs(R), nz(N);
        std::vector<uint8_t> E(R, 0), NE(N, 0);
        for (size_t m = 0; m < M; ++m) {
            const float* xc = x + ((size_t)t * M + m) * R;
            for (size_t r = 0; r < R; ++r) col[r] = canon(xc[r]);
            // Rule "missing": a NaN is a sample that did not arrive.  It is left out of
            // the column's median and MAD (taken over the samples present), scores
            // z = 0, never exceeds and adds 0 to its node's score.  A column with no
            // sample present has med = MAD = NaN and nobody exceeds.
            // peer baseline: median over the ranks present in this step and metric
            work.clear();
            for (size_t r = 0; r < R; ++r)
                if (!std::isnan(col[r])) work.push_back(col[r]);
            const bool any_present = !work.empty();
            const float md = any_present ? median_by_sort(work) : std::nanf("");
            // spread: median of absolute deviations from that median
            work.clear();
            for (size_t r = 0; r < R; ++r)
                if (!std::isnan(col[r])) work.push_back(std::fabs(col[r] - md));
            const float ma = any_present ? median_by_sort(work) : std::nanf("");
            med[(size_t)t * M + m] = md;
            mad[(size_t)t * M + m] = ma;
            // scale with floors, so that a column with MAD = 0 stays finite
            float s = 1.4826f * ma;
            float fl = c->rel_floor * std::fabs(md);
            s = std::max(s, fl);
            s = std::max(s, c->abs_floor);
            const int dir = c->direction[m];
            for (size_t r = 0; r < R; ++r) {
                if (std::isnan(col[r])) {           // missing
                    if (z) z[((size_t)t * M + m) * R + r] = 0.0f;
                    zs[r] = 0.0f;
                    continue;
                }
                float d = col[r] - md;
                float zr = d / s;
                if (z) z[((size_t)t * M + m) * R + r] = zr;
                zs[r] = signed_score(zr, dir);
                if (zs[r] > thr) E[r] |= (uint8_t)(1u << m);
                if (near_threshold(zs[r], thr)) ++near_rank;
            }
            // node score over the node's G consecutive ranks
            for (size_t n = 0; n < N; ++n) {
                const float* q = &zs[n * G];
                float v;
                if (c->node_agg == 0) {
                    // pairwise tree, fixed order (G == 8)
                    float a01 = q[0] + q[1], a23 = q[2] + q[3];
                    float a45 = q[4] + q[5], a67 = q[6] + q[7];
                    float lo = a01 + a23, hi = a45 + a67;
                    float sum = lo + hi;
                    v = c->node_scale * sum;
                } else {
                    v = q[0];
                    for (size_t g = 1; g < G; ++g) v = std::max(v, q[g]);
                    // the largest of zeros of both signs has no sign of its own: a zero
                    // node score is reported as +0 (rule "order" reads -0 as +0 as well)
                    v = canon(v);
                }
                nz[n] = v;
                if (v > thr) NE[n] |= (uint8_t)(1u << m);
                if (near_threshold(v, thr)) ++near_node;
                if (node_z_all) node_z_all[((size_t)t * M + m) * N + n] = v;
                if (m == c->primary_metric) node_z[(size_t)t * N + n] = v;
            }
        }
        // multi-signal rule: the primary metric must exceed, and at least
        // min_signals metrics in total
        for (size_t w = 0; w < RW; ++w) rank_anom[(size_t)t * RW + w] = 0;
        for (size_t r = 0; r < R; ++r) {
            exceed_mask[(size_t)t * R + r] = E[r];
            bool a = ((E[r] >> c->primary_metric) & 1u) &&
                     (uint32_t)__builtin_popcount(E[r]) >= c->min_signals;
            if (a) rank_anom[(size_t)t * RW + r / 64] |= (uint64_t)1 << (r % 64);
        }
        for (size_t w = 0; w < NW; ++w) node_anom[(size_t)t * NW + w] = 0;
        for (size_t n = 0; n < N; ++n) {
            node_mask[(size_t)t * N + n] = NE[n];
            bool a = ((NE[n] >> c->primary_metric) & 1u) &&
                     (uint32_t)__builtin_popcount(NE[n]) >= c->min_signals;
            if (a) node_anom[(size_t)t * NW + n / 64] |= (uint64_t)1 << (n % 64);
        }
    }
    if (near) {
        near[0] += near_rank;
        near[1] += near_node;
    }
}

// Persistence (Section 4.2: a deviation must last over successive evaluations): for every
// item i (a rank or a node) and every step t of the whole history,
//   c_i(t) = number of anomalous steps among the last W steps ending at t
// recomputed by an explicit loop; flag_i(t) = c_i(t) >= k; first_i = first t
// with a flag, or -1.  anom is the full history [T][ceil(n/64)] from step 0.
//   count, flag : values at the last step (all zero if T == 0)
//   first       : over the whole history
//   count_hist  : [T][n] or null
void go_window(uint32_t n, const uint64_t* anom, uint64_t T, uint32_t W, uint32_t k,
               uint16_t* count, uint8_t* flag, int32_t* first, uint16_t* count_hist) {
    const size_t words = ((size_t)n + 63) / 64;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        std::vector<uint8_t> a(T);
        for (uint64_t t = 0; t < T; ++t) a[t] = (anom[t * words + i / 64] >> (i % 64)) & 1u;
        int32_t f = -1;
        uint32_t c = 0;
        for (uint64_t t = 0; t < T; ++t) {
            uint64_t lo = t + 1 >= W ? t + 1 - W : 0;
            c = 0;
            for (uint64_t u = lo; u <= t; ++u) c += a[u];
            if (c >= k && f < 0) f = (int32_t)t;
            if (count_hist) count_hist[t * n + i] = (uint16_t)c;
        }
        count[i] = (uint16_t)c;
        flag[i] = (T > 0 && c >= k) ? 1 : 0;
        first[i] = f;
    }
}

// Node flag byte reported to the operator: bit 0 = the node's own persistence
// flag, bit 1 = at least one of its G ranks is currently flagged.
void go_node_flag_byte(uint32_t N, uint32_t G, const uint8_t* node_flag, const uint8_t* rank_flag,
                       uint8_t* out) {
    for (uint32_t n = 0; n < N; ++n) {
        uint8_t b = node_flag[n] ? 1 : 0;
        for (uint32_t g = 0; g < G; ++g)
            if (rank_flag[(size_t)n * G + g]) b |= 2;
        out[n] = b;
    }
}

// Ranking of the slowest nodes: order all nodes by (persistence count, high
// first; latest primary node score, high first, compared numerically; node
// index, low first) and return the first k with the packed key
//   count << 48 | order_key(score) << 16 | (0xFFFF - index).
void go_topk(uint32_t N, const uint16_t* node_count, const float* node_z_last, uint32_t k,
             int32_t* idx, uint64_t* key) {
    std::vector<uint32_t> order(N);
    for (uint32_t n = 0; n < N; ++n) order[n] = n;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        if (node_count[a] != node_count[b]) return node_count[a] > node_count[b];
        float za = node_z_last[a], zb = node_z_last[b];
        if (za != zb) return za > zb;
        return a < b;
    });
    for (uint32_t j = 0; j < k && j < N; ++j) {
        uint32_t n = order[j];
        idx[j] = (int32_t)n;
        key[j] = ((uint64_t)node_count[n] << 48) |
                 ((uint64_t)order_key(canon(node_z_last[n])) << 16) | (uint64_t)(0xFFFFu - n);
    }
}

// Severity of the performance impact of a flagged node (Section 4.2, the tiered
// response: no observable impact / moderate, sustained slowdown of about 10% /
// severe degradation of 20% or more).  Reading: over the last min(T, W) steps of
// the history x[t][m][r], every sample of the node's G GPUs in the primary metric
// is divided by that step's cross-rank median (med[t][M] as go_score wrote it);
// a lower-is-worse primary divides the other way round, a two-sided one takes
// whichever quotient is >= 1.  The node's slowdown is the median of those
// min(T, W) * G quotients (rule "median") minus 1, each operation rounded to fp32.
// Missing samples (NaN, rule "missing") and steps whose median is NaN are left out;
// a flagged node with no quotient at all reports slowdown 0 in tier 1.
//   tier 0: node_flag_byte[n] == 0 (not flagged; slowdown reported as 0)
//   tier 1: flagged, slowdown <  moderate           ("pending verification")
//   tier 2: flagged, moderate <= slowdown < severe  (mitigate at next checkpoint)
//   tier 3: flagged, slowdown >= severe             (replace the node now)
void go_severity(const go_config* c, const float* x, uint64_t T, const float* med,
                 const uint8_t* node_flag_byte, float moderate, float severe, float* slowdown,
                 uint8_t* tier) {
    const uint32_t R = c->n_ranks, G = c->gpus_per_node, M = c->n_metrics, N = R / G;
    const uint32_t p = c->primary_metric;
    const int dir = c->direction[p];
    const uint64_t Ws = T < c->window ? T : c->window;
    for (uint32_t n = 0; n < N; ++n) {
        slowdown[n] = 0.0f;
        tier[n] = 0;
        if (!node_flag_byte[n] || Ws == 0) continue;
        std::vector<float> q;
        for (uint64_t t = T - Ws; t < T; ++t) {
            const float m = med[t * M + p];
            for (uint32_t g = 0; g < G; ++g) {
                const float xv = canon(x[(t * M + p) * (uint64_t)R + (uint64_t)n * G + g]);
                if (std::isnan(xv) || std::isnan(m)) continue;     // rule "missing": left out
                float r;
                if (dir > 0) r = xv / m;
                else if (dir < 0) r = m / xv;
                else r = xv >= m ? xv / m : m / xv;
                q.push_back(r);
            }
        }
        if (q.empty()) {            // flagged, but nothing arrived inside the window
            tier[n] = 1;
            continue;
        }
        const float s = median_by_sort(q) - 1.0f;
        slowdown[n] = s;
        tier[n] = s >= severe ? 3 : (s >= moderate ? 2 : 1);
    }
}

// Single-node sweep scoring (Section 5, "Single-Node Sweep": consistent sustained
// throughput across the GPUs of a node; connectivity and symmetry of the pairwise
// intra-node bandwidth).  Reading, per node b of n_nodes, G = 8:
//   flops[b][g]      sustained throughput of GPU g
//   bw[b][i][j]      bandwidth measured from GPU i to GPU j (the diagonal is ignored)
//   m8   = median of the 8 throughputs (rule "median");
//   shortfall[b][g] = (m8 - flops_g) / m8;          gpu_mask bit g : shortfall > tol_compute
//   m56  = median of the 56 off-diagonal bandwidths;
//   for every pair i < j, numbered p = 0..27 row by row ((0,1), (0,2), ... (6,7)):
//     hi = max(bw_ij, bw_ji), lo = min(bw_ij, bw_ji)
//     link_mask bit p : (hi - lo) / hi > tol_sym  ||  (m56 - lo) / m56 > tol_bw
//   verdict[b] = (gpu_mask != 0) | (link_mask != 0) << 1
// every operation rounded to fp32.
void go_sweep(uint32_t n_nodes, const float* flops, const float* bw, float tol_compute, float tol_sym,
              float tol_bw, float* shortfall, uint8_t* gpu_mask, uint32_t* link_mask,
              uint8_t* verdict) {
    for (uint32_t b = 0; b < n_nodes; ++b) {
        const float* f = flops + (size_t)b * 8;
        const float* w = bw + (size_t)b * 64;
        std::vector<float> v(f, f + 8);
        const float m8 = median_by_sort(v);
        uint8_t gm = 0;
        for (int g = 0; g < 8; ++g) {
            const float d = m8 - f[g];
            const float sf = d / m8;
            shortfall[(size_t)b * 8 + g] = sf;
            if (sf > tol_compute) gm |= (uint8_t)(1u << g);
        }
        std::vector<float> off;
        for (int i = 0; i < 8; ++i)
            for (int j = 0; j < 8; ++j)
                if (i != j) off.push_back(w[i * 8 + j]);
        const float m56 = median_by_sort(off);
        uint32_t lm = 0;
        int p = 0;
        for (int i = 0; i < 8; ++i)
            for (int j = i + 1; j < 8; ++j, ++p) {
                const float a = w[i * 8 + j], c = w[j * 8 + i];
                const float hi = std::max(a, c), lo = std::min(a, c);
                const float gap = hi - lo;
                const float asym = gap / hi;
                const float d = m56 - lo;
                const float sf = d / m56;
                if (asym > tol_sym || sf > tol_bw) lm |= 1u << p;
            }
        gpu_mask[b] = gm;
        link_mask[b] = lm;
        verdict[b] = (uint8_t)((gm ? 1 : 0) | (lm ? 2 : 0));
    }
}

// Rule "combine" on its own (Section 4.2: several indicators must deviate, the
// primary one -- training step time -- among them): from exceed bytes mask[T][n]
// (bit m = metric m exceeds) to the anomaly words anom[T][ceil(n/64)] that go_score
// itself writes: bit set iff bit `primary` is set and at least min_signals bits are.
void go_combine(uint32_t n, uint32_t primary, uint32_t min_signals, const uint8_t* mask, uint64_t T,
                uint64_t* anom) {
    const size_t words = ((size_t)n + 63) / 64;
    for (uint64_t t = 0; t < T; ++t) {
        for (size_t w = 0; w < words; ++w) anom[t * words + w] = 0;
        for (uint32_t i = 0; i < n; ++i) {
            const uint8_t b = mask[t * n + i];
            uint32_t set = 0;
            for (int m = 0; m < 8; ++m) set += (b >> m) & 1u;
            if (((b >> primary) & 1u) && set >= min_signals) anom[t * words + i / 64] |= 1ull << (i % 64);
        }
    }
}

// Elastic membership (ranks join and leave a job; polled telemetry does not always
// answer, Section 7.1): active[T][ceil(R/64)] has bit r%64 of word r/64 set when rank
// r takes part in step t.  A rank that does not is, for every metric of that step, a
// sample that did not arrive: its value becomes the quiet NaN 0x7FC00000 (rule
// "missing").  In place on x[T][M][R].
void go_apply_membership(float* x, uint64_t T, uint32_t M, uint32_t R, const uint64_t* active) {
    const size_t words = ((size_t)R + 63) / 64;
    const uint32_t qnan = 0x7FC00000u;
    for (uint64_t t = 0; t < T; ++t)
        for (uint32_t m = 0; m < M; ++m)
            for (uint32_t r = 0; r < R; ++r)
                if (!((active[t * words + r / 64] >> (r % 64)) & 1ull))
                    std::memcpy(&x[(t * M + m) * (uint64_t)R + r], &qnan, 4);
}

// Persistence kept per indicator (the other reading of Section 4.2's rule that several
// indicators must deviate and keep deviating over successive evaluations:
// each indicator must itself be sustained, and the indicators are combined
// afterwards).  mask is the full history [T][n] of exceed bytes (bit m = metric m
// exceeds for that item at that step) from step 0.  For every item and step:
//   c_m(t) = number of steps among the last W ending at t with bit m set
//   p_m(t) = c_m(t) >= k
//   flag(t) = p_primary(t)  and  (number of m with p_m(t)) >= min_signals
//   count [8][n], pmask [n] (bit m = p_m), flag [n] : at the last step (0 if T == 0)
//   first [n] : first step with flag, or -1
void go_metric_window(uint32_t n, uint32_t primary, uint32_t min_signals, const uint8_t* mask,
                      uint64_t T, uint32_t W, uint32_t k, uint16_t* count, uint8_t* pmask,
                      uint8_t* flag, int32_t* first) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        int32_t f = -1;
        uint32_t c[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        uint8_t pm = 0, fl = 0;
        for (uint64_t t = 0; t < T; ++t) {
            const uint64_t lo = t + 1 >= W ? t + 1 - W : 0;
            pm = 0;
            uint32_t np = 0;
            for (int m = 0; m < 8; ++m) {
                c[m] = 0;
                for (uint64_t u = lo; u <= t; ++u) c[m] += (mask[u * n + i] >> m) & 1u;
                if (c[m] >= k) { pm |= (uint8_t)(1u << m); ++np; }
            }
            fl = ((pm >> primary) & 1u) && np >= min_signals ? 1 : 0;
            if (fl && f < 0) f = (int32_t)t;
        }
        for (int m = 0; m < 8; ++m) count[(size_t)m * n + i] = (uint16_t)c[m];
        pmask[i] = pm;
        flag[i] = fl;
        first[i] = f;
    }
}

// Node score averaged over the window, for ranking: each step's primary node score
// is quantised to an integer, q = clamp(round-half-even(node_z * quant), -32768, 32767)
// (the product rounded to fp32 first; a NaN counts as 0), and
//   sum[n] = q summed over the last min(T, W) steps of the history node_z[T][N].
// All nodes share the divisor, so ordering by the sum is ordering by the mean; integer
// sums do not depend on the order of addition.
void go_score_ring(uint32_t N, const float* node_z, uint64_t T, uint32_t W, float quant,
                   int32_t* sum) {
    const uint64_t Ws = T < W ? T : W;
    for (uint32_t n = 0; n < N; ++n) {
        int32_t s = 0;
        for (uint64_t t = T - Ws; t < T; ++t) {
            const float v = node_z[t * N + n] * quant;
            int32_t q = 0;
            if (!std::isnan(v)) {
                float r = std::nearbyintf(v);       // round to nearest, ties to even
                if (r > 32767.0f) r = 32767.0f;
                if (r < -32768.0f) r = -32768.0f;
                q = (int32_t)r;
            }
            s += q;
        }
        sum[n] = s;
    }
}

// Ranking by (persistence count, high first; windowed score sum, high first; node
// index, low first), key = count << 48 | (sum + 2^31) << 16 | (0xFFFF - index).
void go_topk_mean(uint32_t N, const uint16_t* node_count, const int32_t* sum, uint32_t k,
                  int32_t* idx, uint64_t* key) {
    std::vector<uint32_t> order(N);
    for (uint32_t n = 0; n < N; ++n) order[n] = n;
    std::sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) {
        if (node_count[a] != node_count[b]) return node_count[a] > node_count[b];
        if (sum[a] != sum[b]) return sum[a] > sum[b];
        return a < b;
    });
    for (uint32_t j = 0; j < k && j < N; ++j) {
        const uint32_t n = order[j];
        idx[j] = (int32_t)n;
        const uint32_t biased = (uint32_t)((int64_t)sum[n] + 2147483648ll);
        key[j] = ((uint64_t)node_count[n] << 48) | ((uint64_t)biased << 16) | (uint64_t)(0xFFFFu - n);
    }
}

// Recurrence (Section 7, triage: a node sent to triage `limit` times within a
// period -- three times within a week in the paper's clusters -- is taken to be
// terminally bad).  flag_hist[T][N] is the node persistence flag of every step from
// step 0.  An episode starts at step t when flag(t) is set and flag(t-1) is not
// (nothing is set before step 0).  For every step,
//   e(t) = number of episode starts s with t - horizon < s <= t;
//   terminal_first[n] = first t with e(t) >= limit, or -1;
//   episodes[n] = min(e(T-1), limit)   (0 if T == 0).
void go_recurrence(uint32_t N, const uint8_t* flag_hist, uint64_t T, uint64_t horizon, uint32_t limit,
                   uint8_t* episodes, int32_t* terminal_first) {
    for (uint32_t n = 0; n < N; ++n) {
        std::vector<uint64_t> starts;
        int32_t tf = -1;
        uint32_t e = 0;
        for (uint64_t t = 0; t < T; ++t) {
            const bool now = flag_hist[t * N + n] != 0;
            const bool before = t > 0 && flag_hist[(t - 1) * N + n] != 0;
            if (now && !before) starts.push_back(t);
            e = 0;
            for (uint64_t s : starts)
                if (s + horizon > t) ++e;
            if (e >= limit && tf < 0) tf = (int32_t)t;
        }
        episodes[n] = (uint8_t)(e < limit ? e : limit);
        terminal_first[n] = tf;
    }
}

}  // extern "C"
