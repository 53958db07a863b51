// Host side of the C ABI declared in guard.h: configuration checks, the layout
// of the caller's state buffer, argument validation and the kernel launches.
// No device memory is allocated here and no call synchronises.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <string>

#include "../../include/guard.h"
#include "gd_internal.h"

struct gd_handle_s {
    gd_config cfg;
    uint32_t N, RW, NW;
    gd_state_layout lay;
    uint8_t* d_state;
    uint32_t split_steps;
    const float* hint_med;
    const float* hint_mad;
    gd_ledger_config lcfg;
    gd_ledger_layout llay;
    uint8_t* d_led;
    uint32_t led_max_T;
    std::string err;
};

namespace {

std::string g_create_error;

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

gd_state_layout make_layout(uint32_t R, uint32_t N, uint32_t W) {
    const size_t RW = (R + 63) / 64, NW = (N + 63) / 64;
    gd_state_layout l;
    size_t o = 0;
    l.rank_ring = o;   o = align256(o + (size_t)W * RW * 8);
    l.node_ring = o;   o = align256(o + (size_t)W * NW * 8);
    l.rank_count = o;  o = align256(o + (size_t)R * 2);
    l.node_count = o;  o = align256(o + (size_t)N * 2);
    l.rank_first = o;  o = align256(o + (size_t)R * 4);
    l.node_first = o;  o = align256(o + (size_t)N * 4);
    l.node_z_last = o; o = align256(o + (size_t)N * 4);
    l.total = o;
    return l;
}

gd_ledger_layout make_ledger_layout(uint32_t R, uint32_t N, uint32_t W, uint32_t max_T) {
    const size_t NW = (N + 63) / 64;
    gd_ledger_layout l;
    size_t o = 0;
    l.head = o;        o = align256(o + 32);
    l.rank_ring = o;   o = align256(o + (size_t)W * R);
    l.node_ring = o;   o = align256(o + (size_t)W * N);
    l.rank_cnt = o;    o = align256(o + (size_t)R * 16);
    l.node_cnt = o;    o = align256(o + (size_t)N * 16);
    l.node_ccnt = o;   o = align256(o + (size_t)N * 2);
    l.counts_bytes = o - l.rank_cnt;
    l.counts_new = o;  o += l.counts_bytes;
    l.rank_first = o;  o = align256(o + (size_t)R * 4);
    l.node_first = o;  o = align256(o + (size_t)N * 4);
    l.node_qring = o;  o = align256(o + (size_t)W * N * 2);
    l.node_qsum = o;   o = align256(o + (size_t)N * 4);
    l.node_starts = o; o = align256(o + (size_t)N * 32);
    l.node_term = o;   o = align256(o + (size_t)N * 4);
    l.rise = o;        o = align256(o + (size_t)max_T * NW * 8);
    l.total = o;
    return l;
}

gd_status fail(gd_handle h, gd_status st, const std::string& msg) {
    if (h) h->err = msg; else g_create_error = msg;
    return st;
}

gd_status hip_fail(gd_handle h, hipError_t e, const char* what) {
    return fail(h, GD_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

}  // namespace

extern "C" {

void gd_default_config(gd_config* c, uint32_t n_ranks, uint32_t n_metrics, uint32_t window,
                       uint32_t persist_k) {
    if (!c) return;
    memset(c, 0, sizeof(*c));
    c->struct_size = (uint32_t)sizeof(gd_config);
    c->n_ranks = n_ranks;
    c->gpus_per_node = 8;
    c->n_metrics = n_metrics;
    c->primary_metric = 0;
    c->min_signals = n_metrics < 2 ? n_metrics : 2;
    c->window = window;
    c->persist_k = persist_k;
    const uint32_t N = n_ranks / 8;
    c->topk = N < 64 ? N : 64;
    c->node_agg = GD_NODE_SUM_SCALED;
    c->z_threshold = 3.5f;
    c->node_scale = 0.35355338f;   // 1/sqrt(8)
    c->rel_floor = 1e-6f;
    c->abs_floor = 1e-30f;
    for (int i = 0; i < GD_MAX_METRICS; ++i) c->direction[i] = 1;
}

gd_status gd_create(const gd_config* c, gd_handle* out) {
    if (out) *out = nullptr;
    if (!c || !out) return fail(nullptr, GD_ERR_INVALID_ARG, "gd_create: null argument");
    if (c->struct_size != sizeof(gd_config))
        return fail(nullptr, GD_ERR_BAD_CONFIG, "struct_size does not match this library's gd_config");
    if (c->gpus_per_node != 8)
        return fail(nullptr, GD_ERR_UNSUPPORTED, "only gpus_per_node = 8 is built");
    if (c->n_ranks < 8 || c->n_ranks % 8 != 0)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "n_ranks must be a positive multiple of gpus_per_node");
    if (c->n_ranks > GD_MAX_RANKS)
        return fail(nullptr, GD_ERR_UNSUPPORTED, "n_ranks above 65536 is not built");
    if (c->n_metrics < 1 || c->n_metrics > GD_MAX_METRICS)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "n_metrics must be 1..8");
    if (c->primary_metric >= c->n_metrics)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "primary_metric out of range");
    if (c->min_signals < 1 || c->min_signals > c->n_metrics)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "min_signals must be 1..n_metrics");
    if (c->window < 1 || c->window > GD_MAX_WINDOW)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "window must be 1..1024");
    if (c->persist_k < 1 || c->persist_k > c->window)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "persist_k must be 1..window");
    const uint32_t N = c->n_ranks / 8;
    if (c->topk > N) return fail(nullptr, GD_ERR_BAD_CONFIG, "topk exceeds the number of nodes");
    if (c->node_agg != GD_NODE_SUM_SCALED && c->node_agg != GD_NODE_MAX)
        return fail(nullptr, GD_ERR_BAD_CONFIG, "unknown node_agg");
    if (!isfinite(c->z_threshold) || !isfinite(c->node_scale) || !(c->rel_floor >= 0.0f) ||
        !(c->abs_floor > 0.0f) || !isfinite(c->rel_floor) || !isfinite(c->abs_floor))
        return fail(nullptr, GD_ERR_BAD_CONFIG,
                    "threshold and node_scale must be finite, rel_floor >= 0, abs_floor > 0");
    for (uint32_t m = 0; m < c->n_metrics; ++m)
        if (c->direction[m] < -1 || c->direction[m] > 1)
            return fail(nullptr, GD_ERR_BAD_CONFIG, "direction must be -1, 0 or +1");
    gd_handle h = new (std::nothrow) gd_handle_s();
    if (!h) return fail(nullptr, GD_ERR_INVALID_ARG, "out of host memory");
    h->cfg = *c;
    h->N = N;
    h->RW = (c->n_ranks + 63) / 64;
    h->NW = (N + 63) / 64;
    h->lay = make_layout(c->n_ranks, N, c->window);
    h->d_state = nullptr;
    h->split_steps = GD_DEFAULT_STREAMING_STEPS;
    h->hint_med = nullptr;
    h->hint_mad = nullptr;
    h->d_led = nullptr;
    h->led_max_T = 0;
    *out = h;
    return GD_OK;
}

gd_status gd_destroy(gd_handle h) {
    delete h;
    return GD_OK;
}

gd_status gd_set_streaming_steps(gd_handle h, uint32_t max_steps) {
    if (!h) return GD_ERR_INVALID_ARG;
    h->split_steps = max_steps;
    return GD_OK;
}

gd_status gd_set_streaming_hints(gd_handle h, const float* d_med, const float* d_mad) {
    if (!h) return GD_ERR_INVALID_ARG;
    if ((d_med == nullptr) != (d_mad == nullptr))
        return fail(h, GD_ERR_INVALID_ARG, "gd_set_streaming_hints: give both arrays or neither");
    if (((uintptr_t)d_med & 3) || ((uintptr_t)d_mad & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_set_streaming_hints: misaligned pointer");
    h->hint_med = d_med;
    h->hint_mad = d_mad;
    return GD_OK;
}

size_t gd_state_bytes(gd_handle h) { return h ? h->lay.total : 0; }

gd_status gd_bind_state(gd_handle h, void* d_state, size_t state_bytes) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!d_state) return fail(h, GD_ERR_INVALID_ARG, "gd_bind_state: null state");
    if (((uintptr_t)d_state & 255) != 0)
        return fail(h, GD_ERR_INVALID_ARG, "gd_bind_state: state must be 256-byte aligned");
    if (state_bytes < h->lay.total)
        return fail(h, GD_ERR_BUFFER_TOO_SMALL, "gd_bind_state: buffer smaller than gd_state_bytes");
    h->d_state = static_cast<uint8_t*>(d_state);
    return GD_OK;
}

gd_status gd_score_batch(gd_handle h, const float* d_x, uint32_t T, float* d_med, float* d_mad,
                         float* d_z, uint8_t* d_exceed_mask, uint64_t* d_rank_anom,
                         float* d_node_z, uint8_t* d_node_mask, uint64_t* d_node_anom,
                         void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (T == 0) return GD_OK;
    if (!d_x || !d_med || !d_mad || !d_exceed_mask || !d_rank_anom || !d_node_z || !d_node_mask ||
        !d_node_anom)
        return fail(h, GD_ERR_INVALID_ARG, "gd_score_batch: a required pointer is null");
    if (((uintptr_t)d_x & 15) || ((uintptr_t)d_z & 15) || ((uintptr_t)d_exceed_mask & 3) ||
        ((uintptr_t)d_rank_anom & 7) || ((uintptr_t)d_node_anom & 7) || ((uintptr_t)d_node_z & 3) ||
        ((uintptr_t)d_med & 3) || ((uintptr_t)d_mad & 3))
        return fail(h, GD_ERR_INVALID_ARG,
                    "gd_score_batch: x and z must be 16-byte aligned, the other arrays naturally aligned");
    gd_score_args a;
    a.x = d_x; a.med = d_med; a.mad = d_mad; a.z = d_z;
    a.exceed_mask = d_exceed_mask; a.rank_anom = d_rank_anom;
    a.node_z = d_node_z; a.node_mask = d_node_mask; a.node_anom = d_node_anom;
    a.T = T; a.R = h->cfg.n_ranks; a.M = h->cfg.n_metrics; a.N = h->N;
    a.primary = h->cfg.primary_metric; a.min_signals = h->cfg.min_signals;
    a.node_agg = h->cfg.node_agg;
    a.split_steps = h->split_steps;
    a.hint_med = h->hint_med; a.hint_mad = h->hint_mad;
    a.thr = h->cfg.z_threshold; a.node_scale = h->cfg.node_scale;
    a.rel_floor = h->cfg.rel_floor; a.abs_floor = h->cfg.abs_floor;
    memcpy(a.dir, h->cfg.direction, 8);
    hipError_t e = gd_launch_score(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_score_batch");
    return GD_OK;
}

gd_status gd_update_window(gd_handle h, const uint64_t* d_rank_anom, const uint64_t* d_node_anom,
                           const float* d_node_z, uint32_t T, uint64_t first_step_index,
                           void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_state) return fail(h, GD_ERR_INVALID_ARG, "gd_update_window: no state bound");
    if (T == 0) return GD_OK;
    if (!d_rank_anom || !d_node_anom || !d_node_z)
        return fail(h, GD_ERR_INVALID_ARG, "gd_update_window: a required pointer is null");
    if (((uintptr_t)d_rank_anom & 7) || ((uintptr_t)d_node_anom & 7) || ((uintptr_t)d_node_z & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_update_window: misaligned pointer");
    if (first_step_index + (uint64_t)T > 0x7FFFFFFFull)
        return fail(h, GD_ERR_INVALID_ARG, "gd_update_window: step index beyond 2^31 - 1");
    gd_window_args a;
    a.state = h->d_state; a.lay = h->lay;
    a.rank_anom = d_rank_anom; a.node_anom = d_node_anom; a.node_z = d_node_z;
    a.T = T; a.R = h->cfg.n_ranks; a.N = h->N; a.W = h->cfg.window; a.K = h->cfg.persist_k;
    a.first_step = first_step_index;
    hipError_t e = gd_launch_window(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_update_window");
    return GD_OK;
}

gd_status gd_flags(gd_handle h, uint8_t* d_rank_flag, uint16_t* d_rank_count,
                   int32_t* d_rank_first, uint8_t* d_node_flag, uint16_t* d_node_count,
                   int32_t* d_node_first, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_state) return fail(h, GD_ERR_INVALID_ARG, "gd_flags: no state bound");
    if (((uintptr_t)d_rank_count & 1) || ((uintptr_t)d_node_count & 1) ||
        ((uintptr_t)d_rank_first & 3) || ((uintptr_t)d_node_first & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_flags: misaligned pointer");
    gd_flags_args a;
    a.state = h->d_state; a.lay = h->lay;
    a.rank_flag = d_rank_flag; a.rank_count = d_rank_count; a.rank_first = d_rank_first;
    a.node_flag = d_node_flag; a.node_count = d_node_count; a.node_first = d_node_first;
    a.R = h->cfg.n_ranks; a.N = h->N; a.K = h->cfg.persist_k;
    hipError_t e = gd_launch_flags(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_flags");
    return GD_OK;
}

gd_status gd_topk_nodes(gd_handle h, uint32_t k, int32_t* d_idx, uint64_t* d_key, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_state) return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes: no state bound");
    if (k == 0) k = h->cfg.topk;
    if (k == 0) return GD_OK;
    if (k > h->N) return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes: k exceeds the number of nodes");
    if (!d_idx) return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes: null index output");
    if (((uintptr_t)d_idx & 3) || ((uintptr_t)d_key & 7))
        return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes: misaligned pointer");
    gd_topk_args a;
    a.count = reinterpret_cast<const uint16_t*>(h->d_state + h->lay.node_count);
    a.z_last = reinterpret_cast<const float*>(h->d_state + h->lay.node_z_last);
    a.score_sum = nullptr;
    a.idx = d_idx; a.key = d_key; a.N = h->N; a.k = k;
    hipError_t e = gd_launch_topk(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_topk_nodes");
    return GD_OK;
}

gd_status gd_apply_membership(gd_handle h, float* d_x, uint32_t T, const uint64_t* d_active, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (T == 0) return GD_OK;
    if (!d_x || !d_active) return fail(h, GD_ERR_INVALID_ARG, "gd_apply_membership: null pointer");
    if (((uintptr_t)d_x & 15) || ((uintptr_t)d_active & 7))
        return fail(h, GD_ERR_INVALID_ARG, "gd_apply_membership: misaligned pointer");
    if (T > 65535u) return fail(h, GD_ERR_INVALID_ARG, "gd_apply_membership: more than 65535 steps in one call");
    hipError_t e = gd_launch_membership(d_x, d_active, T, h->cfg.n_ranks, h->cfg.n_metrics,
                                        static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_apply_membership");
    return GD_OK;
}

gd_status gd_severity(gd_handle h, const float* d_x, uint32_t T, const float* d_med, float moderate,
                      float severe, float* d_node_slowdown, uint8_t* d_node_tier, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_state) return fail(h, GD_ERR_INVALID_ARG, "gd_severity: no state bound");
    if (!d_node_slowdown || !d_node_tier)
        return fail(h, GD_ERR_INVALID_ARG, "gd_severity: null output");
    if (T > 0 && (!d_x || !d_med)) return fail(h, GD_ERR_INVALID_ARG, "gd_severity: null input");
    if (((uintptr_t)d_x & 3) || ((uintptr_t)d_med & 3) || ((uintptr_t)d_node_slowdown & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_severity: misaligned pointer");
    if (!(moderate <= severe)) return fail(h, GD_ERR_INVALID_ARG, "gd_severity: moderate must not exceed severe");
    gd_severity_args a;
    a.state = h->d_state; a.lay = h->lay; a.x = d_x; a.med = d_med;
    a.slowdown = d_node_slowdown; a.tier = d_node_tier;
    a.T = T; a.R = h->cfg.n_ranks; a.M = h->cfg.n_metrics; a.N = h->N;
    a.W = h->cfg.window; a.K = h->cfg.persist_k; a.primary = h->cfg.primary_metric;
    a.dir = h->cfg.direction[h->cfg.primary_metric];
    a.moderate = moderate; a.severe = severe;
    hipError_t e = gd_launch_severity(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_severity");
    return GD_OK;
}

gd_status gd_sweep_score(gd_handle h, const float* d_flops, const float* d_bw, uint32_t n_nodes,
                         float tol_compute, float tol_sym, float tol_bw, float* d_gpu_shortfall,
                         uint8_t* d_gpu_mask, uint32_t* d_link_mask, uint8_t* d_verdict, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (n_nodes == 0) return GD_OK;
    if (!d_flops || !d_bw || !d_gpu_shortfall || !d_gpu_mask || !d_link_mask || !d_verdict)
        return fail(h, GD_ERR_INVALID_ARG, "gd_sweep_score: null pointer");
    if (((uintptr_t)d_flops & 3) || ((uintptr_t)d_bw & 3) || ((uintptr_t)d_gpu_shortfall & 3) ||
        ((uintptr_t)d_link_mask & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_sweep_score: misaligned pointer");
    gd_sweep_args a;
    a.flops = d_flops; a.bw = d_bw; a.shortfall = d_gpu_shortfall; a.gpu_mask = d_gpu_mask;
    a.link_mask = d_link_mask; a.verdict = d_verdict; a.n_nodes = n_nodes;
    a.tol_compute = tol_compute; a.tol_sym = tol_sym; a.tol_bw = tol_bw;
    hipError_t e = gd_launch_sweep(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_sweep_score");
    return GD_OK;
}

void gd_default_ledger_config(gd_ledger_config* c) {
    if (!c) return;
    memset(c, 0, sizeof(*c));
    c->struct_size = (uint32_t)sizeof(gd_ledger_config);
    c->score_quant = 64.0f;
    c->recur_limit = 3;
    c->recur_horizon = 604800;
}

size_t gd_ledger_bytes(gd_handle h, uint32_t max_T) {
    return h ? make_ledger_layout(h->cfg.n_ranks, h->N, h->cfg.window, max_T).total : 0;
}

gd_status gd_bind_ledger(gd_handle h, const gd_ledger_config* cfg, void* d_ledger, size_t bytes,
                         uint32_t max_T) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!cfg || !d_ledger) return fail(h, GD_ERR_INVALID_ARG, "gd_bind_ledger: null argument");
    if (cfg->struct_size != sizeof(gd_ledger_config))
        return fail(h, GD_ERR_BAD_CONFIG, "struct_size does not match this library's gd_ledger_config");
    if (!isfinite(cfg->score_quant) || !(cfg->score_quant > 0.0f))
        return fail(h, GD_ERR_BAD_CONFIG, "score_quant must be finite and positive");
    if (cfg->recur_limit < 1 || cfg->recur_limit > 8)
        return fail(h, GD_ERR_BAD_CONFIG, "recur_limit must be 1..8");
    if (cfg->recur_horizon < 1 || cfg->recur_horizon > (1ull << 62))
        return fail(h, GD_ERR_BAD_CONFIG, "recur_horizon must be 1..2^62 steps");
    if (max_T < 1) return fail(h, GD_ERR_INVALID_ARG, "gd_bind_ledger: max_T must be at least 1");
    if (((uintptr_t)d_ledger & 255) != 0)
        return fail(h, GD_ERR_INVALID_ARG, "gd_bind_ledger: ledger must be 256-byte aligned");
    const gd_ledger_layout l = make_ledger_layout(h->cfg.n_ranks, h->N, h->cfg.window, max_T);
    if (bytes < l.total)
        return fail(h, GD_ERR_BUFFER_TOO_SMALL, "gd_bind_ledger: buffer smaller than gd_ledger_bytes");
    h->lcfg = *cfg;
    h->llay = l;
    h->d_led = static_cast<uint8_t*>(d_ledger);
    h->led_max_T = max_T;
    return GD_OK;
}

namespace {

// Checks and arguments shared by the two entry points that take a batch into the ledger.
gd_status ledger_update_args(gd_handle h, const char* who, const uint8_t* d_exceed_mask,
                             const uint8_t* d_node_mask, const float* d_node_z, uint32_t T,
                             uint64_t first_step_index, gd_ledger_args* out) {
    const std::string name(who);
    if (!d_exceed_mask || !d_node_mask || !d_node_z)
        return fail(h, GD_ERR_INVALID_ARG, name + ": a required pointer is null");
    if (((uintptr_t)d_exceed_mask & 3) || ((uintptr_t)d_node_z & 3))
        return fail(h, GD_ERR_INVALID_ARG, name + ": misaligned pointer");
    if (first_step_index + (uint64_t)T > 0x7FFFFFFFull)
        return fail(h, GD_ERR_INVALID_ARG, name + ": step index beyond 2^31 - 1");
    gd_ledger_args& a = *out;
    a.led = h->d_led; a.lay = h->llay;
    a.rise = reinterpret_cast<uint64_t*>(h->d_led + h->llay.rise);
    a.counts_new = h->d_led + h->llay.counts_new;
    a.exceed_mask = d_exceed_mask; a.node_mask = d_node_mask; a.node_z = d_node_z;
    a.T = T; a.R = h->cfg.n_ranks; a.N = h->N; a.W = h->cfg.window; a.K = h->cfg.persist_k;
    a.primary = h->cfg.primary_metric; a.min_signals = h->cfg.min_signals;
    // A chunk rebuilds its starting counts from the W steps before it.  Chunks as
    // short as the window double the steps read, but that part only counts (it is
    // the cheaper half), and a long batch needs the workgroups: measured at 65 536
    // ranks x 4 096 steps, W = 256: chunks of 2W 0.40 ms, of W 0.29 ms.
    a.chunk = h->cfg.window < 128 ? 128 : h->cfg.window;
    a.limit = h->lcfg.recur_limit;
    a.quant = h->lcfg.score_quant;
    a.first_step = first_step_index; a.horizon = h->lcfg.recur_horizon;
    return GD_OK;
}

}  // namespace

gd_status gd_update_ledger(gd_handle h, const uint8_t* d_exceed_mask, const uint8_t* d_node_mask,
                           const float* d_node_z, uint32_t T, uint64_t first_step_index,
                           void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_led) return fail(h, GD_ERR_INVALID_ARG, "gd_update_ledger: no ledger bound");
    if (T == 0) return GD_OK;
    if (T > h->led_max_T)
        return fail(h, GD_ERR_INVALID_ARG, "gd_update_ledger: T exceeds the max_T the ledger was bound with");
    gd_ledger_args a;
    const gd_status st = ledger_update_args(h, "gd_update_ledger", d_exceed_mask, d_node_mask, d_node_z, T,
                                            first_step_index, &a);
    if (st != GD_OK) return st;
    hipError_t e = gd_launch_ledger(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_update_ledger");
    return GD_OK;
}

size_t gd_ledger_static_scratch_bytes(void) { return gd_ledger_static_bytes(); }

gd_status gd_update_ledger_static(gd_handle h, const uint8_t* d_exceed_mask, const uint8_t* d_node_mask,
                                  const float* d_node_z, uint32_t T, uint64_t first_step_index,
                                  void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_led) return fail(h, GD_ERR_INVALID_ARG, "gd_update_ledger_static: no ledger bound");
    if (T == 0) return GD_OK;
    gd_ledger_args a;
    const gd_status st = ledger_update_args(h, "gd_update_ledger_static", d_exceed_mask, d_node_mask,
                                            d_node_z, T, first_step_index, &a);
    if (st != GD_OK) return st;
    bool fits = true;
    hipError_t e = gd_launch_ledger_static(a, static_cast<hipStream_t>(stream), &fits);
    if (!fits) {
        char msg[200];
        snprintf(msg, sizeof msg,
                 "gd_update_ledger_static: %u steps of %u nodes need more than the %zu bytes of the "
                 "library's static work area; send shorter batches",
                 T, h->N, gd_ledger_static_bytes());
        return fail(h, GD_ERR_INVALID_ARG, msg);
    }
    if (e != hipSuccess) return hip_fail(h, e, "gd_update_ledger_static");
    return GD_OK;
}

gd_status gd_ledger_flags(gd_handle h, uint8_t* d_rank_pmask, uint8_t* d_rank_pflag,
                          int32_t* d_rank_pfirst, uint8_t* d_node_pmask, uint8_t* d_node_pflag,
                          int32_t* d_node_pfirst, int32_t* d_node_score_sum,
                          uint8_t* d_node_episodes, int32_t* d_node_terminal_first, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_led) return fail(h, GD_ERR_INVALID_ARG, "gd_ledger_flags: no ledger bound");
    if (((uintptr_t)d_rank_pfirst & 3) || ((uintptr_t)d_node_pfirst & 3) ||
        ((uintptr_t)d_node_score_sum & 3) || ((uintptr_t)d_node_terminal_first & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_ledger_flags: misaligned pointer");
    gd_ledger_flags_args a;
    a.led = h->d_led; a.lay = h->llay;
    a.rank_pmask = d_rank_pmask; a.rank_pflag = d_rank_pflag; a.rank_pfirst = d_rank_pfirst;
    a.node_pmask = d_node_pmask; a.node_pflag = d_node_pflag; a.node_pfirst = d_node_pfirst;
    a.node_score_sum = d_node_score_sum; a.node_episodes = d_node_episodes;
    a.node_terminal_first = d_node_terminal_first;
    a.R = h->cfg.n_ranks; a.N = h->N; a.K = h->cfg.persist_k;
    a.primary = h->cfg.primary_metric; a.min_signals = h->cfg.min_signals;
    a.limit = h->lcfg.recur_limit; a.horizon = h->lcfg.recur_horizon;
    hipError_t e = gd_launch_ledger_flags(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_ledger_flags");
    return GD_OK;
}

gd_status gd_topk_nodes_mean(gd_handle h, uint32_t k, int32_t* d_idx, uint64_t* d_key, void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!h->d_led) return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes_mean: no ledger bound");
    if (k == 0) k = h->cfg.topk;
    if (k == 0) return GD_OK;
    if (k > h->N) return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes_mean: k exceeds the number of nodes");
    if (!d_idx) return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes_mean: null index output");
    if (((uintptr_t)d_idx & 3) || ((uintptr_t)d_key & 7))
        return fail(h, GD_ERR_INVALID_ARG, "gd_topk_nodes_mean: misaligned pointer");
    gd_topk_args a;
    a.count = reinterpret_cast<const uint16_t*>(h->d_led + h->llay.node_ccnt);
    a.z_last = nullptr;
    a.score_sum = reinterpret_cast<const int32_t*>(h->d_led + h->llay.node_qsum);
    a.idx = d_idx; a.key = d_key; a.N = h->N; a.k = k;
    hipError_t e = gd_launch_topk(a, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_topk_nodes_mean");
    return GD_OK;
}

gd_status gd_probe_read(gd_handle h, const float* d_x, uint64_t n_bytes, uint32_t* d_sink,
                        void* stream) {
    if (!h) return GD_ERR_INVALID_ARG;
    if (!d_x || !d_sink) return fail(h, GD_ERR_INVALID_ARG, "gd_probe_read: null pointer");
    if (((uintptr_t)d_x & 15) || ((uintptr_t)d_sink & 3))
        return fail(h, GD_ERR_INVALID_ARG, "gd_probe_read: misaligned pointer");
    hipError_t e = gd_launch_read_probe(d_x, n_bytes, d_sink, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(h, e, "gd_probe_read");
    return GD_OK;
}

const char* gd_last_error(gd_handle h) { return h ? h->err.c_str() : g_create_error.c_str(); }

}  // extern "C"
