// Internal interface between the host side of the C ABI and the HIP kernels.
// Nothing here is exported.
#ifndef GD_INTERNAL_H_
#define GD_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

// Arguments of the scoring kernel (a workgroup scores whole steps: all M
// columns of R ranks, Section 4.2 peer-relative evaluation).
struct gd_score_args {
    const float* x;        // [T][M][R]
    float* med;            // [T][M]
    float* mad;            // [T][M]
    float* z;              // [T][M][R] or null
    uint8_t* exceed_mask;  // [T][R]
    uint64_t* rank_anom;   // [T][RW]
    float* node_z;         // [T][N]
    uint8_t* node_mask;    // [T][N]
    uint64_t* node_anom;   // [T][NW]
    uint32_t T, R, M, N;
    uint32_t primary, min_signals, node_agg;
    uint32_t split_steps;  // batches of at most this many steps take one workgroup per column
    const float* hint_med;  // [M] medians and
    const float* hint_mad;  // [M] MADs of a recent step, or null: where a one-step call starts looking
    float thr, node_scale, rel_floor, abs_floor;
    int8_t dir[8];
};

// Where each part of the caller's state buffer lives (byte offsets, each a
// multiple of 256).  Zero bytes are a fresh window: counts 0, "first flagged
// step" stored as step+1 so that 0 means never.
struct gd_state_layout {
    size_t rank_ring;   // u64 [W][RW]   anomaly bits of the last W steps, slot = step % W
    size_t node_ring;   // u64 [W][NW]
    size_t rank_count;  // u16 [R]
    size_t node_count;  // u16 [N]
    size_t rank_first;  // i32 [R]       first flagged step + 1
    size_t node_first;  // i32 [N]
    size_t node_z_last; // f32 [N]       latest primary node score
    size_t total;
};

struct gd_window_args {
    uint8_t* state;
    gd_state_layout lay;
    const uint64_t* rank_anom;  // [T][RW]
    const uint64_t* node_anom;  // [T][NW]
    const float* node_z;        // [T][N]
    uint32_t T, R, N, W, K;
    uint64_t first_step;
};

struct gd_flags_args {
    const uint8_t* state;
    gd_state_layout lay;
    uint8_t* rank_flag;
    uint16_t* rank_count;
    int32_t* rank_first;
    uint8_t* node_flag;
    uint16_t* node_count;
    int32_t* node_first;
    uint32_t R, N, K;
};

struct gd_topk_args {
    const uint16_t* count;   // [N] window counts
    const float* z_last;     // [N] latest primary node score, or null:
    const int32_t* score_sum;  // [N] windowed sum of quantised node scores (used when z_last is null)
    int32_t* idx;   // [k]
    uint64_t* key;  // [k] or null
    uint32_t N, k;
};

// The ledger: bookkeeping beyond the default rule (persistence per indicator, the
// node score summed over the window, recurrence of flag episodes).  Byte offsets
// into the caller's ledger buffer, each a multiple of 256; zero bytes are a fresh
// ledger.
struct gd_ledger_layout {
    size_t head;         // u64 [4]      [0] = index of the step after the last one taken in
    size_t rank_ring;    // u8  [W][R]   exceed bytes of the last W steps, slot = step % W
    size_t node_ring;    // u8  [W][N]
    size_t rank_cnt;     // u16 [8][R]   per-metric window counts             } one span,
    size_t node_cnt;     // u16 [8][N]                                        } counts_bytes
    size_t node_ccnt;    // u16 [N]      window count of the per-step combined node anomaly  } long
    size_t counts_new;   // the same span again: where a batch cut into chunks leaves its final counts
    size_t counts_bytes;
    size_t rank_first;   // u32 [R]      0xFFFFFFFF - first flagged step, 0 = never
    size_t node_first;   // u32 [N]
    size_t node_qring;   // i16 [W][N]   quantised primary node scores of the last W steps
    size_t node_qsum;    // i32 [N]      their sum
    size_t node_starts;  // i32 [8][N]   the latest episode starts (step + 1, 0 = none), newest first
    size_t node_term;    // i32 [N]      first step with `limit` episodes inside the horizon, + 1
    size_t rise;         // u64 [max_T][NW]  work area: episode starts found in the batch
    size_t total;
};

struct gd_ledger_args {
    uint8_t* led;
    gd_ledger_layout lay;
    // The two spans that only serve the kernels of one call (not part of the ledger's
    // contents): inside the caller's buffer at lay.rise / lay.counts_new, or in the
    // library's own static device array for the entry point that may not allocate.
    uint64_t* rise;               // [NW][T] episode starts found in the batch
    uint8_t* counts_new;          // lay.counts_bytes: final counts of a batch cut into chunks
    const uint8_t* exceed_mask;   // [T][R]
    const uint8_t* node_mask;     // [T][N]
    const float* node_z;          // [T][N]
    uint32_t T, R, N, W, K, primary, min_signals;
    uint32_t chunk;               // steps per workgroup row of the counting kernel
    uint32_t limit;               // episodes that make a node terminal (1..8)
    float quant;
    uint64_t first_step, horizon;
};

struct gd_ledger_flags_args {
    const uint8_t* led;
    gd_ledger_layout lay;
    uint8_t* rank_pmask;  uint8_t* rank_pflag;  int32_t* rank_pfirst;
    uint8_t* node_pmask;  uint8_t* node_pflag;  int32_t* node_pfirst;
    int32_t* node_score_sum;
    uint8_t* node_episodes;
    int32_t* node_terminal_first;
    uint32_t R, N, K, primary, min_signals, limit;
    uint64_t horizon;
};

struct gd_severity_args {
    const uint8_t* state;
    gd_state_layout lay;
    const float* x;     // [T][M][R]
    const float* med;   // [T][M]
    float* slowdown;    // [N]
    uint8_t* tier;      // [N]
    uint32_t T, R, M, N, W, K, primary;
    int32_t dir;        // direction of the primary metric
    float moderate, severe;
};

struct gd_sweep_args {
    const float* flops;   // [n_nodes][8]
    const float* bw;      // [n_nodes][8][8]
    float* shortfall;     // [n_nodes][8]
    uint8_t* gpu_mask;    // [n_nodes]
    uint32_t* link_mask;  // [n_nodes]
    uint8_t* verdict;     // [n_nodes]
    uint32_t n_nodes;
    float tol_compute, tol_sym, tol_bw;
};

hipError_t gd_launch_score(const gd_score_args& a, hipStream_t s);
hipError_t gd_launch_score_with_z(const gd_score_args& a, hipStream_t s);   // score_z.hip
hipError_t gd_launch_sweep(const gd_sweep_args& a, hipStream_t s);
hipError_t gd_launch_membership(float* d_x, const uint64_t* d_active, uint32_t T, uint32_t R, uint32_t M,
                                hipStream_t s);
hipError_t gd_launch_severity(const gd_severity_args& a, hipStream_t s);
hipError_t gd_launch_read_probe(const float* d_x, uint64_t n_bytes, uint32_t* d_sink, hipStream_t s);
hipError_t gd_launch_window(const gd_window_args& a, hipStream_t s);
hipError_t gd_launch_flags(const gd_flags_args& a, hipStream_t s);
hipError_t gd_launch_topk(const gd_topk_args& a, hipStream_t s);
hipError_t gd_launch_ledger(const gd_ledger_args& a, hipStream_t s);
// The same launch with the work spans placed in the library's static device array;
// *fits = false (and nothing launched) when the batch needs more than the array holds.
hipError_t gd_launch_ledger_static(gd_ledger_args a, hipStream_t s, bool* fits);
size_t gd_ledger_static_bytes();
hipError_t gd_launch_ledger_flags(const gd_ledger_flags_args& a, hipStream_t s);

#endif  // GD_INTERNAL_H_
