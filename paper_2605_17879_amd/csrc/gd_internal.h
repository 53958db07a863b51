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
    const uint8_t* state;
    gd_state_layout lay;
    int32_t* idx;   // [k]
    uint64_t* key;  // [k] or null
    uint32_t N, k;
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
hipError_t gd_launch_sweep(const gd_sweep_args& a, hipStream_t s);
hipError_t gd_launch_severity(const gd_severity_args& a, hipStream_t s);
hipError_t gd_launch_read_probe(const float* d_x, uint64_t n_bytes, uint32_t* d_sink, hipStream_t s);
hipError_t gd_launch_window(const gd_window_args& a, hipStream_t s);
hipError_t gd_launch_flags(const gd_flags_args& a, hipStream_t s);
hipError_t gd_launch_topk(const gd_topk_args& a, hipStream_t s);

#endif  // GD_INTERNAL_H_
