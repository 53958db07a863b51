// Sliding-window persistence (k anomalous evaluations among the last W: the
// requirement of Section 4.2 that a deviation persists over several evaluations
// in a row before a node is flagged) and the read-out of the current flags.
//
// State in HBM, per item (a rank or a node): a ring of the last W anomaly bits,
// stored as the scoring kernel's own bit words ring[step % W][item / 64]; a u16
// count of set bits inside the window; the first flagged step (+1, 0 = never).
//
// One thread owns one item and one wave owns one 64-item word column of the
// ring, so every ring word is read and written by a single wave.  A wave takes
// 64 steps at a time (fetched a few blocks ahead): lane l fetches the word
// entering at step s0 + l and the
// word leaving the window at that step (the one that entered W steps earlier,
// from the batch itself when recent enough, else from the ring).  Two 64x64 bit
// transposes across the lanes turn them into per-item time vectors, so a block
// of 64 steps updates the count with two popcounts.  Only an item that could
// reach k inside the block (count + entering bits >= k, not flagged before)
// walks the block step by step to find its first flagged step.
#include "gd_internal.h"
#include "gd_lanes.h"

namespace {

constexpr int WAVE = 64;
constexpr int WIN_NT = 256;

// Items [0, R) are ranks, then, starting at a fresh workgroup, items [0, N) are nodes.
// RING > 0: the window is RING blocks of 64 steps long, so the bits leaving during a
// block are the bits that entered RING blocks earlier -- already transposed then and
// kept in registers; only the blocks that reach back beyond the batch transpose ring
// words.  RING == 0: any window length, two transposes per block.
template <int RING>
__global__ __launch_bounds__(WIN_NT) void window_kernel(const gd_window_args a) {
    const uint32_t rank_blocks = (a.R + WIN_NT - 1) / WIN_NT;
    const bool is_node = blockIdx.x >= rank_blocks;
    const uint32_t n_items = is_node ? a.N : a.R;
    const uint32_t blk = is_node ? blockIdx.x - rank_blocks : blockIdx.x;
    const uint32_t item = blk * WIN_NT + threadIdx.x;
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const uint32_t words = (n_items + 63) / 64;
    const uint32_t word = item / 64;                 // uniform over the wave
    if (word >= words) return;                       // whole wave out of range
    const uint64_t* anom = is_node ? a.node_anom : a.rank_anom;
    uint64_t* ring = reinterpret_cast<uint64_t*>(a.state + (is_node ? a.lay.node_ring : a.lay.rank_ring));
    uint16_t* count = reinterpret_cast<uint16_t*>(a.state + (is_node ? a.lay.node_count : a.lay.rank_count));
    int32_t* first = reinterpret_cast<int32_t*>(a.state + (is_node ? a.lay.node_first : a.lay.rank_first));
    const bool live = item < n_items;
    const uint32_t W = a.W, K = a.K, T = a.T;

    // the entering and the leaving word of step s (lane l of a block asks for s0 + l)
    auto fetch = [&](uint32_t s, uint64_t* win, uint64_t* wout) {
        *win = 0; *wout = 0;
        if (s < T) {
            *win = anom[(size_t)s * words + word];
            const uint64_t t = a.first_step + s;
            if (t >= W) {
                if (s < W) *wout = ring[(size_t)(t % W) * words + word];
                else if (RING == 0) *wout = anom[(size_t)(s - W) * words + word];
                // (RING > 0: these bits are still in registers from RING blocks ago)
            }
        }
    };

    uint32_t c = live ? count[item] : 0;
    int32_t f = live ? first[item] : 0;
    // Blocks are fetched AHEAD blocks in advance (the loop is latency-bound: one wave
    // per word column walks its steps in order).
    constexpr int AHEAD = RING > 4 ? RING : 4;
    uint64_t win[AHEAD], wout[AHEAD];
    uint64_t entered[RING > 0 ? RING : 1];      // transposed entering bits of the last RING blocks
#pragma unroll
    for (int q = 0; q < AHEAD; ++q) fetch(q * WAVE + lane, &win[q], &wout[q]);
    for (uint32_t s0 = 0; s0 < T; s0 += AHEAD * WAVE) {
#pragma unroll
        for (int q = 0; q < AHEAD; ++q) {
            const uint32_t sq = s0 + q * WAVE;        // uniform over the wave
            if (sq >= T) break;
            const uint64_t wi = win[q], wo = wout[q];
            fetch(sq + AHEAD * WAVE + lane, &win[q], &wout[q]);
            // bit j of `in` / `out`: does this item enter / leave as anomalous at step sq + j
            const uint64_t in = gd_transpose64(wi, lane);
            uint64_t out;
            if (RING > 0 && sq >= W) {               // (sq and W are multiples of 64)
                const uint32_t n = T - sq;           // steps of the batch in this block
                out = entered[q % (RING > 0 ? RING : 1)] & (n < 64 ? (1ull << n) - 1 : ~0ull);
            }
            else out = gd_transpose64(wo, lane);
            if (RING > 0) entered[q % (RING > 0 ? RING : 1)] = in;
            const uint32_t pin = __popcll(in), pout = __popcll(out);
            if (f == 0 && c + pin >= K) {             // the flag may first rise inside this block
                const uint32_t n = min((uint32_t)WAVE, T - sq);
                for (uint32_t j = 0; j < n; ++j) {
                    const uint64_t upto = (2ull << j) - 1;
                    if (c + __popcll(in & upto) - __popcll(out & upto) >= K) {
                        f = (int32_t)(a.first_step + sq + j) + 1;
                        break;
                    }
                }
            }
            c += pin - pout;
        }
    }
    if (live) {
        count[item] = (uint16_t)c;
        first[item] = f;
    }
    // The last min(T, W) words of the batch become the ring's newest slots.
    // Every ring read above has been consumed before these stores are issued,
    // and no other wave touches this word column.
    const uint32_t keep = T < W ? T : W;
    for (uint32_t i = lane; i < keep; i += WAVE) {
        const uint32_t s = T - keep + i;
        ring[(size_t)((a.first_step + s) % W) * words + word] = anom[(size_t)s * words + word];
    }
    if (is_node && live && T > 0) {
        float* last = reinterpret_cast<float*>(a.state + a.lay.node_z_last);
        last[item] = a.node_z[(size_t)(T - 1) * a.N + item];
    }
}

__global__ __launch_bounds__(WIN_NT) void flags_kernel(const gd_flags_args a) {
    const uint32_t i = blockIdx.x * WIN_NT + threadIdx.x;
    const uint16_t* rc = reinterpret_cast<const uint16_t*>(a.state + a.lay.rank_count);
    const int32_t* rf = reinterpret_cast<const int32_t*>(a.state + a.lay.rank_first);
    const uint16_t* nc = reinterpret_cast<const uint16_t*>(a.state + a.lay.node_count);
    const int32_t* nf = reinterpret_cast<const int32_t*>(a.state + a.lay.node_first);
    if (i < a.R) {
        const uint32_t c = rc[i];
        if (a.rank_flag) a.rank_flag[i] = c >= a.K ? 1 : 0;
        if (a.rank_count) a.rank_count[i] = (uint16_t)c;
        if (a.rank_first) a.rank_first[i] = rf[i] - 1;
    }
    if (i < a.N) {
        const uint32_t c = nc[i];
        if (a.node_flag) {
            uint8_t b = c >= a.K ? 1 : 0;
            // 8 GPUs per node: two 8-byte loads of the ranks' counts
            const uint4 q = *reinterpret_cast<const uint4*>(rc + (size_t)i * 8);
            const uint32_t v[4] = {q.x, q.y, q.z, q.w};
            bool any = false;
#pragma unroll
            for (int j = 0; j < 4; ++j) any |= (v[j] & 0xFFFFu) >= a.K || (v[j] >> 16) >= a.K;
            if (any) b |= 2;
            a.node_flag[i] = b;
        }
        if (a.node_count) a.node_count[i] = (uint16_t)c;
        if (a.node_first) a.node_first[i] = nf[i] - 1;
    }
}

}  // namespace

hipError_t gd_launch_window(const gd_window_args& a, hipStream_t s) {
    if (a.T == 0) return hipSuccess;
    const uint32_t blocks = (a.R + WIN_NT - 1) / WIN_NT + (a.N + WIN_NT - 1) / WIN_NT;
    // batches longer than the window, whose length is a whole number of 64-step blocks
    const uint32_t ring = a.W % 64 == 0 && a.T > a.W ? a.W / 64 : 0;
    switch (ring) {
        case 1: hipLaunchKernelGGL(window_kernel<1>, dim3(blocks), dim3(WIN_NT), 0, s, a); break;
        case 2: hipLaunchKernelGGL(window_kernel<2>, dim3(blocks), dim3(WIN_NT), 0, s, a); break;
        case 4: hipLaunchKernelGGL(window_kernel<4>, dim3(blocks), dim3(WIN_NT), 0, s, a); break;
        case 8: hipLaunchKernelGGL(window_kernel<8>, dim3(blocks), dim3(WIN_NT), 0, s, a); break;
        case 16: hipLaunchKernelGGL(window_kernel<16>, dim3(blocks), dim3(WIN_NT), 0, s, a); break;
        default: hipLaunchKernelGGL(window_kernel<0>, dim3(blocks), dim3(WIN_NT), 0, s, a); break;
    }
    return hipGetLastError();
}

hipError_t gd_launch_flags(const gd_flags_args& a, hipStream_t s) {
    const uint32_t blocks = (a.R + WIN_NT - 1) / WIN_NT;
    hipLaunchKernelGGL(flags_kernel, dim3(blocks), dim3(WIN_NT), 0, s, a);
    return hipGetLastError();
}
