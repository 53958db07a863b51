// Single-node sweep scoring (Section 5, "Single-Node Sweep": consistent sustained
// throughput across a node's GPUs; connectivity and symmetry of the pairwise
// intra-node bandwidth), batched over many nodes.
//
// One wave per node.  Lanes 0-7 hold the 8 throughputs, all 64 lanes one entry of
// the 8x8 bandwidth matrix each.  Both medians come from bitonic networks of lane
// exchanges on order-preserving integer keys (the 8 diagonal entries are replaced
// by keys above everything, so the 56 others sort into lanes 0-55); the shortfall
// and symmetry tests are then one division or two per lane.
#include "gd_internal.h"
#include "gd_lanes.h"

namespace {

constexpr int WAVE = 64;
constexpr int SWEEP_NT = 256;

__device__ __forceinline__ uint32_t key_of(float f) {
    uint32_t b = __float_as_uint(f);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float float_of_key(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// One compare-exchange stage across the wave: lanes whose bit J is clear keep
// the smaller key when `asc`, the larger otherwise; their partners the other.
template <int J>
__device__ __forceinline__ uint32_t exchange(uint32_t v, uint32_t lane, bool asc) {
    const uint32_t o = gd_lane_xor<J>(v, lane);
    const bool keep_min = ((lane & J) == 0) == asc;
    return keep_min ? min(v, o) : max(v, o);
}

// 64 keys, one per lane, into ascending order.
__device__ __forceinline__ uint32_t sort64(uint32_t v, uint32_t lane) {
    v = exchange<1>(v, lane, (lane & 2) == 0);
    v = exchange<2>(v, lane, (lane & 4) == 0);
    v = exchange<1>(v, lane, (lane & 4) == 0);
    v = exchange<4>(v, lane, (lane & 8) == 0);
    v = exchange<2>(v, lane, (lane & 8) == 0);
    v = exchange<1>(v, lane, (lane & 8) == 0);
    v = exchange<8>(v, lane, (lane & 16) == 0);
    v = exchange<4>(v, lane, (lane & 16) == 0);
    v = exchange<2>(v, lane, (lane & 16) == 0);
    v = exchange<1>(v, lane, (lane & 16) == 0);
    v = exchange<16>(v, lane, (lane & 32) == 0);
    v = exchange<8>(v, lane, (lane & 32) == 0);
    v = exchange<4>(v, lane, (lane & 32) == 0);
    v = exchange<2>(v, lane, (lane & 32) == 0);
    v = exchange<1>(v, lane, (lane & 32) == 0);
    v = exchange<32>(v, lane, true);
    v = exchange<16>(v, lane, true);
    v = exchange<8>(v, lane, true);
    v = exchange<4>(v, lane, true);
    v = exchange<2>(v, lane, true);
    v = exchange<1>(v, lane, true);
    return v;
}

// Every group of 8 lanes into ascending order.
__device__ __forceinline__ uint32_t sort8(uint32_t v, uint32_t lane) {
    v = exchange<1>(v, lane, (lane & 2) == 0);
    v = exchange<2>(v, lane, (lane & 4) == 0);
    v = exchange<1>(v, lane, (lane & 4) == 0);
    v = exchange<4>(v, lane, true);
    v = exchange<2>(v, lane, true);
    v = exchange<1>(v, lane, true);
    return v;
}

__device__ __forceinline__ float lane_value(uint32_t v, int src) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)v, src));
}

__global__ __launch_bounds__(SWEEP_NT) void sweep_kernel(const gd_sweep_args a) {
    const uint32_t lane = threadIdx.x & (WAVE - 1);
    const uint32_t b = blockIdx.x * (SWEEP_NT / WAVE) + threadIdx.x / WAVE;      // uniform over the wave
    if (b >= a.n_nodes) return;
    // throughput: lanes 0-7 (the other lanes repeat them, harmlessly)
    const float f = a.flops[(size_t)b * 8 + (lane & 7)];
    const uint32_t fs = sort8(key_of(f), lane);
    const float m8 = 0.5f * (float_of_key((uint32_t)__builtin_amdgcn_readlane((int)fs, 3)) +
                             float_of_key((uint32_t)__builtin_amdgcn_readlane((int)fs, 4)));
    const float shortfall = (m8 - f) / m8;
    const uint64_t gmask = __ballot(lane < 8 && shortfall > a.tol_compute);
    if (lane < 8) a.shortfall[(size_t)b * 8 + lane] = shortfall;
    // bandwidth: lane = 8*i + j holds bw[i][j]
    const uint32_t i = lane >> 3, j = lane & 7;
    const float w = a.bw[(size_t)b * 64 + lane];
    const uint32_t ws = sort64(i == j ? 0xFFFFFFFFu : key_of(w), lane);
    const float m56 = 0.5f * (float_of_key((uint32_t)__builtin_amdgcn_readlane((int)ws, 27)) +
                              float_of_key((uint32_t)__builtin_amdgcn_readlane((int)ws, 28)));
    // the opposite direction of this lane's link sits in lane 8*j + i
    const float back = __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute((int)((j * 8 + i) * 4),
                                                                              (int)__float_as_uint(w)));
    const float hi = fmaxf(w, back), lo = fminf(w, back);
    const float asym = (hi - lo) / hi;
    const float sf = (m56 - lo) / m56;
    const bool bad = i < j && (asym > a.tol_sym || sf > a.tol_bw);
    // pair number of (i, j), i < j, row by row: pairs before row i, then the place in the row
    const uint32_t p = i * 8 - i * (i + 1) / 2 + (j - i - 1);
    uint32_t bits = bad ? 1u << (p & 31) : 0u;
    bits |= gd_lane_xor<1>(bits, lane); bits |= gd_lane_xor<2>(bits, lane); bits |= gd_lane_xor<4>(bits, lane);
    bits |= gd_lane_xor<8>(bits, lane); bits |= gd_lane_xor<16>(bits, lane); bits |= gd_lane_xor<32>(bits, lane);
    if (lane == 0) {
        a.gpu_mask[b] = (uint8_t)gmask;
        a.link_mask[b] = bits;
        a.verdict[b] = (uint8_t)((gmask ? 1 : 0) | (bits ? 2 : 0));
    }
}

}  // namespace

hipError_t gd_launch_sweep(const gd_sweep_args& a, hipStream_t s) {
    if (a.n_nodes == 0) return hipSuccess;
    const uint32_t per = SWEEP_NT / WAVE;
    hipLaunchKernelGGL(sweep_kernel, dim3((a.n_nodes + per - 1) / per), dim3(SWEEP_NT), 0, s, a);
    return hipGetLastError();
}
