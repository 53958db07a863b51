// Ranking of the slowest nodes for the operator: nodes ordered by (window
// count, latest primary node score, node index) -- the nodes Section 4.2 would
// remove from the healthy pool first.
//
// The middle field of the key is the latest primary node score or, for the
// ranking by the score averaged over the window, the window's sum of quantised
// scores.
//
// One workgroup builds a unique 64-bit key per node (N <= 8192) and writes the k
// largest in descending order.
//
// k <= 64 (the usual request): no full sort.  Every thread keeps its few keys in
// registers.  The k-th largest of the per-thread maxima is a threshold that at
// least k keys reach and, the maxima being the likeliest top keys, few more do.
// The keys that reach it are compacted into LDS and the k largest of them taken.
// Both "k largest of a list" steps work on 64-key chunks, one key per lane: each
// wave sorts a chunk with a bitonic network of lane exchanges, then one wave
// folds the sorted chunks together, keeping the upper 64 of two chunks at a time
// (max of chunk A's i-th and chunk B's (63-i)-th key is a bitonic sequence that
// holds the 64 largest of both; six more exchange stages sort it).
//
// Larger k: all keys are sorted in LDS with a bitonic network.
#include "gd_internal.h"
#include "gd_lanes.h"

namespace {

constexpr int WAVE = 64;
constexpr int TOPK_NT = 1024;
constexpr int TOPK_MAX = 8192;
constexpr int KPT = TOPK_MAX / TOPK_NT;     // keys per thread
constexpr int CHUNKS = TOPK_NT / WAVE;      // 64-key chunks that one folding pass takes

__device__ __forceinline__ uint32_t key_of(float f) {
    uint32_t b = __float_as_uint(f);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

// One compare-exchange stage across the wave: lanes whose bit J is clear keep
// the larger key when `desc`, the smaller otherwise; their partners the other.
template <int J>
__device__ __forceinline__ uint64_t exchange(uint64_t v, uint32_t lane, bool desc) {
    const uint64_t o = gd_lane_xor64<J>(v, lane);
    const bool keep_max = ((lane & J) == 0) == desc;
    return keep_max ? (v > o ? v : o) : (v < o ? v : o);
}

// A bitonic sequence (one key per lane) into descending order.
__device__ __forceinline__ uint64_t merge_desc(uint64_t v, uint32_t lane) {
    v = exchange<32>(v, lane, true);
    v = exchange<16>(v, lane, true);
    v = exchange<8>(v, lane, true);
    v = exchange<4>(v, lane, true);
    v = exchange<2>(v, lane, true);
    v = exchange<1>(v, lane, true);
    return v;
}

// Any 64 keys (one per lane) into descending order.
__device__ __forceinline__ uint64_t sort_desc(uint64_t v, uint32_t lane) {
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
    return merge_desc(v, lane);
}

// The 64 largest of `chunks` sorted 64-key chunks in LDS, descending, one per
// lane of the calling wave.
__device__ __forceinline__ uint64_t fold_chunks(const uint64_t* lists, uint32_t chunks, uint32_t lane) {
    uint64_t best = lists[lane];
    for (uint32_t c = 1; c < chunks; ++c) {
        const uint64_t other = lists[c * WAVE + (WAVE - 1 - lane)];
        best = merge_desc(best > other ? best : other, lane);
    }
    return best;
}

__global__ __launch_bounds__(TOPK_NT) void topk_kernel(const gd_topk_args a) {
    __shared__ uint64_t keys[TOPK_MAX];
    __shared__ uint64_t threshold;
    __shared__ uint32_t n_reach;
    const uint16_t* nc = a.count;
    const float* nz = a.z_last;
    const uint32_t tid = threadIdx.x, lane = tid & (WAVE - 1), w = tid / WAVE;
    auto make_key = [&](uint32_t n) -> uint64_t {
        if (n >= a.N) return 0;                     // padding sorts last
        uint32_t mid;
        if (nz) mid = key_of(nz[n] + 0.0f);         // -0 ranks as +0
        else mid = (uint32_t)a.score_sum[n] ^ 0x80000000u;   // sum + 2^31: signed order as unsigned
        return ((uint64_t)nc[n] << 48) | ((uint64_t)mid << 16) | (uint64_t)(0xFFFFu - n);
    };
    auto write_out = [&](uint32_t i, uint64_t k) {
        a.idx[i] = (int32_t)(0xFFFFu - (uint32_t)(k & 0xFFFFu));
        if (a.key) a.key[i] = k;
    };

    if (a.k <= (uint32_t)WAVE) {
        uint64_t mine[KPT], top = 0;
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            mine[q] = make_key(q * TOPK_NT + tid);
            top = mine[q] > top ? mine[q] : top;
        }
        if (tid == 0) n_reach = 0;
        keys[tid] = sort_desc(top, lane);           // chunk w of the per-thread maxima
        __syncthreads();
        if (w == 0) {
            const uint64_t best = fold_chunks(keys, CHUNKS, lane);
            if (lane == a.k - 1) threshold = best;  // at least k keys are >= this one
        }
        __syncthreads();
        const uint64_t thr = threshold;
#pragma unroll
        for (int q = 0; q < KPT; ++q) {
            if (mine[q] >= thr && mine[q] != 0) {
                const uint32_t pos = atomicAdd(&n_reach, 1u);
                if (pos < (uint32_t)TOPK_NT) keys[pos] = mine[q];
            }
        }
        __syncthreads();
        // k <= m <= KPT * k: only the k threads with the largest maxima hold such keys
        const uint32_t m = min(n_reach, (uint32_t)TOPK_NT);
        const uint32_t chunks = (m + WAVE - 1) / WAVE;
        if (w < chunks) {
            const uint32_t i = w * WAVE + lane;
            const uint64_t sorted = sort_desc(i < m ? keys[i] : 0, lane);
            keys[i] = sorted;                       // a wave rewrites only its own chunk
        }
        __syncthreads();
        if (w == 0) {
            const uint64_t best = fold_chunks(keys, chunks, lane);
            if (lane < a.k) write_out(lane, best);
        }
        return;
    }

    uint32_t P = 64;
    while (P < a.N) P <<= 1;                       // power of two >= N, <= TOPK_MAX
    for (uint32_t n = tid; n < P; n += TOPK_NT) keys[n] = make_key(n);
    __syncthreads();
    // bitonic sort, descending
    for (uint32_t k = 2; k <= P; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < P / 2; i += TOPK_NT) {
                const uint32_t lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));   // index with bit j clear
                const uint32_t hi = lo | j;
                const bool desc = (lo & k) == 0;
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
            }
            __syncthreads();
        }
    }
    for (uint32_t i = tid; i < a.k; i += TOPK_NT) write_out(i, keys[i]);
}

}  // namespace

hipError_t gd_launch_topk(const gd_topk_args& a, hipStream_t s) {
    if (a.k == 0) return hipSuccess;
    if (a.N > TOPK_MAX || a.k > a.N) return hipErrorInvalidValue;
    hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(TOPK_NT), 0, s, a);
    return hipGetLastError();
}
