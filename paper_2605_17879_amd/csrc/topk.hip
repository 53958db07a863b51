// Ranking of the slowest nodes for the operator: nodes ordered by (window
// count, latest primary node score, node index) -- the nodes Section 4.2 would
// remove from the healthy pool first.
//
// One workgroup builds a unique 64-bit key per node, sorts all keys in LDS with
// a bitonic network (N <= 8192 keys, 64 KB) and writes the first k.
#include "gd_internal.h"

namespace {

constexpr int TOPK_NT = 1024;
constexpr int TOPK_MAX = 8192;

__device__ __forceinline__ uint32_t key_of(float f) {
    uint32_t b = __float_as_uint(f);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

__global__ __launch_bounds__(TOPK_NT) void topk_kernel(const gd_topk_args a) {
    __shared__ uint64_t keys[TOPK_MAX];
    const uint16_t* nc = reinterpret_cast<const uint16_t*>(a.state + a.lay.node_count);
    const float* nz = reinterpret_cast<const float*>(a.state + a.lay.node_z_last);
    uint32_t P = 64;
    while (P < a.N) P <<= 1;                       // power of two >= N, <= TOPK_MAX
    for (uint32_t n = threadIdx.x; n < P; n += TOPK_NT) {
        uint64_t k = 0;                             // padding sorts last
        if (n < a.N) {
            const float z = nz[n] + 0.0f;           // -0 ranks as +0
            k = ((uint64_t)nc[n] << 48) | ((uint64_t)key_of(z) << 16) | (uint64_t)(0xFFFFu - n);
        }
        keys[n] = k;
    }
    __syncthreads();
    // bitonic sort, descending
    for (uint32_t k = 2; k <= P; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = threadIdx.x; i < P / 2; i += TOPK_NT) {
                const uint32_t lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));   // index with bit j clear
                const uint32_t hi = lo | j;
                const bool desc = (lo & k) == 0;
                const uint64_t x = keys[lo], y = keys[hi];
                if ((x < y) == desc) { keys[lo] = y; keys[hi] = x; }
            }
            __syncthreads();
        }
    }
    for (uint32_t i = threadIdx.x; i < a.k; i += TOPK_NT) {
        const uint64_t k = keys[i];
        a.idx[i] = (int32_t)(0xFFFFu - (uint32_t)(k & 0xFFFFu));
        if (a.key) a.key[i] = k;
    }
}

}  // namespace

hipError_t gd_launch_topk(const gd_topk_args& a, hipStream_t s) {
    if (a.k == 0) return hipSuccess;
    if (a.N > TOPK_MAX || a.k > a.N) return hipErrorInvalidValue;
    hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(TOPK_NT), 0, s, a);
    return hipGetLastError();
}
