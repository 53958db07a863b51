// Severity of the performance impact of the flagged nodes (Section 4.2: the
// tiered response -- no observable impact, a moderate sustained slowdown of
// about 10%, a severe one of 20% or more).
//
// One workgroup per node.  A node that is not flagged (its own window count and
// those of its 8 ranks all below k) reports tier 0 and leaves at once.  For a
// flagged node the workgroup forms the quotient of each of the node's 8
// primary-metric samples of the last min(T, W) steps by that step's cross-rank
// median, sorts the at most 8192 quotients in LDS (bitonic network on
// order-preserving integer keys) and takes the median of them minus one.
// Missing samples (NaN) are left out.
#include "gd_internal.h"

namespace {

constexpr int SEV_NT = 256;
constexpr int SEV_MAX = 8192;     // 8 GPUs x the longest window

__device__ __forceinline__ uint32_t key_of(float f) {
    uint32_t b = __float_as_uint(f);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}
__device__ __forceinline__ float float_of_key(uint32_t k) {
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

__global__ __launch_bounds__(SEV_NT) void severity_kernel(const gd_severity_args a) {
    __shared__ uint32_t q[SEV_MAX];
    __shared__ uint32_t n_present;
    const uint32_t n = blockIdx.x, tid = threadIdx.x;
    const uint16_t* rc = reinterpret_cast<const uint16_t*>(a.state + a.lay.rank_count);
    const uint16_t* nc = reinterpret_cast<const uint16_t*>(a.state + a.lay.node_count);
    bool flagged = nc[n] >= a.K;
    for (int g = 0; g < 8; ++g) flagged |= rc[(size_t)n * 8 + g] >= a.K;   // uniform over the workgroup
    const uint32_t ws = a.T < a.W ? a.T : a.W;
    if (!flagged || ws == 0) {
        if (tid == 0) { a.slowdown[n] = 0.0f; a.tier[n] = 0; }
        return;
    }
    const uint32_t cnt = ws * 8;
    if (tid == 0) n_present = 0;
    __syncthreads();
    uint32_t P = 64;
    while (P < cnt) P <<= 1;                   // power of two >= cnt, <= SEV_MAX
    for (uint32_t i = tid; i < P; i += SEV_NT) {
        uint32_t k = 0xFFFFFFFFu;              // padding sorts last
        if (i < cnt) {
            const size_t t = a.T - ws + i / 8;
            const float m = a.med[t * a.M + a.primary];
            const float xv = a.x[(t * a.M + a.primary) * (size_t)a.R + (size_t)n * 8 + (i & 7)] + 0.0f;
            float r;
            if (a.dir > 0) r = xv / m;
            else if (a.dir < 0) r = m / xv;
            else r = xv >= m ? xv / m : m / xv;
            // a missing sample (NaN), or a step without a median, is left out: its key
            // sorts with the padding
            if (xv == xv && m == m) {
                k = key_of(r);
                atomicAdd(&n_present, 1u);
            }
        }
        q[i] = k;
    }
    __syncthreads();
    for (uint32_t k = 2; k <= P; k <<= 1) {    // bitonic sort, ascending
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < P / 2; i += SEV_NT) {
                const uint32_t lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const uint32_t hi = lo | j;
                const bool asc = (lo & k) == 0;
                const uint32_t u = q[lo], w = q[hi];
                if ((u > w) == asc) { q[lo] = w; q[hi] = u; }
            }
            __syncthreads();
        }
    }
    if (tid == 0) {
        const uint32_t np = n_present;
        if (np == 0) {              // flagged, but nothing arrived inside the window
            a.slowdown[n] = 0.0f;
            a.tier[n] = 1;
            return;
        }
        // the middle quotient, or the two middle ones added, then halved
        const float mid = (np & 1) ? float_of_key(q[np / 2])
                                   : 0.5f * (float_of_key(q[np / 2 - 1]) + float_of_key(q[np / 2]));
        const float s = mid - 1.0f;
        a.slowdown[n] = s;
        a.tier[n] = s >= a.severe ? 3 : (s >= a.moderate ? 2 : 1);
    }
}

}  // namespace

hipError_t gd_launch_severity(const gd_severity_args& a, hipStream_t s) {
    if (a.N == 0) return hipSuccess;
    hipLaunchKernelGGL(severity_kernel, dim3(a.N), dim3(SEV_NT), 0, s, a);
    return hipGetLastError();
}
