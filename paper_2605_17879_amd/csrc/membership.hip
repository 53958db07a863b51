// Elastic membership: ranks that take no part in a step (they joined later, left,
// or their telemetry was not polled in time -- Section 7.1) become missing samples
// of that step, i.e. quiet NaNs in every metric, which the scoring kernel leaves
// out of the peer statistics.
//
// One thread per four consecutive ranks of one (step, metric) column: it reads the
// four membership bits and stores NaNs only where a bit is clear, so a batch in
// which everybody takes part costs T*R/8 bytes of reads and no writes.
#include "gd_internal.h"

namespace {

constexpr int MEM_NT = 256;

__global__ __launch_bounds__(MEM_NT) void membership_kernel(float* x, const uint64_t* active, uint32_t R,
                                                            uint32_t M, uint32_t RW) {
    const uint32_t quad = blockIdx.x * MEM_NT + threadIdx.x;      // ranks 4*quad .. 4*quad + 3
    const uint32_t t = blockIdx.y;
    if (quad * 4 >= R) return;                                    // (R is a multiple of 8)
    const uint32_t r = quad * 4;
    const uint32_t bits = (uint32_t)(active[(size_t)t * RW + r / 64] >> (r % 64)) & 0xFu;
    if (bits == 0xFu) return;
    const float qnan = __uint_as_float(0x7FC00000u);
    for (uint32_t m = 0; m < M; ++m) {
        float* p = x + ((size_t)t * M + m) * R + r;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (!((bits >> i) & 1u)) p[i] = qnan;
    }
}

}  // namespace

hipError_t gd_launch_membership(float* d_x, const uint64_t* d_active, uint32_t T, uint32_t R, uint32_t M,
                                hipStream_t s) {
    if (T == 0) return hipSuccess;
    if (T > 65535u) return hipErrorInvalidValue;                  // (grid y)
    const uint32_t RW = (R + 63) / 64;
    hipLaunchKernelGGL(membership_kernel, dim3((R / 4 + MEM_NT - 1) / MEM_NT, T), dim3(MEM_NT), 0, s, d_x,
                       d_active, R, M, RW);
    return hipGetLastError();
}
