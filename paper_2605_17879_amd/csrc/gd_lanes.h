// Cross-lane helpers shared by the kernels: wave-wide moves with immediate
// patterns (DPP, swizzle, permlane swap) -- no address registers involved.
#ifndef GD_LANES_H_
#define GD_LANES_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

// Value held by lane (lane ^ J) of the same wave, J a power of two below 64.
template <int J>
__device__ __forceinline__ uint32_t gd_lane_xor(uint32_t v, uint32_t lane) {
    if constexpr (J == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);
    else if constexpr (J == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);
    else if constexpr (J == 8) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x128, 0xF, 0xF, true);
    else if constexpr (J == 4 || J == 16)
        return (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x1F | (J << 10));
    else {
        static_assert(J == 32, "gd_lane_xor");
        auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return (lane & 32) ? r[0] : r[1];
    }
}

template <int J>
__device__ __forceinline__ uint64_t gd_lane_xor64(uint64_t v, uint32_t lane) {
    const uint32_t lo = gd_lane_xor<J>((uint32_t)v, lane);
    const uint32_t hi = gd_lane_xor<J>((uint32_t)(v >> 32), lane);
    return ((uint64_t)hi << 32) | lo;
}

// Transpose of the 64x64 bit matrix whose row i is the word held by lane i:
// afterwards bit j of lane i is what bit i of lane j was.  For every index bit
// K the rows and columns exchange that bit (a butterfly with the lane i ^ K).
template <int K>
__device__ __forceinline__ uint64_t gd_transpose_stage(uint64_t x, uint32_t lane) {
    constexpr uint64_t m = K == 32 ? 0x00000000FFFFFFFFull
                         : K == 16 ? 0x0000FFFF0000FFFFull
                         : K == 8  ? 0x00FF00FF00FF00FFull
                         : K == 4  ? 0x0F0F0F0F0F0F0F0Full
                         : K == 2  ? 0x3333333333333333ull
                                   : 0x5555555555555555ull;
    const uint64_t p = gd_lane_xor64<K>(x, lane);
    if ((lane & K) == 0) {
        const uint64_t t = ((x >> K) ^ p) & m;
        return x ^ (t << K);
    }
    const uint64_t t = ((p >> K) ^ x) & m;
    return x ^ t;
}

__device__ __forceinline__ uint64_t gd_transpose64(uint64_t x, uint32_t lane) {
    x = gd_transpose_stage<32>(x, lane);
    x = gd_transpose_stage<16>(x, lane);
    x = gd_transpose_stage<8>(x, lane);
    x = gd_transpose_stage<4>(x, lane);
    x = gd_transpose_stage<2>(x, lane);
    x = gd_transpose_stage<1>(x, lane);
    return x;
}

#endif  // GD_LANES_H_
