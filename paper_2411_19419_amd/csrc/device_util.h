// Small device-side helpers shared by the build and apply kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace convspmv {

constexpr int kWave = 64;   // CDNA wavefront width

// DPP cross-lane move.  The controls used here are all XOR butterflies inside
// a row of 16 lanes: quad_perm [1,0,3,2] = lane^1, [2,3,0,1] = lane^2,
// row_half_mirror = lane^7, row_mirror = lane^15.  Every lane of the wave
// must be active when these are executed.
constexpr int kDppXor1 = 0xB1;
constexpr int kDppXor2 = 0x4E;
constexpr int kDppXor7 = 0x141;
constexpr int kDppXor15 = 0x140;

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over aligned groups of G consecutive lanes (G = 1, 2, 4, 8, 16); every
// lane of the group ends up with the total.
template <int G>
__device__ __forceinline__ float group_sum(float v) {
    static_assert(G == 1 || G == 2 || G == 4 || G == 8 || G == 16, "group width");
    if (G >= 2) v += dpp_move<kDppXor1>(v);
    if (G >= 4) v += dpp_move<kDppXor2>(v);
    if (G >= 8) v += dpp_move<kDppXor7>(v);
    if (G >= 16) v += dpp_move<kDppXor15>(v);
    return v;
}

// floor(a / d) for 0 <= a < 2^21 and d >= 1, with inv = 1/d in fp32 (an error
// of one ulp in inv is tolerated).  a + 0.5 is exact; inv and the product are
// off by at most 2^-23 and 2^-24 relative, so the computed value is within
// 1.5 * 2^-24 * 2^21 / d < 0.19/d of (a + 0.5)/d, which itself is at least
// 0.5/d away from every integer: truncation gives the exact quotient.
__device__ __forceinline__ int div_small(int a, float inv) {
    return (int)(((float)a + 0.5f) * inv);
}

// Where the lanes of one wave hand data to each other through LDS without a workgroup barrier
// (the LDS instructions of a wave execute in order): later LDS accesses of this wave stay
// behind earlier ones, for the compiler too.
__device__ __forceinline__ void wave_lds_order() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

}  // namespace convspmv
