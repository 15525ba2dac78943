// Device-side helpers shared by the gfx950 kernels: the fused elementwise
// program, wavefront (64-lane) reductions.
#pragma once

#include <hip/hip_runtime.h>

#include "kernels.h"

namespace clg {

constexpr int kWave = 64;

__device__ __forceinline__ float gelu_erf(float v) {
    return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f));
}

// Applies the fused steps to one value.  `off` is the element's offset in the
// output tensor (EPI_ADD operands have the output's shape); `chan` its channel
// for EPI_BIAS.  The program sits in the kernel-argument segment, so the loop
// and its tests are wave-uniform; the loop is kept rolled on purpose: unrolled,
// the interpreter multiplies the code size of every kernel that calls it per
// value, and a small kernel then spends its time on instruction-cache misses.
__device__ __forceinline__ float apply_steps(const Epilogue &e, float v, int64_t off, int chan) {
#pragma unroll 1
    for (int s = 0; s < e.n; ++s) {
        const int op = e.s[s].op;
        if (op == EPI_BIAS) v += e.s[s].ptr[chan];
        else if (op == EPI_ADD) v += e.s[s].ptr[off];
        else if (op == EPI_RELU) v = v > 0.f ? v : 0.f;
        else if (op == EPI_GELU) v = gelu_erf(v);
        else if (op == EPI_TANH) v = tanhf(v);
        else if (op == EPI_SCALE) v *= e.s[s].scalar;
    }
    return v;
}

__device__ __forceinline__ int chan_of(const Epilogue &e, int64_t off) {
    return e.bias_c ? (int)((off / e.bias_inner) % e.bias_c) : 0;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}

// Sum over the 64 lanes on the data-parallel-primitive path of the vector ALU (no LDS traffic, unlike
// the general lane shuffle): four steps give every lane the sum of its row of 16 lanes, the four row
// sums are then read as scalars and added in row order.  Every lane gets the same value.
template <int CTRL>
__device__ __forceinline__ float dpp_lane(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
    v += dpp_lane<0xB1>(v);      // quad_perm [1,0,3,2]
    v += dpp_lane<0x4E>(v);      // quad_perm [2,3,0,1]
    v += dpp_lane<0x141>(v);     // row_half_mirror
    v += dpp_lane<0x140>(v);     // row_mirror
    return (__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0)) +
            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32)) +
            __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48)));
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = kWave / 2; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}

}  // namespace clg
