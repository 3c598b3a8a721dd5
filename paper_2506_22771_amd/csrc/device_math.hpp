// Device-side arithmetic shared by the HIP translation units of libffint8 (gfx950): wavefront reductions, the
// counter-based random word and the quantiser's code rule (Section IV: symmetric uniform quantiser; Section IV-B:
// stochastic rounding), and the exponential behind the loss derivatives (Eq. (1), Eq. (2)).  Every fp32 operation
// that decides an int8 code is a single correctly rounded IEEE operation in a fixed order: include this header only
// in files compiled with -ffp-contract=off.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ffi {

// ------------------------------------------------------------------------------------------------
// wavefront (64 lanes) reductions with DPP row operations + readlane across the four rows
// ------------------------------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}

// After this every lane of a 16-lane row holds the row's maximum.
__device__ __forceinline__ uint32_t row_max_u32(uint32_t v)
{
    v = max(v, dpp_u32<0xB1>(v));   // quad_perm [1,0,3,2]
    v = max(v, dpp_u32<0x4E>(v));   // quad_perm [2,3,0,1]
    v = max(v, dpp_u32<0x141>(v));  // row_half_mirror
    v = max(v, dpp_u32<0x140>(v));  // row_mirror
    return v;
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v)
{
    v = row_max_u32(v);
    uint32_t a = __builtin_amdgcn_readlane((int)v, 0), b = __builtin_amdgcn_readlane((int)v, 16);
    uint32_t c = __builtin_amdgcn_readlane((int)v, 32), d = __builtin_amdgcn_readlane((int)v, 48);
    return max(max(a, b), max(c, d));
}

// one random word per element: two multiply / xor-shift stages over (low index word ^ key)
__device__ __forceinline__ uint32_t sr_mix(uint32_t v)
{
    v ^= v >> 16;
    v *= 0x7FEB352Du;
    v ^= v >> 15;
    v *= 0x846CA68Bu;
    v ^= v >> 16;
    return v;
}

// STOCH: floor + Bernoulli(frac) from the counter-based word; else round-to-nearest-even.
// `word_in` is (low 32 bits of the element index) ^ key, already adjusted for the high index half.
template <bool STOCH>
__device__ __forceinline__ int quant_code(float v, float inv, uint32_t word_in)
{
    const float t = v * inv;
    int code;
    if (STOCH) {
        const float f = floorf(t);
        const float frac = t - f;
        const float u = (float)(sr_mix(word_in) >> 8) * 0x1p-24f;
        code = (int)f + (u < frac ? 1 : 0);
    } else {
        code = (int)rintf(t);
    }
    return min(max(code, -127), 127);
}

// exp(z) for z <= 0 with a fixed operation sequence (it feeds the gradient quantiser through the sigmoid)
__device__ __forceinline__ float exp_nonpos(float z)
{
    // exp(z) for z <= 0 with a fixed operation sequence (it feeds the gradient quantiser through the sigmoid)
    z = fmaxf(z, -87.0f);
    z = fminf(z, 0.0f);
    const float kf = rintf(z * 0x1.715476p+0f);
    float r = __builtin_fmaf(-kf, 0x1.62e4p-1f, z);
    r = __builtin_fmaf(-kf, 0x1.7f7d1cp-20f, r);
    float p = 0x1.a01a02p-13f;
    p = __builtin_fmaf(p, r, 0x1.6c16c2p-10f);
    p = __builtin_fmaf(p, r, 0x1.111112p-7f);
    p = __builtin_fmaf(p, r, 0x1.555556p-5f);
    p = __builtin_fmaf(p, r, 0x1.555556p-3f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    return ldexpf(p, (int)kf);
}

}  // namespace ffi
