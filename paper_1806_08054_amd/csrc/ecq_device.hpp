// Device-side building blocks shared by the ECQ kernels (gfx950, wave64).
//
// Everything the method computes per element lives here so that the single-pass kernel, the
// two-pass kernels and the decode kernels produce the same bits:
//   compensate (Eq. 7), stochastic rounding (Eq. 8-9), dequantised value (Eq. 8), error
//   accumulation (Eq. 6) of Wu et al., ICML 2018, Section 4, plus Philox4x32-10 of
//   Salmon et al. (SC'11) for the rounding decision.
//
// Floating point: this file must be compiled with -ffp-contract=off; every binary32 operation
// below is meant to round on its own.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ecq {

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

struct U4 {
    uint32_t x, y, z, w;
};

// One Philox4x32-10 block.  The key schedule and every term that only depends on (c1, c2,
// c3, k0, k1) are wave-uniform at the call sites and end up on the scalar unit.
__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)kPhiloxM1 * (uint64_t)c2;
        const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    return U4{c0, c1, c2, c3};
}

// Parameters of the rounding that are uniform over a launch.
struct Levels {
    int s;        // non-zero levels
    float sf;     // (float)s
};

// Eq. (7).
__device__ __forceinline__ float compensate(float g, float alpha, float h)
{
    const float ah = alpha * h;
    return g + ah;
}

// Eq. (8)-(9): magnitude level m in [0, s] of |v| on the grid scale*{0,1/s,...,1}; `scale`
// must be > 0.  u = (word >> 8) * 2^-24 is exact, so is frac; the level moves up iff u < frac.
__device__ __forceinline__ int round_level(float v, float scale, const Levels &lv, uint32_t word)
{
    const float a = __builtin_fabsf(v) / scale;
    const float x = a * lv.sf;
    const float l = __builtin_floorf(x);
    const float frac = x - l;
    const float u = (float)(word >> 8) * 0x1p-24f;
    int m = (int)l + ((u < frac) ? 1 : 0);
    return m < lv.s ? m : lv.s;
}

// Eq. (8): scale * fl(m/s) with the sign of v when m > 0.  `xi` is fl(m/s).
// m > 0 implies v != 0, so "v < 0" and "sign bit of v" agree whenever the sign is applied.
__device__ __forceinline__ float dequant_signed(float scale, float xi, int m, float v)
{
    const float gt = scale * xi;
    const uint32_t sign = (m > 0) ? (__float_as_uint(v) & 0x80000000u) : 0u;
    return __uint_as_float(__float_as_uint(gt) ^ sign);
}

// Eq. (6).
__device__ __forceinline__ float error_update(float beta, float h, float g, float gt)
{
    const float bh = beta * h;
    const float d = g - gt;
    return bh + d;
}

// ---- cross-lane helpers ---------------------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, CTRL, 0xF, 0xF, false);
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Max over each row of 16 lanes, result in every lane of the row.  Operates on the bit
// patterns of non-negative floats, for which unsigned order equals float order.
__device__ __forceinline__ uint32_t row16_max(uint32_t x)
{
    x = umax(x, dpp_u32<0xB1>(x));    // quad_perm [1,0,3,2]
    x = umax(x, dpp_u32<0x4E>(x));    // quad_perm [2,3,0,1]
    x = umax(x, dpp_u32<0x141>(x));   // row_half_mirror
    x = umax(x, dpp_u32<0x140>(x));   // row_mirror
    return x;
}

// Max over the whole wave, returned as a wave-uniform value.
__device__ __forceinline__ uint32_t wave_max_uniform(uint32_t x)
{
    x = row16_max(x);
    const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)x, 0);
    const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)x, 16);
    const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)x, 32);
    const uint32_t d = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
    return umax(umax(a, b), umax(c, d));
}

// Max over aligned groups of `lanes` lanes (a power of two, 1..64), result in every lane.
__device__ __forceinline__ uint32_t group_max(uint32_t x, int lanes)
{
    if (lanes >= 2) x = umax(x, dpp_u32<0xB1>(x));
    if (lanes >= 4) x = umax(x, dpp_u32<0x4E>(x));
    if (lanes >= 8) x = umax(x, dpp_u32<0x141>(x));
    if (lanes >= 16) x = umax(x, dpp_u32<0x140>(x));
    if (lanes >= 32) x = umax(x, (uint32_t)__shfl_xor((int)x, 16, 64));
    if (lanes >= 64) x = umax(x, (uint32_t)__shfl_xor((int)x, 32, 64));
    return x;
}

// ---- code packing -----------------------------------------------------------------------

// Store the low `nbytes` bytes of `bits` at dst, skipping bytes at or beyond `limit` bytes
// from dst (the end of the encoded row).
__device__ __forceinline__ void store_code_bytes(uint8_t *dst, uint64_t bits, int nbytes,
                                                 int64_t limit)
{
#pragma unroll
    for (int b = 0; b < 8; ++b)
        if (b < nbytes && (int64_t)b < limit) dst[b] = (uint8_t)(bits >> (8 * b));
}

}  // namespace ecq
