// Device-side building blocks shared by the ECQ kernels (gfx950, wave64).
//
// Everything the method computes per element lives here so that the single-pass kernel, the
// two-pass kernels and the decode kernels produce the same bits:
//   compensate (Eq. 7), stochastic rounding (Eq. 8-9), dequantised value (Eq. 8), error
//   accumulation (Eq. 6) of Wu et al., ICML 2018, Section 4, plus Philox4x32-10 of
//   Salmon et al. (SC'11) for the rounding decision.
//
// Floating point: this file must be compiled with -ffp-contract=off and with fp32 denormals
// enabled; every binary32 operation of the method rounds on its own.  The only fused
// multiply-adds are the explicit ones inside the division routine, where they are the
// standard way to obtain a correctly rounded quotient.
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
        // a ^ b ^ c in one instruction: the three-input bitwise operation with truth table 0x96.
        const uint32_t n0 = (uint32_t)__builtin_amdgcn_bitop3_b32((int)(uint32_t)(p1 >> 32), (int)c1, (int)k0, 0x96);
        const uint32_t n2 = (uint32_t)__builtin_amdgcn_bitop3_b32((int)(uint32_t)(p0 >> 32), (int)c3, (int)k1, 0x96);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    return U4{c0, c1, c2, c3};
}

// Eq. (7).
__device__ __forceinline__ float compensate(float g, float alpha, float h)
{
    const float ah = alpha * h;
    return g + ah;
}

// Eq. (6).
__device__ __forceinline__ float error_update(float beta, float h, float g, float gt)
{
    const float bh = beta * h;
    const float d = g - gt;
    return bh + d;
}

// ---- correctly rounded |v| / scale with the divisor-only work hoisted out -----------------
//
// Every element of a bucket is divided by the same norm, and 0 <= |v| <= norm.  The quotient
// is produced by the classic reciprocal / two-residual-corrections scheme (the one the
// compiler itself emits for a correctly rounded binary32 division once operands are in a
// range where no rescaling is needed): the reciprocal and its Newton step are computed once
// per bucket, each element costs one multiply and four fused multiply-adds.  The scheme is
// exact only while quotient and residuals stay normal, so operands outside a safe window
// (divisor outside [2^-100, 2^100], or 0 < |v| < max(1, divisor) * 2^-100) take the plain
// division instead.  With SCALE24 the quotient comes out multiplied by 2^24 (an exact
// scaling folded into the per-bucket constants).
struct Ratio {
    float d;        // divisor: the norm, or 1 when the norm is 0
    float neg_d;    // -d            (* 2^-24 with SCALE24)
    float y;        // ~ 1/d         (* 2^24 with SCALE24); 0 when the norm is 0
    float tiny;     // numerators in (0, tiny) use the plain division
    bool fast;      // divisor inside the safe window
};

template <bool SCALE24>
__device__ __forceinline__ Ratio make_ratio(float norm)
{
    Ratio rt;
    rt.d = norm > 0.0f ? norm : 1.0f;
    rt.fast = (rt.d >= 0x1p-100f) && (rt.d <= 0x1p100f);
    float r = __builtin_amdgcn_rcpf(rt.d);
    const float e = __builtin_fmaf(-rt.d, r, 1.0f);
    r = __builtin_fmaf(e, r, r);
    rt.y = SCALE24 ? r * 0x1p24f : r;
    rt.neg_d = SCALE24 ? -rt.d * 0x1p-24f : -rt.d;
    rt.tiny = (rt.d > 1.0f ? rt.d : 1.0f) * 0x1p-100f;
    // ||v|| = 0: every level is 0, whatever the elements are (with the l2 norm the squares of
    // tiny elements can all round to 0).  A zero reciprocal makes every quotient 0 on the
    // fast route, and the smallest denormal as `tiny` keeps every numerator on it.
    if (!(norm > 0.0f)) {
        rt.y = 0.0f;
        rt.tiny = __uint_as_float(1u);
    }
    return rt;
}

template <bool SCALE24>
__device__ __forceinline__ float ratio(float av, const Ratio &rt)
{
    float q = av * rt.y;
    float e = __builtin_fmaf(rt.neg_d, q, av);
    q = __builtin_fmaf(e, rt.y, q);
    e = __builtin_fmaf(rt.neg_d, q, av);
    q = __builtin_fmaf(e, rt.y, q);
    // (bits - 1) as unsigned sends 0 to the top of the range: true only for 0 < av < tiny.
    const bool rare = !rt.fast || (__float_as_uint(av) - 1u) < (__float_as_uint(rt.tiny) - 1u);
    if (__builtin_expect(rare, 0)) {
        q = av / rt.d;
        if (SCALE24) q = q * 0x1p24f;
    }
    return q;
}

// ---- Eq. (8)-(9) for one element ------------------------------------------------------------

struct Quantized {
    uint32_t code;  // level + s, in [0, 2s]
    float gt;       // dequantised value with its sign (Eq. 8)
};

// s = 1 (ternary, 2-bit codes).  With x = |v|/norm in [0,1] the level is 1 iff u < x: for
// x < 1 the lower grid point is 0 and x itself is the round-up probability, and x = 1 (the
// element that attains the norm) gives level 1 for every u < 1.  The comparison is done on
// both sides scaled by 2^24: k < x * 2^24 with k = word >> 8.
__device__ __forceinline__ Quantized quantize_ternary(float v, float norm, const Ratio &rt, uint32_t word)
{
    const float x24 = ratio<true>(__builtin_fabsf(v), rt);
    const bool up = (float)(word >> 8) < x24;
    const uint32_t sign = __float_as_uint(v) & 0x80000000u;
    Quantized out;
    out.gt = up ? __uint_as_float(__float_as_uint(norm) | sign) : 0.0f;
    out.code = up ? (sign ? 0u : 2u) : 1u;
    return out;
}

// General s.  sxi_tab[c] = +-fl(|c - s|/s), indexed by the code c = level + s, so the sign of
// the dequantised value comes with the table entry.  x >= 0, so truncation is floor and
// x - floor(x) is exact.  With the l_inf norm the quotient never exceeds 1; the computed l2
// norm can fall below |v_i| when fl(v_i^2) is denormal (a quotient up to about 1.12), so the
// level is capped at s, the end of the grid of Eq. (8).
__device__ __forceinline__ Quantized quantize_levels(float v, float norm, const Ratio &rt, int s, float sf,
                                                     const float *sxi_tab, uint32_t word)
{
    const float a = ratio<false>(__builtin_fabsf(v), rt);
    const float x = a * sf;
    const float frac = __builtin_amdgcn_fractf(x);
    const float u = (float)(word >> 8) * 0x1p-24f;
    int m = (int)x + ((u < frac) ? 1 : 0);
    m = m < s ? m : s;
    const int smask = (int)__float_as_uint(v) >> 31;          // 0, or -1 for negative v
    const int c = s + ((m ^ smask) - smask);                   // s - m for negative v, s + m otherwise
    Quantized out;
    out.gt = norm * sxi_tab[c];
    out.code = (uint32_t)c;
    return out;
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

// ---- wave-level synchronisation and prefix sums (entropy coders) ------------------------------

// Orders a wave's LDS writes before its later LDS reads of other lanes' data.  Only that wave
// touches the memory in question, and a wave's LDS operations complete in order.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Inclusive prefix sum over the 64 lanes of a wave: four shifts inside each row of 16 lanes,
// then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3.  Lanes without
// a source add 0.
__device__ __forceinline__ unsigned int wave_inclusive_scan(unsigned int x)
{
    x += (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xF, 0xF, false);   // row_shr:1
    x += (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xF, 0xF, false);   // row_shr:2
    x += (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xF, 0xF, false);   // row_shr:4
    x += (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xF, 0xF, false);   // row_shr:8
    x += (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xA, 0xF, false);   // row_bcast:15
    x += (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xC, 0xF, false);   // row_bcast:31
    return x;
}

// ---- l2 norm: sum of squares over a balanced binary tree by element index --------------------
//
// a + b == b + a in IEEE arithmetic, so a butterfly in which both partners add leaves the same
// value in both lanes, and the exchange order (distance 1, 2, 4, ... lanes) is exactly the
// index tree because a lane owns 4 consecutive elements and lanes own consecutive groups.

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x)
{
    return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(x)));
}

// Tree sum of the squares of a lane's 4 consecutive elements.
__device__ __forceinline__ float sum_squares4(const float (&v)[4])
{
    const float s0 = v[0] * v[0], s1 = v[1] * v[1], s2 = v[2] * v[2], s3 = v[3] * v[3];
    const float lo = s0 + s1;
    const float hi = s2 + s3;
    return lo + hi;
}

// Tree sum over aligned groups of `lanes` lanes (a power of two, 1..64), result in every lane.
__device__ __forceinline__ float group_sum_tree(float x, int lanes)
{
    if (lanes >= 2) x = x + dpp_f32<0xB1>(x);
    if (lanes >= 4) x = x + dpp_f32<0x4E>(x);
    if (lanes >= 8) x = x + dpp_f32<0x141>(x);
    if (lanes >= 16) x = x + dpp_f32<0x140>(x);
    if (lanes >= 32) x = x + __shfl_xor(x, 16, 64);
    if (lanes >= 64) x = x + __shfl_xor(x, 32, 64);
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

// Store the low NBYTES bytes of `bits` at dst (any address) in as few pieces as possible: a
// dword, a short and a byte where needed.  Global stores need no natural alignment here.
template <int NBYTES>
__device__ __forceinline__ void store_code_bytes_whole(uint8_t *dst, uint64_t bits)
{
    static_assert(NBYTES >= 1 && NBYTES <= 8, "at most one 64-bit word");
    int at = 0;
    if constexpr (NBYTES >= 4) {
        const uint32_t w = (uint32_t)bits;
        __builtin_memcpy(dst, &w, 4);
        at = 4;
    }
    if constexpr ((NBYTES & 3) >= 2) {
        const uint16_t w = (uint16_t)(bits >> (8 * at));
        __builtin_memcpy(dst + at, &w, 2);
        at += 2;
    }
    if constexpr (NBYTES == 8) {
        const uint32_t w = (uint32_t)(bits >> 32);
        __builtin_memcpy(dst + 4, &w, 4);
    } else if constexpr ((NBYTES & 1) == 1) {
        dst[at] = (uint8_t)(bits >> (8 * at));
    }
}

// ---- reading packed codes ------------------------------------------------------------------

// The R bytes that hold the codes of the 8 elements starting at `elem` (a multiple of 8).
template <int R>
__device__ __forceinline__ uint64_t load_code_group(const uint8_t *__restrict__ crow,
                                                    int64_t row_bytes, int64_t elem)
{
    const int64_t byte_off = (elem >> 3) * R;
    uint64_t bits = 0;
#pragma unroll
    for (int b = 0; b < R; ++b)
        if (byte_off + b < row_bytes) bits |= (uint64_t)crow[byte_off + b] << (8 * b);
    return bits;
}

// The codes of the 16 consecutive elements a lane owns: 2*R bytes starting at `src`, which is
// 4-byte aligned for even R and 2-byte aligned for odd R.  No bounds checks.
template <int R>
struct Codes16 {
    static constexpr int kWords = (R + 1) / 2;
    uint32_t w[kWords];
    // NT: non-temporal loads, for codes that are read once and should not take room in (or evict
    // dirty lines from) the last-level cache.
    template <bool NT = false>
    __device__ __forceinline__ void load(const uint8_t *__restrict__ src)
    {
        if constexpr ((R & 1) == 0) {
#pragma unroll
            for (int i = 0; i < R / 2; ++i) {
                const uint32_t *at = reinterpret_cast<const uint32_t *>(src) + i;
                w[i] = NT ? __builtin_nontemporal_load(at) : *at;
            }
        } else {
            // 2*R bytes at a 2-byte aligned address: whole dwords (global loads need no natural
            // alignment here), then one short.
            typedef uint32_t u32_unaligned __attribute__((aligned(2)));
            typedef uint16_t u16_aligned __attribute__((aligned(2)));
#pragma unroll
            for (int i = 0; i < kWords - 1; ++i) {
                const u32_unaligned *at = reinterpret_cast<const u32_unaligned *>(src + 4 * i);
                w[i] = NT ? __builtin_nontemporal_load(at) : *at;
            }
            const u16_aligned *last = reinterpret_cast<const u16_aligned *>(src + 4 * (kWords - 1));
            w[kWords - 1] = NT ? __builtin_nontemporal_load(last) : *last;
        }
    }
    // The same for a lane at the ragged end of a row: bytes at or beyond row_bytes read as 0.
    // `elem` = index of the lane's first element (a multiple of 16).
    __device__ __forceinline__ void load_guarded(const uint8_t *__restrict__ crow, int64_t row_bytes, int64_t elem)
    {
        const uint64_t g0 = elem < 0 ? 0ull : load_code_group<R>(crow, row_bytes, elem);
        const uint64_t g1 = load_code_group<R>(crow, row_bytes, elem + 8);
        // 16*R bits: g0 holds the first 8*R, g1 the next 8*R.
        uint64_t lo = g0, hi = 0;
        if constexpr (R == 8) hi = g1;
        else {
            lo |= g1 << (8 * R);
            hi = g1 >> (64 - 8 * R);
        }
        w[0] = (uint32_t)lo;
        if constexpr (kWords > 1) w[1] = (uint32_t)(lo >> 32);
        if constexpr (kWords > 2) w[2] = (uint32_t)hi;
        if constexpr (kWords > 3) w[3] = (uint32_t)(hi >> 32);
    }
    // Code of element e (compile-time constant after unrolling).
    __device__ __forceinline__ uint32_t code(int e) const
    {
        const int bit = R * e, i = bit >> 5, sh = bit & 31;
        uint32_t c = w[i] >> sh;
        if (sh + R > 32) c |= w[i + 1] << (32 - sh);
        return c & ((1u << R) - 1u);
    }
};

}  // namespace ecq
