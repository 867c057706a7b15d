// HIP kernels of the ECQ-SGD codec for gfx950 (MI355X), wave64.
//
// Single pass ("bucket in registers"): every bucket of b elements is owned by a team of
// lanes that loads its share of g and h once, keeps it in VGPRs across the max-abs
// reduction (DPP inside a wave, LDS across waves), then rounds, packs, stores the codes and
// writes h back: 12 + r/8 + 4/b bytes of HBM traffic per element, the minimum for
//   v = g + alpha*h (Eq. 7), Q_s(v) (Eq. 8-9), r-bit encoding, h <- beta*h + (g - g~) (Eq. 6)
// of Wu et al., ICML 2018, Section 4.  Buckets that do not fit a team's registers, or whose
// size is not a supported shape, take a two-pass route (norm kernel, then quantise kernel).
//
// A lane always owns 4 consecutive elements starting at a multiple of 4, which is exactly one
// Philox4x32-10 block (counter low word = element index >> 2), so no random word is wasted.
#include "ecq_device.hpp"
#include "ecq_internal.hpp"

namespace ecq {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f2 __attribute__((ext_vector_type(2)));

// ---------------------------------------------------------------------------------------------
// Per-lane work on 4 consecutive elements.
// ---------------------------------------------------------------------------------------------

// g and h are streamed exactly once per call and h is written back once, so all three use
// non-temporal accesses: on MI355X that alone is worth ~8 % of bandwidth for this traffic mix.
//
// Loads elements [off, off+4) of a row segment of `len` elements; missing ones read as 0.
__device__ __forceinline__ void load4(const float *__restrict__ row, int64_t off, int64_t len,
                                      float (&x)[4])
{
    if (off + 4 <= len) {
        const f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(row + off));
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = (off + e < len) ? row[off + e] : 0.0f;
    }
}

// The same without bounds checks.
__device__ __forceinline__ void load4_full(const float *__restrict__ src, float (&x)[4])
{
    const f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(src));
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}

__device__ __forceinline__ void store4_full(float *__restrict__ dst, const float (&x)[4])
{
    f4 t;
    t.x = x[0]; t.y = x[1]; t.z = x[2]; t.w = x[3];
    __builtin_nontemporal_store(t, reinterpret_cast<f4 *>(dst));
}

__device__ __forceinline__ void store4(float *__restrict__ row, int64_t off, int64_t len,
                                       const float (&x)[4])
{
    if (off + 4 <= len) {
        f4 t;
        t.x = x[0]; t.y = x[1]; t.z = x[2]; t.w = x[3];
        __builtin_nontemporal_store(t, reinterpret_cast<f4 *>(row + off));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (off + e < len) row[off + e] = x[e];
    }
}

// v = g + alpha*h for a lane's 4 elements (Eq. 7); returns the bit pattern of max |v|
// (0 for missing elements, which were loaded as zeros).
__device__ __forceinline__ uint32_t compensate4(const float (&g)[4], const float (&h)[4], float alpha,
                                               float (&v)[4])
{
    uint32_t m = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[e] = compensate(g[e], alpha, h[e]);
        // max of non-negative floats; |v| is an operand modifier, so one instruction per element
        m = __float_as_uint(__builtin_fmaxf(__uint_as_float(m), __builtin_fabsf(v[e])));
    }
    return m;
}

// Per-bucket constants of the rounding step.
template <int R>
struct Rounder {
    float norm;
    Ratio rt;
    int s;
    float sf;
    const float *xi_tab;
    __device__ __forceinline__ Rounder(float norm_, int s_, const float *xi_tab_)
        : norm(norm_), rt(make_ratio<R == 2>(norm_)), s(s_), sf((float)s_), xi_tab(xi_tab_) {}
    __device__ __forceinline__ Quantized operator()(float v, uint32_t word) const
    {
        if constexpr (R == 2) return quantize_ternary(v, norm, rt, word);      // r = 2 <=> s = 1
        else return quantize_levels(v, norm, rt, s, sf, xi_tab, word);
    }
};

// Rounds, encodes and (optionally) accumulates the error for a lane's 4 elements.
//   valid : how many of the 4 exist (0..4); codes of missing elements are zero bits.
// Returns the 4*R encoded bits, element e in bits [e*R, (e+1)*R).
constexpr int kChunksPerWave = 2;

template <int R, bool UPDATE>
__device__ __forceinline__ uint32_t quantize4(const float (&g)[4], float (&h)[4], const float (&v)[4],
                                              int valid, const Rounder<R> &rounder, float beta,
                                              const U4 &words)
{
    const uint32_t w[4] = {words.x, words.y, words.z, words.w};
    uint32_t bits = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const Quantized qz = rounder(v[e], w[e]);
        bits |= (e < valid) ? (qz.code << (R * e)) : 0u;
        if (UPDATE) h[e] = error_update(beta, h[e], g[e], qz.gt);
    }
    return bits;
}

// Stores a lane's 4*R code bits.  `elem` = index of the lane's first element in the row (a
// multiple of 4; a multiple of 8 on even lanes).  For odd R two neighbouring lanes share
// whole bytes, so the even lane stores both lanes' bits.  Must be called by all lanes.
template <int R>
__device__ __forceinline__ void store_codes(uint8_t *__restrict__ crow, int64_t row_bytes,
                                            int64_t elem, int valid, uint32_t bits, int lane)
{
    if constexpr ((R & 1) == 0) {
        constexpr int NB = R / 2;
        const int64_t byte_off = (elem >> 2) * NB;
        if (valid == 4) {
            uint8_t *dst = crow + byte_off;
            if constexpr (NB == 1) {
                *dst = (uint8_t)bits;
            } else if constexpr (NB == 2) {
                *reinterpret_cast<uint16_t *>(dst) = (uint16_t)bits;
            } else if constexpr (NB == 4) {
                *reinterpret_cast<uint32_t *>(dst) = bits;
            } else {
                store_code_bytes_whole<NB>(dst, bits);
            }
        } else if (valid > 0) {
            store_code_bytes(crow + byte_off, bits, NB, row_bytes - byte_off);
        }
    } else {
        const uint32_t next = dpp_u32<0xF5>(bits);            // quad_perm [1,1,3,3]
        if ((lane & 1) == 0 && valid > 0) {
            const uint64_t both = (uint64_t)bits | ((uint64_t)next << (4 * R));
            const int64_t byte_off = (elem >> 3) * R;
            // Bits of elements past the row's end are zero, so whole bytes inside the row are
            // written as they are.
            if (byte_off + R <= row_bytes) store_code_bytes_whole<R>(crow + byte_off, both);
            else store_code_bytes(crow + byte_off, both, R, row_bytes - byte_off);
        }
    }
}

// Signed table of the rounding step, indexed by the code c = level + s: +-fl(|level|/s).
__device__ __forceinline__ void fill_sxi_table(float *sxi_tab, int s)
{
    for (int c = threadIdx.x; c <= 2 * s; c += blockDim.x) {
        const int q = c - s;
        const float xi = (float)(q < 0 ? -q : q) / (float)s;
        sxi_tab[c] = q < 0 ? -xi : xi;
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// Single pass, buckets of 256 elements or more: a team of W waves per bucket, J float4 per lane.
// ---------------------------------------------------------------------------------------------
// The work of one block of k_fused_team.
template <int R, int J, bool UPDATE, bool FULL>
__device__ __forceinline__ void fused_team_block(const Args &a, const int w_shift, const uint32_t p,
                                                 const uint32_t row_block, const float *xi_tab, uint32_t *wave_norm)
{

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int W = 1 << w_shift;
    const int team = wave >> w_shift;
    const int wit = wave & (W - 1);
    const int teams = blockDim.x >> (6 + w_shift);
    const int64_t k = (int64_t)row_block * teams + team;
    // FULL: every team of the block owns a complete bucket of exactly W*J*256 elements, so no
    // load, store or code needs a bounds check.
    const bool active = FULL || k < a.nb;
    const int64_t e0 = active ? k * (int64_t)a.bucket : 0;
    const int64_t rest = a.n - e0;
    const int len = FULL ? a.bucket : (active ? (int)(rest < a.bucket ? rest : (int64_t)a.bucket) : 0);

    const float *__restrict__ grow = a.g + (int64_t)p * a.gh_stride + e0;
    float *__restrict__ hrow = a.h + (int64_t)p * a.gh_stride + e0;

    // v = g + alpha*h is kept in registers between the two phases while it fits (J <= 4);
    // with 8 float4 per lane it is recomputed instead.
    constexpr bool kKeepV = J <= 4;
    float g[J][4], h[J][4], v[kKeepV ? J : 1][4];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int off = ((wit * J + j) * 64 + lane) * 4;
        if constexpr (FULL) {
            load4_full(grow + off, g[j]);
            load4_full(hrow + off, h[j]);
        } else {
            load4(grow, off, len, g[j]);
            load4(hrow, off, len, h[j]);
        }
    }
    uint32_t mx = 0;
#pragma unroll
    for (int j = 0; j < J; ++j) mx = umax(mx, compensate4(g[j], h[j], a.alpha, v[kKeepV ? j : 0]));

    float scale;
    if (!a.norm_l2) {
        uint32_t norm = wave_max_uniform(mx);
        if (W > 1) {
            if (lane == 0) wave_norm[wave] = norm;
            __syncthreads();
            for (int t = 0; t < W; ++t) norm = umax(norm, wave_norm[(team << w_shift) + t]);
        }
        scale = __uint_as_float(norm);
    } else {
        // Tree by index: lanes of a 256-element run, then the wave's J runs, then the team's waves.
        float part[J];
#pragma unroll
        for (int j = 0; j < J; ++j) {
            if constexpr (!kKeepV) compensate4(g[j], h[j], a.alpha, v[0]);
            part[j] = group_sum_tree(sum_squares4(v[kKeepV ? j : 0]), 64);
        }
#pragma unroll
        for (int w = 1; w < J; w *= 2)
#pragma unroll
            for (int j = 0; j + w < J; j += 2 * w) part[j] = part[j] + part[j + w];
        float total = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane((int)__float_as_uint(part[0])));
        if (W > 1) {
            if (lane == 0) wave_norm[wave] = __float_as_uint(total);
            __syncthreads();
            float t[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) t[i] = i < W ? __uint_as_float(wave_norm[(team << w_shift) + i]) : 0.0f;
#pragma unroll
            for (int w = 1; w < 16; w *= 2)
#pragma unroll
                for (int i = 0; i + w < 16; i += 2 * w) t[i] = t[i] + t[i + w];
            total = t[0];
        }
        scale = __builtin_sqrtf(total);
    }
    const Rounder<R> rounder(scale, a.s, xi_tab);

    uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int chunk = (wit * J + j) * 256;
        if (!FULL && chunk >= len) continue;                   // wave-uniform
        const int off = chunk + lane * 4;
        const int64_t elem = e0 + off;
        int valid = 4;
        if constexpr (!FULL) {
            valid = len - off;
            valid = valid < 0 ? 0 : (valid > 4 ? 4 : valid);
        }
        const U4 words = philox4x32_10((uint32_t)(elem >> 2), p, a.step_lo, a.step_hi, a.key0, a.key1);
        if constexpr (!kKeepV) compensate4(g[j], h[j], a.alpha, v[0]);
        const uint32_t bits =
            quantize4<R, UPDATE>(g[j], h[j], v[kKeepV ? j : 0], valid, rounder, a.beta, words);
        store_codes<R>(crow, a.row_bytes, elem, valid, bits, lane);
        if constexpr (UPDATE) {
            if constexpr (FULL) store4_full(hrow + off, h[j]);
            else store4(hrow, off, len, h[j]);
        }
    }
    if (active && wit == 0 && lane == 0) a.scales[(int64_t)p * a.scale_stride + k] = scale;
}

template <int R, int J, bool UPDATE>
__global__ void __launch_bounds__(1024) k_fused_team(const Args a, const int w_shift, const int64_t stripe,
                                                     const uint32_t blocks_per_row, const uint32_t worker0,
                                                     const uint32_t workers)
{
    __shared__ float xi_tab[256];
    __shared__ uint32_t wave_norm[16];
    // Block -> (worker row, block of the row).  Workgroups go to the chip's 8 XCDs round-robin
    // by id.  With stripe > 0 the launch is one-dimensional and XCD x takes the x-th eighth of
    // all blocks in address order, so each XCD streams through its own contiguous region and
    // stays compact in memory however far the XCDs drift apart during a long launch.
    // A launch covers workers worker0 .. worker0 + workers - 1.
    uint32_t row_block = blockIdx.x, p = worker0 + blockIdx.y;
    if (stripe > 0) {
        const int64_t id = (int64_t)(blockIdx.x & 7u) * stripe + (blockIdx.x >> 3);
        if (id >= (int64_t)blocks_per_row * workers) return;    // whole block
        const uint32_t row = (uint32_t)(id / blocks_per_row);
        p = worker0 + row;
        row_block = (uint32_t)(id - (int64_t)row * blocks_per_row);
    }
    if constexpr (R != 2) fill_sxi_table(xi_tab, a.s);
    // Uniform over the block: all of its buckets are complete and exactly fill their teams.
    const int teams_per_block = blockDim.x >> (6 + w_shift);
    const bool full = a.bucket == (J * 256 << w_shift) &&
                      (int64_t)(row_block + 1) * teams_per_block * a.bucket <= a.n;
    // The check-free path pays where arithmetic is the limit (quantising without the update of
    // h: +11 %); with the update the kernel waits for memory either way and the smaller code wins.
    if constexpr (!UPDATE) {
        if (full) {
            fused_team_block<R, J, UPDATE, true>(a, w_shift, p, row_block, xi_tab, wave_norm);
            return;
        }
    }
    fused_team_block<R, J, UPDATE, false>(a, w_shift, p, row_block, xi_tab, wave_norm);
}

// ---------------------------------------------------------------------------------------------
// A lane owns one float4 of each of two consecutive chunks of its wave (all loads are issued
// before any is used).  The 64 lanes of a wave form slots of `slot_lanes` lanes (a power of two)
// and a slot covers `span` consecutive elements with its first span/4 lanes:
//   single pass, buckets of 8..248 elements: a slot is one bucket (span = bucket); slot_lanes is
//       the bucket's lane count rounded up to a power of two, so the norm is a max (or the
//       index tree of squares, the idle lanes standing for the padding zeros) over the slot;
//   second pass of the two-pass route: one slot of 64 lanes, span 256, norms read from scales.
// A chunk is what the wave's slots cover together: (64 / slot_lanes) * span elements.
// ---------------------------------------------------------------------------------------------
template <int R, bool UPDATE>
__global__ void __launch_bounds__(256) k_quant_chunk(const Args a, const int slot_lanes, const int span,
                                                     const int read_norms)
{
    __shared__ float xi_tab[256];
    if constexpr (R != 2) fill_sxi_table(xi_tab, a.s);

    constexpr int J = kChunksPerWave;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int slots = 64 / slot_lanes;                         // per wave
    const int64_t chunk_elems = (int64_t)slots * span;
    const int64_t chunk0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + wave) * J;
    const uint32_t p = blockIdx.y;
    if (chunk0 * chunk_elems >= a.n) return;                   // wave-uniform

    const int slot = lane / slot_lanes, in_slot = lane & (slot_lanes - 1);
    const bool used = in_slot * 4 < span;                      // (idle lanes read nothing and store nothing)
    const float *__restrict__ grow = a.g + (int64_t)p * a.gh_stride;
    float *__restrict__ hrow = a.h + (int64_t)p * a.gh_stride;
    float g[J][4], h[J][4], v[J][4];
    uint32_t mx[J];
    int64_t elem[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {                              // all loads first (nothing is read beyond n)
        elem[j] = used ? ((chunk0 + j) * slots + slot) * span + in_slot * 4 : a.n;
        load4(grow, elem[j], a.n, g[j]);
        load4(hrow, elem[j], a.n, h[j]);
    }
#pragma unroll
    for (int j = 0; j < J; ++j) mx[j] = compensate4(g[j], h[j], a.alpha, v[j]);
#pragma unroll
    for (int j = 0; j < J; ++j) {
        if ((chunk0 + j) * chunk_elems >= a.n) break;          // wave-uniform
        const int64_t rest = a.n - elem[j];
        const int valid = rest <= 0 ? 0 : (rest > 4 ? 4 : (int)rest);
        float scale;
        if (!read_norms) {
            scale = a.norm_l2 ? __builtin_sqrtf(group_sum_tree(sum_squares4(v[j]), slot_lanes))
                              : __uint_as_float(group_max(mx[j], slot_lanes));
            if (valid > 0 && in_slot == 0) a.scales[(int64_t)p * a.scale_stride + ((chunk0 + j) * slots + slot)] = scale;
        } else {
            scale = valid > 0 ? a.scales[(int64_t)p * a.scale_stride + elem[j] / a.bucket] : 0.0f;
        }
        const Rounder<R> rounder(scale, a.s, xi_tab);
        const U4 words = philox4x32_10((uint32_t)(elem[j] >> 2), p, a.step_lo, a.step_hi, a.key0, a.key1);
        const uint32_t bits = quantize4<R, UPDATE>(g[j], h[j], v[j], valid, rounder, a.beta, words);
        store_codes<R>(a.codes + (int64_t)p * a.code_stride, a.row_bytes, elem[j], valid, bits, lane);
        if (UPDATE) store4(hrow, elem[j], a.n, h[j]);
    }
}

// First pass of the two-pass route: scales[p][k] = max |g + alpha*h| over bucket k, taken with
// an unsigned atomic max on the bit patterns (order-preserving for non-negative floats).
// scales must hold zeros on entry.  Atomic operations on one address are served one at a time,
// so both kernels below reduce as far as they can before they issue one.
//
// Buckets shorter than 256 elements (and not a power of two): a lane owns one float4, which
// never straddles buckets (they are multiples of 8 elements).  The lanes of a bucket are
// neighbours, so a segmented prefix maximum over the wave (six shuffle steps on the pair
// (bucket, max)) leaves each bucket's maximum in its last lane, and only that lane sends it:
// at most two atomic operations per bucket and wave boundary.
__global__ void __launch_bounds__(256) k_bucket_norm_small(const Args a)
{
    const int lane = threadIdx.x & 63;
    const int64_t elem = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    const uint32_t p = blockIdx.y;
    float g[4], h[4];
    load4(a.g + (int64_t)p * a.gh_stride, elem, a.n, g);
    load4(a.h + (int64_t)p * a.gh_stride, elem, a.n, h);
    float v[4];
    uint32_t mx = compensate4(g, h, a.alpha, v);
    const bool exists = elem < a.n;
    // Element indices grow with the lane, so lane 0 holds the wave's lowest bucket, and if lane 0
    // is past the end of the row the whole wave is.
    const int64_t wave_elem = elem - (int64_t)lane * 4;
    if (wave_elem >= a.n) return;                              // wave-uniform
    const int64_t k_lead = wave_elem / a.bucket;
    // Bucket relative to the wave's first one; lanes past the end get one no bucket has.
    const int k = exists ? (int)(elem / a.bucket - k_lead) : 0x7FFFFFFF;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int below_k = __shfl_up(k, d, 64);
        const uint32_t below_mx = (uint32_t)__shfl_up((int)mx, d, 64);
        if (lane >= d && below_k == k) mx = umax(mx, below_mx);
    }
    const int next_k = __shfl_down(k, 1, 64);
    const bool last_of_bucket = lane == 63 || next_k != k;
    if (exists && last_of_bucket)
        atomicMax(reinterpret_cast<uint32_t *>(a.scales + (int64_t)p * a.scale_stride) + (k_lead + k), mx);
}

// Buckets longer than 32768 elements, up to the whole row: a bucket is cut into `parts` pieces
// of `part_len` elements (a multiple of 1024); a block walks one piece, 2048 elements at a
// time, and sends one atomic max for it.  blockIdx.x = bucket * parts + part.
__global__ void __launch_bounds__(256) k_bucket_norm_large(const Args a, const int parts, const int64_t part_len)
{
    __shared__ uint32_t wave_norm[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t p = blockIdx.y;
    const int64_t k = blockIdx.x / parts;
    const int part = (int)(blockIdx.x - k * parts);
    const int64_t bucket_begin = k * (int64_t)a.bucket;
    int64_t bucket_end = bucket_begin + a.bucket;
    if (bucket_end > a.n) bucket_end = a.n;
    const int64_t begin = bucket_begin + (int64_t)part * part_len;
    int64_t end = begin + part_len;
    if (end > bucket_end) end = bucket_end;
    const float *__restrict__ grow = a.g + (int64_t)p * a.gh_stride;
    const float *__restrict__ hrow = a.h + (int64_t)p * a.gh_stride;
    uint32_t mx = 0;
    // `end` is a multiple of 4 or the row's end, so load4's own guard (elements >= end read as
    // 0, and |0| never raises a maximum) is all a ragged piece needs.
    for (int64_t at = begin + (int64_t)threadIdx.x * 4; at < end; at += 2048) {
        float g0[4], h0[4], g1[4], h1[4], v[4];
        load4(grow, at, end, g0);
        load4(hrow, at, end, h0);
        load4(grow, at + 1024, end, g1);
        load4(hrow, at + 1024, end, h1);
        mx = umax(mx, compensate4(g0, h0, a.alpha, v));
        mx = umax(mx, compensate4(g1, h1, a.alpha, v));
    }
    mx = wave_max_uniform(mx);
    if (lane == 0) wave_norm[wave] = mx;
    __syncthreads();
    if (threadIdx.x == 0 && begin < end) {
        const uint32_t norm = umax(umax(wave_norm[0], wave_norm[1]), umax(wave_norm[2], wave_norm[3]));
        atomicMax(reinterpret_cast<uint32_t *>(a.scales + (int64_t)p * a.scale_stride) + k, norm);
    }
}

// l2 norm of buckets longer than 32768 elements (two launches).  The sum of squares follows the
// balanced tree by element index (the bucket padded with zeros to a power of two; adding a
// zero changes nothing): a block takes an aligned piece of 8192 elements of one bucket -- the
// lanes of each 256-element run, the four runs of a kilo-element, the eight kilo-elements --
// and leaves the piece's sum in `pieces`; then one block per bucket adds the pieces pairwise by
// index, level by level between two buffers, and takes the square root.
// The caller lends the buffers: `pieces` and `spare` live in the worker's row of `codes`, which
// the second pass overwrites afterwards.  blockIdx.x = bucket * pieces_per_bucket + piece.
constexpr int kSumPiece = 8192;

__global__ void __launch_bounds__(256) k_bucket_sumsq(const Args a, const int64_t pieces_per_bucket)
{
    __shared__ float wave_sum[kSumPiece / 1024][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t p = blockIdx.y;
    const int64_t k = blockIdx.x / pieces_per_bucket;
    const int64_t piece = blockIdx.x - k * pieces_per_bucket;
    const int64_t bucket_begin = k * (int64_t)a.bucket;
    int64_t bucket_end = bucket_begin + a.bucket;
    if (bucket_end > a.n) bucket_end = a.n;
    const int64_t begin = bucket_begin + piece * kSumPiece + (int64_t)threadIdx.x * 4;
    const float *__restrict__ grow = a.g + (int64_t)p * a.gh_stride;
    const float *__restrict__ hrow = a.h + (int64_t)p * a.gh_stride;
#pragma unroll
    for (int i = 0; i < kSumPiece / 1024; ++i) {
        // Elements at or beyond the bucket's end read as 0 and add 0.
        float g[4], h[4], v[4];
        load4(grow, begin + i * 1024, bucket_end, g);
        load4(hrow, begin + i * 1024, bucket_end, h);
        compensate4(g, h, a.alpha, v);
        const float run = group_sum_tree(sum_squares4(v), 64);
        if (lane == 0) wave_sum[i][wave] = run;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float t[kSumPiece / 1024];
#pragma unroll
        for (int i = 0; i < kSumPiece / 1024; ++i) {
            const float lo = wave_sum[i][0] + wave_sum[i][1];
            const float hi = wave_sum[i][2] + wave_sum[i][3];
            t[i] = lo + hi;
        }
#pragma unroll
        for (int w = 1; w < kSumPiece / 1024; w *= 2)
#pragma unroll
            for (int i = 0; i + w < kSumPiece / 1024; i += 2 * w) t[i] = t[i] + t[i + w];
        reinterpret_cast<float *>(a.codes + (int64_t)p * a.code_stride)[blockIdx.x] = t[0];
    }
}

__global__ void __launch_bounds__(256) k_bucket_sumsq_finish(const Args a, const int64_t pieces_per_bucket)
{
    const uint32_t p = blockIdx.y;
    const int64_t k = blockIdx.x;
    const int64_t half = (pieces_per_bucket + 1) / 2;
    float *row = reinterpret_cast<float *>(a.codes + (int64_t)p * a.code_stride);
    float *src = row + k * pieces_per_bucket;                  // this bucket's pieces
    float *dst = row + (int64_t)a.nb * pieces_per_bucket + k * half;   // ... and its spare buffer
    int64_t count = pieces_per_bucket;
    while (count > 1) {
        const int64_t pairs = (count + 1) / 2;
        for (int64_t i = threadIdx.x; i < pairs; i += blockDim.x) {
            const float lo = src[2 * i];
            const float hi = 2 * i + 1 < count ? src[2 * i + 1] : 0.0f;
            dst[i] = lo + hi;
        }
        __syncthreads();                                       // the block's writes, before its next reads
        float *t = src;
        src = dst;
        dst = t;
        count = pairs;
    }
    if (threadIdx.x == 0) a.scales[(int64_t)p * a.scale_stride + k] = __builtin_sqrtf(src[0]);
}

__global__ void __launch_bounds__(256) k_zero_scales(const Args a)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < a.nb) a.scales[(int64_t)blockIdx.y * a.scale_stride + k] = 0.0f;
}

// ---------------------------------------------------------------------------------------------
// Decode side.
// ---------------------------------------------------------------------------------------------

// Decode table of the decoding kernels for r > 2, in LDS: sxi[c] = +-fl(|c-s|/s) for the codes
// 0..2s and 0 beyond, so that g~ = norm * sxi[c] (Eq. 8).  r = 2 needs no table.
template <int R>
__device__ __forceinline__ void fill_agg_table(float *table, int s)
{
    if constexpr (R != 2) {
        for (int c = threadIdx.x; c < 256; c += blockDim.x) {
            const int q = c - s;
            const int m = q < 0 ? -q : q;
            const float xi = (m <= s) ? (float)m / (float)s : 0.0f;
            table[c] = q < 0 ? -xi : xi;
        }
        __syncthreads();
    }
}

// Eq. (8) from a code c = level + s: scale * sxi[c], sxi[c] = +-fl(|c - s|/s).  Codes beyond 2s
// (no message of this library holds one) decode as level 0, here as in the aggregation kernel.
template <int R>
__device__ __forceinline__ float decode_one(uint64_t bits, int e, float scale, const float *sxi)
{
    const uint32_t c = (uint32_t)(bits >> (R * e)) & ((1u << R) - 1u);
    if constexpr (R == 2) {
        const float level = c == 0u ? -1.0f : (c == 2u ? 1.0f : 0.0f);
        return scale * level;
    } else {
        return scale * sxi[c];
    }
}

// The 4*R code bits of the 4 elements starting at `elem` (a multiple of 4).  They start at bit
// 0 or 4 of a byte and span (R+1)/2 bytes.
template <int R>
__device__ __forceinline__ uint32_t load_codes4(const uint8_t *__restrict__ crow, int64_t row_bytes,
                                                int64_t elem, bool full)
{
    const int64_t bit0 = elem * R;
    const int64_t byte0 = bit0 >> 3;
    if constexpr (R == 2) {
        if (full) return crow[byte0];
    } else if constexpr (R == 4) {
        if (full) return *reinterpret_cast<const uint16_t *>(crow + byte0);
    } else if constexpr (R == 8) {
        if (full) return *reinterpret_cast<const uint32_t *>(crow + byte0);
    }
    constexpr int NB = (R + 1) / 2;
    uint32_t w = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b)
        if (byte0 + b < row_bytes) w |= (uint32_t)crow[byte0 + b] << (8 * b);
    w >>= (int)(bit0 & 7);
    return (R == 8) ? w : (w & ((1u << (4 * (R & 7))) - 1u));
}

// Eq. (6) from an encoded message, in the access pattern of the fused kernel: a wave owns two
// runs of 256 consecutive elements, a lane 4 consecutive elements of each (one float4 of g and
// of h, 4*R code bits, one norm), everything streamed once with non-temporal accesses.
// bucket_shift >= 0 when the bucket is a power of two.
template <int R>
__global__ void __launch_bounds__(256) k_error_update(const Args a, const int bucket_shift)
{
    __shared__ float sxi[R == 2 ? 1 : 256];
    fill_agg_table<R>(sxi, a.s);
    constexpr int J = 2;
    const int lane = threadIdx.x & 63;
    const uint32_t p = blockIdx.y;
    int64_t base = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * (256 * J);
    base = ((int64_t)__builtin_amdgcn_readfirstlane((int)(base >> 32)) << 32) |
           (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
    if (base >= a.n) return;                                   // wave-uniform
    const float *__restrict__ grow = a.g + (int64_t)p * a.gh_stride;
    float *__restrict__ hrow = a.h + (int64_t)p * a.gh_stride;
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    const float *__restrict__ srow = a.scales + (int64_t)p * a.scale_stride;
    // Bucket of the wave's first element, once per wave; lanes add a 32-bit quotient.
    const int64_t k0 = bucket_shift >= 0 ? (base >> bucket_shift) : (base / a.bucket);
    const uint32_t rem0 = (uint32_t)(base - k0 * a.bucket);

    float g[J][4], h[J][4], scale[J];
    uint32_t bits[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int64_t elem = base + j * 256 + lane * 4;
        load4(grow, elem, a.n, g[j]);
        load4(hrow, elem, a.n, h[j]);
        const bool exists = elem < a.n;
        bits[j] = exists ? load_codes4<R>(crow, a.row_bytes, elem, elem + 4 <= a.n) : 0u;
        const uint32_t r = rem0 + (uint32_t)(j * 256 + lane * 4);
        const int64_t k = k0 + (bucket_shift >= 0 ? (r >> bucket_shift) : (r / (uint32_t)a.bucket));
        scale[j] = exists ? srow[k] : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int64_t elem = base + j * 256 + lane * 4;
        if (elem >= a.n) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            h[j][e] = error_update(a.beta, h[j][e], g[j][e], decode_one<R>(bits[j], e, scale[j], sxi));
        store4(hrow, elem, a.n, h[j]);
    }
}

// sum += one worker's dequantised values for a lane's 4 elements.
//   r = 2: sum = fma(norm, level, sum) equals sum + norm * level because that product is exact.
template <int R>
__device__ __forceinline__ void agg_add(const float *table, uint32_t bits, float norm, float (&sum)[4])
{
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if constexpr (R == 2) {
            const uint32_t c = (bits >> (2 * e)) & 3u;
            const float level = c == 0u ? -1.0f : (c == 2u ? 1.0f : 0.0f);
            sum[e] = __builtin_fmaf(norm, level, sum[e]);
        } else {
            const float gt = norm * table[(bits >> (R * e)) & ((1u << R) - 1u)];
            sum[e] = sum[e] + gt;
        }
    }
}

// One run of 256 outputs starting at `run`, any bucket size, ragged end allowed: the slow,
// fully guarded route (per-lane bucket index, one worker at a time).
template <int R>
__device__ __forceinline__ void agg_run_guarded(const Args &a, const float *table, int64_t run, int lane,
                                             int bucket_shift, float inv_p)
{
    const int64_t elem = run + lane * 4;
    const bool exists = elem < a.n;
    const bool full = elem + 4 <= a.n;
    const int64_t k = !exists ? 0 : (bucket_shift >= 0 ? (elem >> bucket_shift) : (elem / a.bucket));
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const uint8_t *__restrict__ crow = a.codes;
    const float *__restrict__ srow = a.scales;
    for (int p = 0; p < a.workers; ++p) {
        const uint32_t bits = exists ? load_codes4<R>(crow, a.row_bytes, elem, full) : 0u;
        agg_add<R>(table, bits, srow[k], acc);
        crow += a.code_stride;
        srow += a.scale_stride;
    }
    const float pf = (float)a.workers;
    float o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = inv_p > 0.0f ? acc[e] * inv_p : acc[e] / pf;
    if (a.out) store4(a.out, elem, a.n, o);
    if (a.w) {
        float wv[4];
        load4(a.w, elem, a.n, wv);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float stepv = a.eta * o[e];
            wv[e] = wv[e] - stepv;
        }
        store4(a.w, elem, a.n, wv);
    }
}

// Pair table of the r = 2 fast path: a nibble (two codes) -> the two levels {-1, 0, +1} as
// floats, one copy per lane of a half-wave.  The LDS serves a 64-bit read to 32 lanes per
// clock over 64 banks, so with entry `nib` of copy `lane & 31` at float2 index nib*32 + copy
// the lanes served together always hit 32 different bank pairs: no conflicts whatever the
// codes are.  (A table shared by all lanes conflicts on three cycles out of four.)
__device__ __forceinline__ void fill_pair_table(f2 *pair, int)
{
    for (int i = threadIdx.x; i < 16 * 32; i += blockDim.x) {
        const int nib = i >> 5, c0 = nib & 3, c1 = nib >> 2;
        f2 lv;
        lv.x = c0 == 0 ? -1.0f : (c0 == 2 ? 1.0f : 0.0f);
        lv.y = c1 == 0 ? -1.0f : (c1 == 2 ? 1.0f : 0.0f);
        pair[i] = lv;
    }
    __syncthreads();
}

// Byte table of the r = 4 fast path: one code byte (two codes) -> their signed grid points
// +-fl(|c - s|/s) as a float2, shared by all lanes: half the address arithmetic of one lookup
// per code.  The entry of byte t sits in slot t ^ (t >> 4): the bytes that occur together in a
// message mostly differ from the most frequent one (both levels 0) in one nibble, and this
// spreads them over different banks whichever nibble it is (lanes that read the same entry
// are served together).
__device__ __forceinline__ void fill_byte_table(f2 *tab, int s)
{
    for (int t = threadIdx.x; t < 256; t += blockDim.x) {
        float xi[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int c = (t >> (4 * k)) & 15, q = c - s, m = q < 0 ? -q : q;
            const float v = (m <= s) ? (float)m / (float)s : 0.0f;
            xi[k] = q < 0 ? -v : v;
        }
        f2 e;
        e.x = xi[0];
        e.y = xi[1];
        tab[t ^ (t >> 4)] = e;
    }
    __syncthreads();
}

// Byte 1 of `at` <- the low (HIGH = 0) or high (HIGH = 1) nibble of byte k of x; the other bytes
// of `at` stay.  A partial-register write must not be read by the very next vector instruction
// on this chip, and the compiler does not see inside the statement: the idle slot after it
// keeps that distance whatever is scheduled next.
template <int HIGH>
__device__ __forceinline__ void pair_address(uint32_t &at, uint32_t x, int k)
{
#define ECQ_PAIR_ADDRESS(K)                                                                                      \
    if (HIGH)                                                                                                    \
        asm("v_lshrrev_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD "            \
            "src1_sel:BYTE_" #K "\n\ts_nop 0"                                                                    \
            : "+v"(at)                                                                                           \
            : "v"(4u), "v"(x));                                                                                  \
    else                                                                                                         \
        asm("v_and_b32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_" #K " "          \
            "src1_sel:DWORD\n\ts_nop 0"                                                                          \
            : "+v"(at)                                                                                           \
            : "v"(x), "v"(0x0Fu))
    switch (k) {
    case 0: ECQ_PAIR_ADDRESS(0); break;
    case 1: ECQ_PAIR_ADDRESS(1); break;
    case 2: ECQ_PAIR_ADDRESS(2); break;
    default: ECQ_PAIR_ADDRESS(3); break;
    }
#undef ECQ_PAIR_ADDRESS
}

// acc += one worker's dequantised values for a lane's 16 elements (Eq. 8).
//   r = 2: levels from the pair table; acc = fma(norm, level, acc) equals acc + norm * level
//          because that product is exact.
//   r = 4: two grid points per lookup from the byte table, g~ = norm * sxi[c], then acc + g~.
//   else : g~ = norm * sxi[c], then acc + g~, as in agg_add.
template <int R>
__device__ __forceinline__ void agg_add16(const float *sxi, const f2 *pair, uint32_t lane_off, const Codes16<R> &cd,
                                          float norm_lo, float norm_hi, float (&acc)[16])
{
    // norm_lo scales the lane's first 8 outputs, norm_hi the other 8 (two buckets when the bucket
    // size is an odd multiple of 8; else the same value twice).
    if constexpr (R == 2) {
        const uint32_t x = cd.w[0];
        // Byte offset nib*256 + (lane & 31)*8 of a lookup: the lane's copy offset sits in byte 0,
        // the nibble goes into byte 1 with one sub-dword-addressed instruction that takes byte K
        // of the codes, masks or shifts it, and writes only that byte of the address register.
        // Two address registers alternate between the low and the high nibbles.
        uint32_t lo_at = lane_off, hi_at = lane_off;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float norm = k < 2 ? norm_lo : norm_hi;
            pair_address<0>(lo_at, x, k);
            const f2 a = *reinterpret_cast<const f2 *>(reinterpret_cast<const char *>(pair) + lo_at);
            acc[4 * k] = __builtin_fmaf(norm, a.x, acc[4 * k]);
            acc[4 * k + 1] = __builtin_fmaf(norm, a.y, acc[4 * k + 1]);
            pair_address<1>(hi_at, x, k);
            const f2 b = *reinterpret_cast<const f2 *>(reinterpret_cast<const char *>(pair) + hi_at);
            acc[4 * k + 2] = __builtin_fmaf(norm, b.x, acc[4 * k + 2]);
            acc[4 * k + 3] = __builtin_fmaf(norm, b.y, acc[4 * k + 3]);
        }
    } else if constexpr (R == 4) {
        // `pair` is the byte table here: g~ = norm * sxi[c] for the byte's two codes, then acc + g~.
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const float norm = i == 0 ? norm_lo : norm_hi;
            const uint32_t x = cd.w[i], y = x ^ ((x >> 4) & 0x0F0F0F0Fu);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t off = ((y >> (8 * k)) & 0xFFu) << 3;
                const f2 xi = *reinterpret_cast<const f2 *>(reinterpret_cast<const char *>(pair) + off);
                const float g0 = norm * xi.x, g1 = norm * xi.y;
                acc[8 * i + 2 * k] = acc[8 * i + 2 * k] + g0;
                acc[8 * i + 2 * k + 1] = acc[8 * i + 2 * k + 1] + g1;
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const float gt = (e < 8 ? norm_lo : norm_hi) * sxi[cd.code(e)];
            acc[e] = acc[e] + gt;
        }
    }
}

constexpr int kAggRun = 1024;          // outputs per wave
constexpr int kAggStageStride = 20;    // floats between lanes in the transposition buffer

// Eq. (4): out[i] = (sum_{p=0}^{P-1} g~_p[i]) / P, workers added in index order.
// A wave owns 1024 consecutive outputs, a lane 16 consecutive ones, so every worker costs a
// lane one aligned load of 2*R code bytes (a wave reads 128*R contiguous bytes per worker) and
// its norms: NORMS = 0 when the bucket is a multiple of 1024 (one norm per wave, a scalar
// load), 1 when it is a multiple of 16 (one per lane), 2 otherwise (buckets are multiples of 8,
// so the lane's two halves of 8 outputs may lie in two buckets: one norm each).  r = 2: U
// workers' codes and norms are requested together, the next U while the current ones are added
// (U = 8 from 16 workers on, else 4: -3 % at 32 workers, +7 % at 8); r = 4: eight at a time.  Codes are read once, with non-temporal loads: a regular load would take a line of the
// last-level cache and push out a dirty line the pass before left there (its code stores), and
// the write-back of up to 256 MB of such lines is charged to this kernel (+14-20 % measured
// at 16 and 32 workers).  The 16 sums of a lane are then transposed through
// LDS so the wave stores (and, for the model update, loads) whole contiguous kilobytes as
// float4 per lane.  The ragged last run of a row goes through agg_run_guarded.
// bucket_shift >= 0 when the bucket is a power of two.
template <int R, int NORMS, int U, bool STREAM>
__global__ void __launch_bounds__(256) k_dequant_aggregate(const Args a, const int bucket_shift, const float inv_p)
{
    // One LDS object with the pair table first: its byte offsets are then LDS addresses, and a
    // lookup address is a single AND-OR of the shifted codes with the lane's copy offset.
    // (r = 4: `pair` holds the byte table, 256 entries.)
    struct Lds {
        f2 pair[R == 2 ? 16 * 32 : (R == 4 ? 256 : 1)];
        float table[R == 2 ? 1 : 256];
        __attribute__((aligned(16))) float stage[4][64 * kAggStageStride];
    };
    __shared__ __attribute__((aligned(4096))) Lds lds;
    float *table = lds.table;
    const f2 *pair = lds.pair;
    fill_agg_table<R>(lds.table, a.s);
    if constexpr (R == 2) fill_pair_table(lds.pair, 0);
    if constexpr (R == 4) fill_byte_table(lds.pair, a.s);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t base = ((int64_t)blockIdx.x * 4 + wave) * kAggRun;
    base = ((int64_t)__builtin_amdgcn_readfirstlane((int)(base >> 32)) << 32) |
           (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
    if (base >= a.n) return;                                   // wave-uniform
    if (base + kAggRun > a.n) {
#pragma unroll 1
        for (int j = 0; j < kAggRun / 256; ++j)
            if (base + j * 256 < a.n) agg_run_guarded<R>(a, table, base + j * 256, lane, bucket_shift, inv_p);
        return;
    }

    const int64_t first = base + lane * 16;
    const int64_t k_lane = bucket_shift >= 0 ? (first >> bucket_shift) : (first / a.bucket);
    const int64_t k_half = bucket_shift >= 0 ? ((first + 8) >> bucket_shift) : ((first + 8) / a.bucket);
    const int64_t k_wave = bucket_shift >= 0 ? (base >> bucket_shift) : (base / a.bucket);
    const uint8_t *__restrict__ cptr = a.codes + ((base * R) >> 3) + lane * (2 * R);
    const float *__restrict__ srow = a.scales;
    const uint32_t lane_off = (uint32_t)(lane & 31) * 8u;
    // One worker's norms for the lane's first and second 8 outputs.
    auto norms_of = [&](const float *__restrict__ row, float &lo, float &hi) {
        lo = NORMS == 0 ? row[k_wave] : row[k_lane];
        if constexpr (NORMS == 2) hi = row[k_half];            // (else `hi` is never read)
    };

    float acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.0f;

    if constexpr (R == 2) {
        // Batches of U workers; the codes and norms of the next batch are requested before the
        // current one is added, so two batches are in flight.  Workers are added in index order.
        const int batches = a.workers / U;
        Codes16<R> cd[U], cd_next[U];
        float lo[U], hi[U], lo_next[U], hi_next[U];
        auto request = [&](Codes16<R> (&c)[U], float (&nl)[U], float (&nh)[U]) {
    #pragma unroll
            for (int u = 0; u < U; ++u) {
                c[u].template load<STREAM>(cptr + u * a.code_stride);
                norms_of(srow + u * a.scale_stride, nl[u], nh[u]);
            }
            cptr += U * a.code_stride;
            srow += U * a.scale_stride;
        };
        if (batches > 0) request(cd_next, lo_next, hi_next);
        for (int b = 0; b < batches; ++b) {
    #pragma unroll
            for (int u = 0; u < U; ++u) {
                cd[u] = cd_next[u];
                lo[u] = lo_next[u];
                if constexpr (NORMS == 2) hi[u] = hi_next[u];
            }
            if (b + 1 < batches) request(cd_next, lo_next, hi_next);
    #pragma unroll
            for (int u = 0; u < U; ++u)
                agg_add16<R>(table, pair, lane_off, cd[u], lo[u], NORMS == 2 ? hi[u] : lo[u], acc);
        }
        for (int p = batches * U; p < a.workers; ++p) {
            Codes16<R> one;
            float one_lo, one_hi;
            one.template load<STREAM>(cptr);
            norms_of(srow, one_lo, one_hi);
            agg_add16<R>(table, pair, lane_off, one, one_lo, NORMS == 2 ? one_hi : one_lo, acc);
            cptr += a.code_stride;
            srow += a.scale_stride;
        }
    } else {
        // r > 2: the table lookups want the compiler's unrolled schedule: V workers per step (a
        // software pipeline like the one above measured 15-20 % slower at r = 4).
        constexpr int V = R == 4 ? 8 : 2;
        int p = 0;
        for (; p + V <= a.workers; p += V) {
            Codes16<R> cd[V];
            float lo[V], hi[V];
#pragma unroll
            for (int u = 0; u < V; ++u) {
                cd[u].template load<STREAM>(cptr + u * a.code_stride);
                norms_of(srow + u * a.scale_stride, lo[u], hi[u]);
            }
#pragma unroll
            for (int u = 0; u < V; ++u)
                agg_add16<R>(table, pair, lane_off, cd[u], lo[u], NORMS == 2 ? hi[u] : lo[u], acc);
            cptr += V * a.code_stride;
            srow += V * a.scale_stride;
        }
        for (; p < a.workers; ++p) {
            Codes16<R> one;
            float one_lo, one_hi;
            one.template load<STREAM>(cptr);
            norms_of(srow, one_lo, one_hi);
            agg_add16<R>(table, pair, lane_off, one, one_lo, NORMS == 2 ? one_hi : one_lo, acc);
            cptr += a.code_stride;
            srow += a.scale_stride;
        }
    }

    // Division by P, then lane-major (16 consecutive outputs per lane) -> float4-per-lane order.
    const float pf = (float)a.workers;
    float *__restrict__ mine = lds.stage[wave];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f4 o;
        if (inv_p > 0.0f) {
            o.x = acc[4 * q] * inv_p; o.y = acc[4 * q + 1] * inv_p; o.z = acc[4 * q + 2] * inv_p; o.w = acc[4 * q + 3] * inv_p;
        } else {
            o.x = acc[4 * q] / pf; o.y = acc[4 * q + 1] / pf; o.z = acc[4 * q + 2] / pf; o.w = acc[4 * q + 3] / pf;
        }
        *reinterpret_cast<f4 *>(&mine[lane * kAggStageStride + 4 * q]) = o;
    }
    // Only this wave touches its buffer, and a wave's LDS operations complete in order.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int f = q * 64 + lane;                           // float4 index inside the run
        const f4 o = *reinterpret_cast<const f4 *>(&mine[(f >> 2) * kAggStageStride + (f & 3) * 4]);
        const int64_t at = base + 4 * f;
        if (a.out) __builtin_nontemporal_store(o, reinterpret_cast<f4 *>(a.out + at));
        if (a.w) {                                             // Alg. 1: w <- w - eta * g~
            f4 wv = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(a.w + at));
            const f4 stepv = o * a.eta;
            wv = wv - stepv;
            __builtin_nontemporal_store(wv, reinterpret_cast<f4 *>(a.w + at));
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Level histogram (the d_k of the entropy-coding bound).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_zero_counts(unsigned long long *counts, int64_t count_stride, int bins)
{
    if ((int)threadIdx.x < bins) counts[(int64_t)blockIdx.x * count_stride + threadIdx.x] = 0ull;
}

// A lane owns four consecutive runs of 16 elements (8*R contiguous bytes); a block walks chunks
// of kHistPerBlock elements of one row, counts into registers or LDS and adds its totals to the
// row's counters once.
//   r = 2: the three levels are counted with bit masks and population counts, 16 codes at a
//          time, in registers.
//   r = 3, 4: every thread has a private set of 16 counters in LDS (17 words apart, so that
//          lanes counting the same level hit 64 different banks) and sends one LDS add per
//          element, without waiting for it.
//   else : level 0 (code s), by far the most frequent, is counted in a register; the other
//          codes go to one histogram per wave with LDS atomic adds.
// Few, long-lived blocks: all blocks of a row end in the same 2s+1 global counters, and atomic
// adds to one address are served one at a time (about 80 ns each on this chip).
constexpr int kHistThreads = 512;
constexpr int kHistIters = 2;
constexpr int kHistGroups = 4;                                 // runs of 16 elements a lane loads together
constexpr int kHistPerBlock = kHistThreads * 16 * kHistGroups * kHistIters;
constexpr int kHistBlocks = 768;                               // target for the whole grid: three per CU

template <int R>
__global__ void __launch_bounds__(kHistThreads) k_level_histogram(const Args a,
                                                                 unsigned long long *__restrict__ counts,
                                                                 const int64_t count_stride)
{
    constexpr bool kPrivate = R > 2 && R <= 4;                 // at most 16 levels
    constexpr int kPrivStride = 17;
    constexpr int kWaves = kHistThreads / 64;
    __shared__ unsigned int hist[kWaves][256];
    __shared__ unsigned int priv[kPrivate ? kHistThreads * kPrivStride : 1];
    for (int c = threadIdx.x; c < kWaves * 256; c += blockDim.x) (&hist[0][0])[c] = 0u;
    if constexpr (kPrivate)
        for (int c = 0; c < kPrivStride; ++c) priv[threadIdx.x * kPrivStride + c] = 0u;
    __syncthreads();
    const uint32_t p = blockIdx.y;
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned int *__restrict__ my_priv = priv + (kPrivate ? threadIdx.x * kPrivStride : 0);
    unsigned int n_center = 0, n1 = 0, n2 = 0, n3 = 0, n_valid = 0;
    // The blocks of a row take its chunks of kHistPerBlock elements round robin.
    for (int64_t begin = (int64_t)blockIdx.x * kHistPerBlock; begin < a.n; begin += (int64_t)gridDim.x * kHistPerBlock)
#pragma unroll
    for (int it = 0; it < kHistIters; ++it) {
        const int64_t elem0 = begin + ((int64_t)it * kHistThreads + threadIdx.x) * (16 * kHistGroups);
        Codes16<R> cd[kHistGroups];
        int valid[kHistGroups];
        if (elem0 + 16 * kHistGroups <= a.n) {                 // the common case: one contiguous piece
            const uint8_t *__restrict__ src = crow + ((elem0 * R) >> 3);
#pragma unroll
            for (int k = 0; k < kHistGroups; ++k) {
                cd[k].load(src + k * 2 * R);
                valid[k] = 16;
            }
        } else {
#pragma unroll
            for (int k = 0; k < kHistGroups; ++k) {
                const int64_t elem = elem0 + 16 * k;
#pragma unroll
                for (int i = 0; i < Codes16<R>::kWords; ++i) cd[k].w[i] = 0u;
                valid[k] = 0;
                if (elem < a.n) {
                    cd[k].load_guarded(crow, a.row_bytes, elem);
                    valid[k] = (int)(a.n - elem < 16 ? a.n - elem : 16);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < kHistGroups; ++k) {
            if constexpr (R == 2) {
                // Pad codes are zero bits (code 0) and are removed through n_valid.
                const uint32_t x = cd[k].w[0], lo = x & 0x55555555u, hi = (x >> 1) & 0x55555555u;
                n1 += __popc(lo & ~hi);
                n2 += __popc(hi & ~lo);
                n3 += __popc(hi & lo);
                n_valid += valid[k];
            } else if constexpr (kPrivate) {
                if (valid[k] == 16) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) atomicAdd(&my_priv[cd[k].code(e)], 1u);
                } else {
#pragma unroll
                    for (int e = 0; e < 16; ++e)
                        if (e < valid[k]) atomicAdd(&my_priv[cd[k].code(e)], 1u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const unsigned int c = cd[k].code(e);
                    if (e < valid[k]) {
                        if (c == (unsigned int)a.s) ++n_center;
                        else atomicAdd(&hist[wave][c], 1u);
                    }
                }
            }
        }
    }
    if constexpr (R == 2) {
        for (int d = 1; d < 64; d <<= 1) {
            n1 += __shfl_xor(n1, d, 64);
            n2 += __shfl_xor(n2, d, 64);
            n3 += __shfl_xor(n3, d, 64);
            n_valid += __shfl_xor(n_valid, d, 64);
        }
        if (lane == 0) {
            hist[wave][0] = n_valid - n1 - n2 - n3;
            hist[wave][1] = n1;
            hist[wave][2] = n2;
        }
    } else if constexpr (kPrivate) {
        __syncthreads();
        // Thread (c, part) adds up level c over 16 of the block's private sets.
        const int c = threadIdx.x & 15, part = threadIdx.x >> 4;
        unsigned int sum = 0;
        for (int t = part * 16; t < part * 16 + 16; ++t) sum += priv[t * kPrivStride + c];
        if (sum) atomicAdd(&hist[0][c], sum);
    } else {
        for (int d = 1; d < 64; d <<= 1) n_center += __shfl_xor(n_center, d, 64);
        if (lane == 0 && n_center) atomicAdd(&hist[wave][a.s], n_center);
    }
    __syncthreads();
    const int bins = 2 * a.s + 1;
    for (int c = threadIdx.x; c < bins; c += blockDim.x) {
        unsigned int total = 0;
        for (int w = 0; w < kWaves; ++w) total += hist[w][c];
        if (total) atomicAdd(&counts[(int64_t)p * count_stride + c], (unsigned long long)total);
    }
}

// ---------------------------------------------------------------------------------------------
// Inspection and calibration kernels.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}

// Division self-check: thread t owns the divisor with significand t (all 2^23) and an exponent
// drawn from `salt`; numerators stay at or below the divisor, or up to an eighth above it (the
// computed l2 norm of a bucket can fall that far below its largest element), as in the kernels.
template <bool SCALE24>
__global__ void __launch_bounds__(256) k_check_division(unsigned long long *mismatches, int per_divisor,
                                                       int wide_exponents, uint32_t salt)
{
    const uint32_t t = blockIdx.x * 256 + threadIdx.x;
    const int ex = wide_exponents ? 1 + (int)(mix32(t + salt) % 253u) : 27 + (int)(mix32(t ^ salt) % 201u);
    const float d = __uint_as_float(((uint32_t)ex << 23) | (t & 0x7FFFFFu));
    const Ratio rt = make_ratio<SCALE24>(d);
    unsigned int bad = 0;
    for (int i = 0; i < per_divisor; ++i) {
        const uint32_t r = mix32(t * 2654435761u + (uint32_t)i * 40503u + salt);
        const uint32_t mode = r & 7u;
        float av;
        if (mode < 5u) {                                       // same binade or the one below
            av = __uint_as_float(((uint32_t)(ex - (int)((r >> 3) & 1u)) << 23) | (mix32(r) & 0x7FFFFFu));
        } else if (mode == 5u) {                               // up to 2^60 smaller
            int ee = ex - (int)(mix32(r) % 60u);
            ee = ee < 0 ? 0 : ee;
            av = __uint_as_float(((uint32_t)ee << 23) | (mix32(r + 1u) & 0x7FFFFFu));
        } else if (mode == 6u) {                               // tiny, denormals included
            av = __uint_as_float(mix32(r) & 0x00FFFFFFu);
        } else if (r & 8u) {
            av = d;
        } else {                                               // up to 2^20 units in the last place above
            av = __uint_as_float(__float_as_uint(d) + (mix32(r + 2u) & 0xFFFFFu));
        }
        if (mode != 7u && !(av <= d)) av = d;
        float want = av / d;
        if (SCALE24) want = want * 0x1p24f;
        bad += __float_as_uint(ratio<SCALE24>(av, rt)) != __float_as_uint(want);
    }
    if (bad) atomicAdd(mismatches, (unsigned long long)bad);
}

__global__ void k_zero_u64(unsigned long long *x) { *x = 0ull; }

__global__ void __launch_bounds__(256) k_philox_words(uint32_t key0, uint32_t key1, uint32_t step_lo,
                                                     uint32_t step_hi, uint32_t p, uint64_t i0,
                                                     int64_t count, uint32_t *__restrict__ words)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= count) return;
    const uint64_t i = i0 + (uint64_t)j;
    const U4 blk = philox4x32_10((uint32_t)(i >> 2), p, step_lo, step_hi, key0, key1);
    const uint32_t lane_word[4] = {blk.x, blk.y, blk.z, blk.w};
    words[j] = lane_word[i & 3];
}

// One float4 per lane, one 4 KiB tile per block, blocks in address order: the access pattern of
// the fused kernel without its arithmetic.
__global__ void __launch_bounds__(256) k_calib_add(const float *__restrict__ x, const float *__restrict__ y,
                                                  float *__restrict__ out, int64_t n)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    float u[4], v[4], w[4];
    load4(x, i, n, u);
    load4(y, i, n, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = u[e] + v[e];
    store4(out, i, n, w);
}

__global__ void __launch_bounds__(256) k_calib_copy(const float *__restrict__ x, float *__restrict__ out,
                                                   int64_t n)
{
    const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    float u[4];
    load4(x, i, n, u);
    store4(out, i, n, u);
}

// ---------------------------------------------------------------------------------------------
// Launchers.
// ---------------------------------------------------------------------------------------------

template <int R, int J>
static void launch_team_j(const Args &a, const Plan &plan, bool update, hipStream_t st)
{
    int w_shift = 0;
    while ((1 << w_shift) < plan.waves_per_bucket) ++w_shift;
    const int teams = plan.block_threads / (64 * plan.waves_per_bucket);
    const unsigned blocks_per_row = cdiv(a.nb, teams);
    // Long launches lose bandwidth on this chip (the XCDs drift apart and the window of
    // addresses in flight widens); rows are therefore issued in groups of about 2^28 elements,
    // one launch per group, back to back on the stream.
    int64_t rows_per_launch = plan.rows_per_launch > 0 ? plan.rows_per_launch : a.workers;
    for (int64_t w0 = 0; w0 < a.workers; w0 += rows_per_launch) {
        const unsigned rows = (unsigned)((a.workers - w0 < rows_per_launch) ? a.workers - w0 : rows_per_launch);
        dim3 grid(blocks_per_row, rows);
        int64_t stripe = 0;
        if (plan.xcd_striped) {
            stripe = ((int64_t)blocks_per_row * rows + 7) / 8;
            grid = dim3((unsigned)(stripe * 8));
        }
        if (update)
            hipLaunchKernelGGL((k_fused_team<R, J, true>), grid, dim3(plan.block_threads), 0, st, a, w_shift, stripe,
                               blocks_per_row, (uint32_t)w0, rows);
        else
            hipLaunchKernelGGL((k_fused_team<R, J, false>), grid, dim3(plan.block_threads), 0, st, a, w_shift, stripe,
                               blocks_per_row, (uint32_t)w0, rows);
    }
}

template <int R>
static void launch_team(const Args &a, const Plan &plan, bool update, hipStream_t st)
{
    switch (plan.vec_per_lane) {
    case 1: launch_team_j<R, 1>(a, plan, update, st); break;
    case 2: launch_team_j<R, 2>(a, plan, update, st); break;
    case 4: launch_team_j<R, 4>(a, plan, update, st); break;
    default: launch_team_j<R, 8>(a, plan, update, st); break;
    }
}

template <int R>
static void launch_chunk(const Args &a, int lanes_per_bucket, int block_threads, bool update, hipStream_t st)
{
    // lanes_per_bucket = 0: second pass of the two-pass route; else a bucket of 8..248 elements.
    int slot_lanes = 64, span = 256;
    if (lanes_per_bucket > 0) {
        slot_lanes = 1;
        while (slot_lanes < lanes_per_bucket) slot_lanes *= 2;
        span = lanes_per_bucket * 4;
    }
    const int64_t chunk_elems = (int64_t)(64 / slot_lanes) * span;
    const int waves = block_threads / 64;
    const dim3 grid(cdiv(cdiv(a.n, chunk_elems), waves * kChunksPerWave), (unsigned)a.workers);
    const int read_norms = lanes_per_bucket == 0;
    if (update)
        hipLaunchKernelGGL((k_quant_chunk<R, true>), grid, dim3(block_threads), 0, st, a, slot_lanes, span, read_norms);
    else
        hipLaunchKernelGGL((k_quant_chunk<R, false>), grid, dim3(block_threads), 0, st, a, slot_lanes, span, read_norms);
}

template <int R>
static void launch_quantize_r(const Args &a, const Plan &plan, bool update, hipStream_t st)
{
    if (plan.path == 1 && plan.lanes_per_bucket == 0) {
        launch_team<R>(a, plan, update, st);
    } else if (plan.path == 1) {
        launch_chunk<R>(a, plan.lanes_per_bucket, 256, update, st);
    } else if (a.norm_l2) {
        // (make_plan admits the l2 norm here only for buckets beyond 32768 elements; the pieces'
        // sums and the spare buffer, 6 bytes per 8192 elements, fit the row of codes many times.)
        const int64_t pieces = cdiv((int64_t)a.bucket, kSumPiece);
        hipLaunchKernelGGL(k_bucket_sumsq, dim3((unsigned)(a.nb * pieces), (unsigned)a.workers), dim3(256), 0, st, a,
                           pieces);
        hipLaunchKernelGGL(k_bucket_sumsq_finish, dim3((unsigned)a.nb, (unsigned)a.workers), dim3(256), 0, st, a,
                           pieces);
        launch_chunk<R>(a, 0, 256, update, st);
    } else {
        hipLaunchKernelGGL(k_zero_scales, dim3(cdiv(a.nb, 256), (unsigned)a.workers), dim3(256), 0, st, a);
        if (a.bucket < 256) {
            hipLaunchKernelGGL(k_bucket_norm_small, dim3(cdiv(cdiv(a.n, 4), 256), (unsigned)a.workers), dim3(256), 0, st,
                               a);
        } else {
            // At most 256 pieces per bucket, none shorter than 8192 elements (unless the bucket is).
            int64_t parts = cdiv((int64_t)a.bucket, 8192);
            if (parts > 256) parts = 256;
            const int64_t part_len = cdiv(cdiv((int64_t)a.bucket, parts), 1024) * 1024;
            parts = cdiv((int64_t)a.bucket, part_len);
            hipLaunchKernelGGL(k_bucket_norm_large, dim3((unsigned)(a.nb * parts), (unsigned)a.workers), dim3(256), 0,
                               st, a, (int)parts, part_len);
        }
        launch_chunk<R>(a, 0, 256, update, st);
    }
}

hipError_t launch_quantize(const Args &a, const Plan &plan, bool update_h, hipStream_t stream)
{
#define CALL(RR) launch_quantize_r<RR>(a, plan, update_h, stream)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_error_update(const Args &a, hipStream_t stream)
{
    const dim3 grid(cdiv(cdiv(a.n, 512), 4), (unsigned)a.workers);
    int bucket_shift = -1;
    if ((a.bucket & (a.bucket - 1)) == 0)
        for (bucket_shift = 0; (1 << bucket_shift) < a.bucket; ++bucket_shift) {}
#define CALL(RR) hipLaunchKernelGGL((k_error_update<RR>), grid, dim3(256), 0, stream, a, bucket_shift)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_dequant_aggregate(const Args &a, hipStream_t stream)
{
    int bucket_shift = -1;
    if ((a.bucket & (a.bucket - 1)) == 0)
        for (bucket_shift = 0; (1 << bucket_shift) < a.bucket; ++bucket_shift) {}
    const int norms = (a.bucket % kAggRun) == 0 ? 0 : ((a.bucket % 16) == 0 ? 1 : 2);
    // Dividing by a power of two and multiplying by its reciprocal round identically.
    const float inv_p = (a.workers & (a.workers - 1)) == 0 ? 1.0f / (float)a.workers : 0.0f;
    const dim3 grid(cdiv(cdiv(a.n, kAggRun), 4));
    const bool wide = a.r == 2 && a.workers >= 16;             // r = 2: workers per batch (other widths ignore it)
    // Messages of up to 96 MB in all are most likely still in the 256 MB last-level cache, where
    // the encoding pass left them; larger ones are streamed past it.
    const int stream_codes = (int64_t)a.workers * a.row_bytes > ((int64_t)96 << 20);
#define LAUNCH(RR, NN, UU)                                                                                      \
    if (stream_codes)                                                                                           \
        hipLaunchKernelGGL((k_dequant_aggregate<RR, NN, UU, true>), grid, dim3(256), 0, stream, a, bucket_shift,  \
                           inv_p);                                                                              \
    else                                                                                                        \
        hipLaunchKernelGGL((k_dequant_aggregate<RR, NN, UU, false>), grid, dim3(256), 0, stream, a, bucket_shift, \
                           inv_p)
#define CALL(RR)                                                 \
    if (norms == 0) {                                            \
        if (RR == 2 && wide) { LAUNCH(RR, 0, (RR == 2 ? 8 : 4)); } \
        else { LAUNCH(RR, 0, 4); }                               \
    } else if (norms == 1) {                                     \
        if (RR == 2 && wide) { LAUNCH(RR, 1, (RR == 2 ? 8 : 4)); } \
        else { LAUNCH(RR, 1, 4); }                               \
    } else {                                                     \
        if (RR == 2 && wide) { LAUNCH(RR, 2, (RR == 2 ? 8 : 4)); } \
        else { LAUNCH(RR, 2, 4); }                               \
    }
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
#undef LAUNCH
    return hipGetLastError();
}

hipError_t launch_level_histogram(const Args &a, unsigned long long *counts, int64_t count_stride,
                                  hipStream_t stream)
{
    hipLaunchKernelGGL(k_zero_counts, dim3((unsigned)a.workers), dim3(256), 0, stream, counts, count_stride, 2 * a.s + 1);
    // About kHistBlocks blocks over all rows, each walking its share of a row.
    unsigned per_row = cdiv(a.n, kHistPerBlock);
    const unsigned want = cdiv(kHistBlocks, a.workers);
    if (per_row > want) per_row = want;
    const dim3 grid(per_row, (unsigned)a.workers);
#define CALL(RR) hipLaunchKernelGGL((k_level_histogram<RR>), grid, dim3(kHistThreads), 0, stream, a, counts, count_stride)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_check_division(int per_divisor, uint32_t salt, unsigned long long *mismatches,
                                 hipStream_t stream)
{
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(1), 0, stream, mismatches);
    const dim3 grid((1u << 23) / 256);
    for (int wide = 0; wide < 2; ++wide) {
        hipLaunchKernelGGL(k_check_division<false>, grid, dim3(256), 0, stream, mismatches, per_divisor, wide, salt);
        hipLaunchKernelGGL(k_check_division<true>, grid, dim3(256), 0, stream, mismatches, per_divisor, wide, salt + 1u);
    }
    return hipGetLastError();
}

hipError_t launch_philox_words(uint32_t key0, uint32_t key1, uint32_t step_lo, uint32_t step_hi,
                               uint32_t p, uint64_t i0, int64_t count, uint32_t *words,
                               hipStream_t stream)
{
    hipLaunchKernelGGL(k_philox_words, dim3(cdiv(count, 256)), dim3(256), 0, stream, key0, key1,
                       step_lo, step_hi, p, i0, count, words);
    return hipGetLastError();
}

hipError_t launch_calib_add(const float *x, const float *y, float *out, int64_t n, hipStream_t stream)
{
    hipLaunchKernelGGL(k_calib_add, dim3(cdiv(n, 1024)), dim3(256), 0, stream, x, y, out, n);
    return hipGetLastError();
}

// The aggregation kernel's loads and stores without its arithmetic: eight workers' code words per
// lane in flight (non-temporal loads), their sum written as the lane's 16 outputs in the same
// float4 pattern.
template <int R>
__global__ void __launch_bounds__(256) k_calib_gather(const Args a)
{
    constexpr int U = 8;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t base = ((int64_t)blockIdx.x * 4 + wave) * kAggRun;
    if (base + kAggRun > a.n) return;
    const uint8_t *__restrict__ cptr = a.codes + ((base * R) >> 3) + lane * (2 * R);
    uint32_t sum = 0;
    int p = 0;
    for (; p + U <= a.workers; p += U) {
        Codes16<R> cd[U];
#pragma unroll
        for (int u = 0; u < U; ++u) cd[u].template load<true>(cptr + (int64_t)(p + u) * a.code_stride);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int i = 0; i < Codes16<R>::kWords; ++i) sum += cd[u].w[i];
    }
    for (; p < a.workers; ++p) {
        Codes16<R> one;
        one.template load<true>(cptr + (int64_t)p * a.code_stride);
#pragma unroll
        for (int i = 0; i < Codes16<R>::kWords; ++i) sum += one.w[i];
    }
    const float r = (float)sum;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f4 o;
        o.x = r; o.y = r; o.z = r; o.w = r;
        __builtin_nontemporal_store(o, reinterpret_cast<f4 *>(a.out + base + 4 * (q * 64 + lane)));
    }
}

hipError_t launch_calib_gather(const Args &a, hipStream_t stream)
{
    const dim3 grid(cdiv(cdiv(a.n, kAggRun), 4));
#define CALL(RR) hipLaunchKernelGGL((k_calib_gather<RR>), grid, dim3(256), 0, stream, a)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_calib_copy(const float *x, float *out, int64_t n, hipStream_t stream)
{
    hipLaunchKernelGGL(k_calib_copy, dim3(cdiv(n, 1024)), dim3(256), 0, stream, x, out, n);
    return hipGetLastError();
}

}  // namespace ecq
