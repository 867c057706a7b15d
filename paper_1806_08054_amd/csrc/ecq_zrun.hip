// Zero-run Huffman coding of the quantised levels on gfx950 (MI355X), wave64.
//
// Section 4 of Wu et al. (ICML 2018) bounds the entropy-coded length of a message by
// sum_k d_k log2(d/d_k) bits.  A Huffman code over single levels spends at least one bit per
// element, while quantised gradients are mostly zeros and the bound is often far below one
// bit.  Here the Huffman code is taken over TOKENS: a run of zero levels together with the
// non-zero level that ends it.
//
// Conventions (the paper fixes none of them; they are the ones documented in ecq.h):
//   tokens     Z = floor(127 / s).  Token z*2s + j: a run of z zeros (z < Z) ended by the non-zero
//              level of rank j (levels -s..-1, 1..s in increasing order); token 2sZ: Z zeros and
//              no level.  2sZ + 1 <= 255 symbols.
//   tiles      a row is cut into tiles of 4096 elements, tokenised on their own: the Z-th zero
//              of a run sends "Z zeros" and restarts the run, a non-zero level sends
//              (run, level); a run still open at the end of the tile is sent as one "Z zeros"
//              token and the decoder drops the zeros beyond the tile.
//   code       one Huffman code per worker row from the row's token counts, built and made
//              canonical by the per-level coder's construction kernel.
//   stream     LSB-first, codewords most significant bit first, tiles back to back.
//   index      the bits of every tile (32 bits each) and the stream bit at which every group of
//              64 tiles starts (64 bits each; the last entry is the row's total).
// Codes beyond 2s (no message of this library holds one) are taken as level 0.
#include "ecq_device.hpp"
#include "ecq_internal.hpp"

namespace ecq {

constexpr int kZTile = ECQ_ZRUN_TILE;                          // elements per tile
constexpr int kZGroup = ECQ_ZRUN_GROUP;                        // tiles per group (one stream offset each)
constexpr int kZBlockTiles = 16;                               // consecutive tiles per block of the coders
constexpr int kZStep = 1024;                                   // elements a wave takes at a time (16 per lane)
constexpr int kZSteps = kZTile / kZStep;
constexpr int kZWaveTiles = kZBlockTiles / 4;                  // consecutive tiles per wave
constexpr int kZWaveSteps = kZWaveTiles * kZSteps;
constexpr int kZMaxLen = 63;                                   // longest codeword handled
constexpr int kZFastBits = 12;                                 // decode: direct table on 12 stream bits
// decode: a lane's output window has 16 or 32 words (template parameter of k_zrun_decode)
// Words of LDS a wave needs for one step: 1024 elements send at most 1025 tokens (every element
// at most one, plus the tile's closing token) of at most 63 bits, plus the up-to-31-bit shift
// that aligns the buffer with the stream's words.
constexpr int kZBufWords = ((kZStep + 1) * kZMaxLen + 31 + 31) / 32 + 1;
// When no codeword is longer than 24 bits a step of 1024 elements fills at most kZKeepAt words of
// that buffer; the rest holds the table entries of the step's tokens, at most 18 per lane (one
// per element, one "Z zeros" completed by the zeros carried in, one closing token).
constexpr int kZKeepAt = ((kZStep + 1) * 24 + 31 + 31) / 32 + 1;
constexpr int kZKeepMax = 18;
static_assert(kZKeepAt + kZKeepMax * 64 <= kZBufWords, "the kept entries fit behind the short codewords");
// A tile of at most this many bits is written in one piece (see k_zrun_write); the list of its
// non-zero levels then sits in the wave's buffer behind the words such a tile can fill.
constexpr unsigned int kZSparseTileBits = 4096;
constexpr int kZListAt = (kZSparseTileBits + 31 + 31) / 32 + 2;

static_assert(kZTile == 4096 && kZGroup == 64 && kZGroup % kZBlockTiles == 0, "a wave scans one group's 64 tile sizes");

struct ZrunShape {
    int s, two_s, Z, zz;                                       // zz = 2sZ: the token "Z zeros"
    unsigned int magic;                                        // x / Z = (x * magic) >> 20 for x < 8192
};

__device__ __forceinline__ ZrunShape zrun_shape(int s)
{
    ZrunShape z;
    z.s = s;
    z.two_s = 2 * s;
    z.Z = 127 / s;
    z.zz = 2 * s * z.Z;
    z.magic = (1u << 20) / (unsigned int)z.Z + 1u;
    return z;
}

// Bit e*STRIDE of the result is set iff element e of the lane's 16 codes is a non-zero level
// (a code below s, or above it up to 2s).
template <int R>
struct NonZero {
    static constexpr int kStride = R == 2 ? 2 : 1;
    static __device__ __forceinline__ uint32_t mask(const Codes16<R> &cd, int s)
    {
        if constexpr (R == 2) {
            // s = 1: codes 0 and 2 are the levels -1 and +1, code 1 is level 0, code 3 is off the grid.
            return ~cd.w[0] & 0x55555555u;
        } else if constexpr (R == 4) {
            // Eight codes per word, tested side by side: a nibble differs from s iff its XOR with s
            // is not zero (bit 3 of ((y & 7) + 7) | y); it exceeds 2s iff adding 15 - 2s carries
            // out of it (low and high nibbles of the bytes apart, so no carry crosses).  The
            // eight flags of a word are then gathered into eight neighbouring bits.
            const uint32_t every = 0x11111111u * (uint32_t)s, room = 0x01010101u * (uint32_t)(15 - 2 * s);
            uint32_t m = 0;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t x = cd.w[i], y = x ^ every;
                const uint32_t differs = ((((y & 0x77777777u) + 0x77777777u) | y) >> 3) & 0x11111111u;
                const uint32_t low_over = (((x & 0x0F0F0F0Fu) + room) >> 4) & 0x01010101u;
                const uint32_t high_over = ((x >> 4) & 0x0F0F0F0Fu) + room;      // flag at bit 4 of each byte
                uint32_t f = differs & ~(low_over | (high_over & 0x10101010u));   // flag of element e at bit 4e
                f = (f | (f >> 3)) & 0x03030303u;
                f = (f | (f >> 6)) & 0x000F000Fu;
                f = (f | (f >> 12)) & 0xFFu;
                m |= f << (8 * i);
            }
            return m;
        } else {
            uint32_t m = 0;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int c = (int)cd.code(e);
                m |= (c != s && c <= 2 * s) ? (1u << e) : 0u;
            }
            return m;
        }
    }
};

// Code of element `pos` (0..15) of a lane's 16 codes, pos not known at compile time.
template <int R>
__device__ __forceinline__ int code_at(const Codes16<R> &cd, int pos)
{
    if constexpr (R == 2) {
        return (int)((cd.w[0] >> (2 * pos)) & 3u);
    } else if constexpr (R == 4) {
        return (int)(((pos < 8 ? cd.w[0] : cd.w[1]) >> (4 * (pos & 7))) & 15u);
    } else {
        const int bit = R * pos, i = bit >> 5, sh = bit & 31;
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int k = 0; k < Codes16<R>::kWords; ++k) {
            lo = k == i ? cd.w[k] : lo;
            hi = k == i + 1 ? cd.w[k] : hi;
        }
        const unsigned long long both = ((unsigned long long)hi << 32) | lo;
        return (int)((both >> sh) & ((1u << R) - 1u));
    }
}

// Walks the tokens of a lane's `valid` consecutive elements in stream order.
//   run    zeros pending before the lane's first element (already below Z);
//   close  the tile ends with the lane's last element: a pending run is sent as "Z zeros".
// Returns the run pending after the lane's last element.
template <int R, class Emit>
__device__ __forceinline__ int lane_tokens(const Codes16<R> &cd, int valid, int run, bool close, const ZrunShape &z,
                                           Emit &&emit)
{
    constexpr int kStride = NonZero<R>::kStride;
    uint32_t mask = NonZero<R>::mask(cd, z.s);
    if (valid < 16) mask &= (1u << (valid * kStride)) - 1u;
    int prev = -1;
    while (mask) {
        const int pos = __builtin_ctz(mask) / kStride;
        mask &= mask - 1u;
        int total = run + (pos - prev - 1);
        while (total >= z.Z) {
            emit(z.zz);
            total -= z.Z;
        }
        const int c = code_at<R>(cd, pos);
        emit(total * z.two_s + (c < z.s ? c : c - 1));
        run = 0;
        prev = pos;
    }
    int total = run + (valid - prev - 1);
    while (total >= z.Z) {
        emit(z.zz);
        total -= z.Z;
    }
    if (close && total > 0) {
        emit(z.zz);
        total = 0;
    }
    return total;
}

// Where a lane stands inside its tile: the zeros pending before its first element.  Every lane
// reports the position (0..1023 inside the step) of its last non-zero element, or -1; an
// inclusive maximum scan over the lanes gives each lane the last non-zero element before it.
//   since  zeros since the tile's last non-zero element (or its start) when the step begins;
//          updated to the value at the step's end (wave-uniform).
template <int R>
__device__ __forceinline__ int lane_run_in(const Codes16<R> &cd, int valid, int lane, int step_valid, int &since,
                                           const ZrunShape &z)
{
    constexpr int kStride = NonZero<R>::kStride;
    uint32_t mask = NonZero<R>::mask(cd, z.s);
    if (valid < 16) mask &= (1u << (valid * kStride)) - 1u;
    const int last = mask ? lane * 16 + (31 - __builtin_clz(mask)) / kStride : -1;
    // Inclusive maximum scan over the wave (lanes without a source take -1), then one lane down.
    int incl = last;
    auto step_max = [&](int other) { incl = other > incl ? other : incl; };
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x111, 0xF, 0xF, false));   // row_shr:1
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x112, 0xF, 0xF, false));   // row_shr:2
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x114, 0xF, 0xF, false));   // row_shr:4
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x118, 0xF, 0xF, false));   // row_shr:8
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x142, 0xA, 0xF, false));   // row_bcast:15
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x143, 0xC, 0xF, false));   // row_bcast:31
    const int before = __builtin_amdgcn_update_dpp(-1, incl, 0x138, 0xF, 0xF, false);   // wave_shr:1
    const int zeros = before >= 0 ? lane * 16 - before - 1 : since + lane * 16;
    const int wave_last = __builtin_amdgcn_readlane(incl, 63);
    since = wave_last >= 0 ? step_valid - wave_last - 1 : since + step_valid;
    // zeros < 4096 + 1024: the multiplication by the reciprocal is exact there.
    return zeros - (int)(((unsigned int)zeros * z.magic) >> 20) * z.Z;
}

// The fixed-length codes of the 16 elements a lane owns in a step; returns how many exist.
template <int R>
__device__ __forceinline__ int load_step_codes(const uint8_t *__restrict__ crow, int64_t row_bytes, int64_t n,
                                               int64_t elem, Codes16<R> &cd)
{
    const int64_t rest = n - elem;
    if (rest >= 16) {
        cd.load(crow + ((elem * R) >> 3));
        return 16;
    }
#pragma unroll
    for (int i = 0; i < Codes16<R>::kWords; ++i) cd.w[i] = 0u;
    if (rest <= 0) return 0;
    cd.load_guarded(crow, row_bytes, elem);
    return (int)rest;
}

// Elements of the step that starts at step_first (all of them, over the wave).
__device__ __forceinline__ int step_elements(int64_t n, int64_t step_first)
{
    const int64_t rest = n - step_first;
    return rest >= kZStep ? kZStep : (rest > 0 ? (int)rest : 0);
}

// Whether the lane's elements [elem, elem + valid) hold the last element of their tile.
__device__ __forceinline__ bool closes_tile(int64_t n, int64_t tile, int64_t elem, int valid)
{
    int64_t tile_end = (tile + 1) * kZTile;
    if (tile_end > n) tile_end = n;
    return valid > 0 && elem + valid == tile_end;
}

// ---------------------------------------------------------------------------------------------
// A whole tile per wave step: lane l owns the 64 consecutive elements [64 l, 64 l + 64) of the
// tile, as four runs of 16.  The two counting passes (token histogram, tile sizes) only need
// sums over a tile's tokens, so they take a tile in one step: one scan over the wave per tile
// instead of one per 1024 elements.
// ---------------------------------------------------------------------------------------------
template <int R>
struct TileCodes {
    Codes16<R> q[4];
    int valid;                                                 // how many of the lane's 64 elements exist
};

template <int R>
__device__ __forceinline__ void load_tile_codes(const uint8_t *__restrict__ crow, int64_t row_bytes, int64_t n,
                                                int64_t elem, TileCodes<R> &t)
{
    if (n - elem >= 64) {                                      // every lane of a tile inside the row
        const uint8_t *at = crow + ((elem * R) >> 3);
#pragma unroll
        for (int k = 0; k < 4; ++k) t.q[k].load(at + 2 * R * k);
        t.valid = 64;
        return;
    }
    int valid = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) valid += load_step_codes<R>(crow, row_bytes, n, elem + 16 * k, t.q[k]);
    t.valid = valid;
}

// The zeros pending before the lane's first element (already below Z).  Every lane of the wave
// must call it.
template <int R>
__device__ __forceinline__ int tile_run_in(const TileCodes<R> &t, int lane, const ZrunShape &z)
{
    constexpr int kStride = NonZero<R>::kStride;
    // The lane's last non-zero element (position inside the tile), or -1.
    int last = -1;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int valid_k = t.valid - 16 * k;
        valid_k = valid_k < 0 ? 0 : (valid_k > 16 ? 16 : valid_k);
        uint32_t mask = NonZero<R>::mask(t.q[k], z.s);
        if (valid_k < 16) mask &= (1u << (valid_k * kStride)) - 1u;
        if (mask) last = lane * 64 + 16 * k + (31 - __builtin_clz(mask)) / kStride;
    }
    // Inclusive maximum scan over the wave (lanes without a source take -1), then one lane down.
    int incl = last;
    auto step_max = [&](int other) { incl = other > incl ? other : incl; };
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x111, 0xF, 0xF, false));   // row_shr:1
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x112, 0xF, 0xF, false));   // row_shr:2
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x114, 0xF, 0xF, false));   // row_shr:4
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x118, 0xF, 0xF, false));   // row_shr:8
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x142, 0xA, 0xF, false));   // row_bcast:15
    step_max(__builtin_amdgcn_update_dpp(-1, incl, 0x143, 0xC, 0xF, false));   // row_bcast:31
    const int before = __builtin_amdgcn_update_dpp(-1, incl, 0x138, 0xF, 0xF, false);   // wave_shr:1
    const int zeros = lane * 64 - before - 1;                  // (before = -1: the tile starts the run)
    return zeros - (int)(((unsigned int)zeros * z.magic) >> 20) * z.Z;   // zeros < 4096: exact
}

// Tokens of the lane's 64 elements in stream order, given the run pending before them;
// `tile_elems` = elements of the tile (4096, or fewer for the last tile of a row).
template <int R, class Emit>
__device__ __forceinline__ void tile_walk(const TileCodes<R> &t, int lane, int tile_elems, int run, const ZrunShape &z,
                                          Emit &&emit)
{
    const bool closes = t.valid > 0 && lane * 64 + t.valid == tile_elems;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int valid_k = t.valid - 16 * k;
        valid_k = valid_k < 0 ? 0 : (valid_k > 16 ? 16 : valid_k);
        const bool close_k = closes && valid_k > 0 && t.valid - 16 * k <= 16;
        run = lane_tokens<R>(t.q[k], valid_k, run, close_k, z, emit);
    }
}

template <int R, class Emit>
__device__ __forceinline__ void tile_tokens(const TileCodes<R> &t, int lane, int tile_elems, const ZrunShape &z,
                                            Emit &&emit)
{
    tile_walk<R>(t, lane, tile_elems, tile_run_in<R>(t, lane, z), z, emit);
}

// ---------------------------------------------------------------------------------------------
// A sparse tile by way of a position list.  The walks above cost a wave as many rounds as its
// busiest lane has non-zero levels, each round the whole token arithmetic for a few lanes.  A
// tile with few non-zero levels is cheaper in two parts: every lane notes where its non-zero
// levels are (a short loop body), at the places a wave prefix sum of the lanes' counts assigns,
// so that the list is in position order; then the wave takes the list 64 entries at a time, a
// token per lane: the zeros before a level are the distance to the entry before it.
//   list[0] = 0 (stands for position -1), list[i + 1] = (position + 1) | index << 13 for the
//   i-th non-zero level (index: its place among the 2s non-zero levels), list[T + 1] = the
//   tile's element count + 1 (the closing entry: the zeros after the last level).
// ---------------------------------------------------------------------------------------------
constexpr int kZListMax = 1024;                                // non-zero levels of a tile the list holds
constexpr int kZListWords = kZListMax + 2;
static_assert(kZListAt + kZListWords <= kZBufWords, "the list fits the encoder's buffer behind a sparse tile's words");

// Returns the number of non-zero levels T (wave-uniform), or -1 when the list cannot hold them
// (then nothing was written).  Every lane of the wave must call it.
template <int R>
__device__ __forceinline__ int tile_list_build(const TileCodes<R> &t, int lane, int tile_elems, const ZrunShape &z,
                                               unsigned int *__restrict__ list)
{
    constexpr int kStride = NonZero<R>::kStride;
    uint32_t mask[4];
    unsigned int count = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        int valid_k = t.valid - 16 * k;
        valid_k = valid_k < 0 ? 0 : (valid_k > 16 ? 16 : valid_k);
        mask[k] = NonZero<R>::mask(t.q[k], z.s);
        if (valid_k < 16) mask[k] &= (1u << (valid_k * kStride)) - 1u;
        count += (unsigned int)__builtin_popcount(mask[k]);
    }
    const unsigned int incl = wave_inclusive_scan(count);
    const int total = __builtin_amdgcn_readlane((int)incl, 63);
    if (total > kZListMax) return -1;
    unsigned int at = incl - count + 1u;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        uint32_t m = mask[k];
        while (m) {
            const int pos = __builtin_ctz(m) / kStride;
            m &= m - 1u;
            const int c = code_at<R>(t.q[k], pos);
            list[at++] = (unsigned int)(lane * 64 + 16 * k + pos + 1) | ((unsigned int)(c < z.s ? c : c - 1) << 13);
        }
    }
    if (lane == 0) {
        list[0] = 0u;
        list[total + 1] = (unsigned int)tile_elems + 1u;
    }
    wave_lds_sync();
    return total;
}

// The tile's tokens, 64 list entries at a time: emit(have, closing, token, zs) once per round in
// every lane; `have`: the lane has an entry; it stands for `zs` tokens "Z zeros" followed, unless
// `closing`, by `token`.
template <class Emit>
__device__ __forceinline__ void tile_list_tokens(const unsigned int *__restrict__ list, int total, int lane,
                                                 const ZrunShape &z, Emit &&emit)
{
    for (int j0 = 0; j0 <= total; j0 += 64) {
        const int j = j0 + lane;
        const bool have = j <= total;
        const int at = have ? j : total;
        const unsigned int cur = list[at + 1], prev = list[at];
        const unsigned int gap = (cur & 0x1FFFu) - (prev & 0x1FFFu) - 1u;
        // gap <= 4096: exact; the product needs 33 bits when Z = 1
        unsigned int zs = (unsigned int)(((unsigned long long)gap * z.magic) >> 20);
        const unsigned int rest = gap - zs * (unsigned int)z.Z;
        const bool closing = j == total;
        zs += closing && rest > 0u ? 1u : 0u;
        emit(have, closing, (int)(rest * (unsigned int)z.two_s + (cur >> 13)), zs);
    }
}

// ---------------------------------------------------------------------------------------------
// Token counts of every worker row.  A block walks units of 16 tiles of one row (a wave 4
// consecutive tiles of each), counts into one LDS histogram per wave and adds its totals to the
// row's counters once: long-lived blocks, because all blocks of a row end in the same global
// counters.
// ---------------------------------------------------------------------------------------------
constexpr int kZHistBlocks = 2048;                             // target for the whole grid: eight per CU

template <int R>
__global__ void __launch_bounds__(256) k_zrun_histogram(const Args a, const int64_t tiles,
                                                       unsigned long long *__restrict__ counts,
                                                       const int64_t count_stride)
{
    __shared__ unsigned int hist[4][256];
    __shared__ unsigned int lists[4][kZListWords];
    for (int c = threadIdx.x; c < 4 * 256; c += blockDim.x) (&hist[0][0])[c] = 0u;
    __syncthreads();
    const ZrunShape z = zrun_shape(a.s);
    const uint32_t p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    unsigned int *__restrict__ mine = hist[wave];
    const int64_t units = (tiles + kZBlockTiles - 1) / kZBlockTiles;
    for (int64_t unit = blockIdx.x; unit < units; unit += gridDim.x) {
        const int64_t first = unit * kZBlockTiles + wave * kZWaveTiles;
        if (first >= tiles) break;                             // wave-uniform
        // The wave's tiles one after the other, the next tile's codes requested a tile ahead.
        TileCodes<R> cd, cd_next;
        load_tile_codes<R>(crow, a.row_bytes, a.n, first * kZTile + lane * 64, cd_next);
#pragma unroll 1
        for (int i = 0; i < kZWaveTiles; ++i) {
            const int64_t tile = first + i;
            if (tile >= tiles) break;                          // wave-uniform
            cd = cd_next;
            load_tile_codes<R>(crow, a.row_bytes, a.n, (tile + 1) * kZTile + lane * 64, cd_next);
            const int64_t rest = a.n - tile * kZTile;
            const int tile_elems = rest < kZTile ? (int)rest : kZTile;
            const int levels = tile_list_build<R>(cd, lane, tile_elems, z, lists[wave]);
            if (levels >= 0) {
                tile_list_tokens(lists[wave], levels, lane, z, [&](bool have, bool closing, int token, unsigned int zs) {
                    if (have && !closing) atomicAdd(&mine[token & 255], 1u);
                    if (have && zs) atomicAdd(&mine[z.zz], zs);
                });
            } else {
                tile_tokens<R>(cd, lane, tile_elems, z, [&](int token) { atomicAdd(&mine[token & 255], 1u); });
            }
        }
    }
    __syncthreads();
    const int symbols = z.zz + 1;
    for (int c = threadIdx.x; c < symbols; c += blockDim.x) {
        const unsigned int total = hist[0][c] + hist[1][c] + hist[2][c] + hist[3][c];
        if (total) atomicAdd(&counts[(int64_t)p * count_stride + c], (unsigned long long)total);
    }
}

// ---------------------------------------------------------------------------------------------
// Encoder, pass 1: the number of stream bits of every tile.  One block per 16 tiles, a wave 4
// consecutive tiles, a tile per step.
// ---------------------------------------------------------------------------------------------
template <int R>
__global__ void __launch_bounds__(256) k_zrun_tile_bits(const Args a, const uint8_t *__restrict__ lengths,
                                                       const int64_t table_stride, const int64_t tiles,
                                                       uint32_t *__restrict__ tile_bits, const int64_t tile_stride)
{
    __shared__ unsigned char len[256];
    __shared__ unsigned int lists[4][kZListWords];
    const ZrunShape z = zrun_shape(a.s);
    const uint32_t p = blockIdx.y;
    for (int c = threadIdx.x; c < 256; c += blockDim.x) {
        const int l = c <= z.zz ? lengths[(int64_t)p * table_stride + c] : 0;
        len[c] = (unsigned char)(l > kZMaxLen ? kZMaxLen : l);
    }
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    const int64_t first = (int64_t)blockIdx.x * kZBlockTiles + wave * kZWaveTiles;
    if (first >= tiles) return;                                // wave-uniform; no barrier follows
    // The wave's tiles one after the other, the next tile's codes requested a tile ahead.
    TileCodes<R> cd, cd_next;
    load_tile_codes<R>(crow, a.row_bytes, a.n, first * kZTile + lane * 64, cd_next);
#pragma unroll 1
    for (int i = 0; i < kZWaveTiles; ++i) {
        const int64_t tile = first + i;
        if (tile >= tiles) break;                              // wave-uniform
        cd = cd_next;
        load_tile_codes<R>(crow, a.row_bytes, a.n, (tile + 1) * kZTile + lane * 64, cd_next);
        const int64_t rest = a.n - tile * kZTile;
        const int tile_elems = rest < kZTile ? (int)rest : kZTile;
        unsigned int bits = 0;
        const int levels = tile_list_build<R>(cd, lane, tile_elems, z, lists[wave]);
        if (levels >= 0) {
            const unsigned int len_zeros = len[z.zz];
            tile_list_tokens(lists[wave], levels, lane, z, [&](bool have, bool closing, int token, unsigned int zs) {
                bits += have ? zs * len_zeros + (closing ? 0u : (unsigned int)len[token & 255]) : 0u;
            });
        } else {
            tile_tokens<R>(cd, lane, tile_elems, z, [&](int token) { bits += len[token & 255]; });
        }
        const unsigned int incl = wave_inclusive_scan(bits);   // a tile has fewer than 2^32 bits
        if (lane == 63) tile_bits[(int64_t)p * tile_stride + tile] = incl;
    }
}

// ---------------------------------------------------------------------------------------------
// Encoder, pass 2: one block per row walks the tile sizes and leaves the stream bit at which
// every group of 64 tiles starts (entry `groups`: the row's total).  It also clears the 32-bit
// stream word in which every wave of pass 3 starts (every 4th tile) and the one that holds the
// end of the row: those are the words two waves may share, and they fill them with atomic ORs.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) k_zrun_scan(const uint32_t *__restrict__ tile_bits, const int64_t tile_stride,
                                                   const int64_t tiles, unsigned long long *__restrict__ group_offsets,
                                                   const int64_t group_stride, uint32_t *__restrict__ streams,
                                                   const int64_t stream_words, const int64_t stream_stride_words)
{
    __shared__ unsigned long long wave_total[2][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t *__restrict__ sizes = tile_bits + (int64_t)blockIdx.x * tile_stride;
    unsigned long long *__restrict__ offs = group_offsets + (int64_t)blockIdx.x * group_stride;
    uint32_t *__restrict__ out = streams + (int64_t)blockIdx.x * stream_stride_words;
    unsigned long long carry = 0;
    int parity = 0;
    for (int64_t base = 0; base < tiles; base += 1024, parity ^= 1) {
        const int64_t t = base + tid;
        const unsigned int mine = t < tiles ? sizes[t] : 0u;   // a wave's 64 tiles: fewer than 2^32 bits
        const unsigned int incl = wave_inclusive_scan(mine);
        if (lane == 63) wave_total[parity][wave] = incl;
        __syncthreads();                                       // one barrier per chunk: the totals alternate buffers
        unsigned long long before = carry, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const unsigned long long tot = wave_total[parity][w];
            before += w < wave ? tot : 0ull;
            all += tot;
        }
        const unsigned long long off = before + (incl - mine);
        if (t < tiles) {
            if ((t & (kZGroup - 1)) == 0) offs[t / kZGroup] = off;
            if ((t & (kZWaveTiles - 1)) == 0) {
                const unsigned long long word = off >> 5;
                if (word < (unsigned long long)stream_words) out[word] = 0u;
            }
        }
        carry += all;
    }
    if (tid == 0) {
        offs[(tiles + kZGroup - 1) / kZGroup] = carry;
        const unsigned long long word = carry >> 5;
        if ((carry & 31ull) && word < (unsigned long long)stream_words) out[word] = 0u;
    }
}

// ---------------------------------------------------------------------------------------------
// Encoder, pass 3: one block per 16 tiles, a wave 4 consecutive tiles, taken in steps of 1024
// elements (the next step's codes requested a step ahead).  Per step a lane walks its tokens twice: once for the sum of their codeword
// lengths (a wave prefix sum then places every lane), once to put the codewords into the wave's
// LDS buffer, which is aligned with the 32-bit words of the stream.  Whole words leave with
// plain coalesced stores; a partial last word is carried into the next step; only the first
// and last word of the wave's whole range, which a neighbouring wave may share, are filled with
// atomic ORs (pass 2 cleared them).
// ---------------------------------------------------------------------------------------------
struct ZEncodeTable {
    unsigned long long rev[256];     // codeword with its bits reversed: the order they enter the stream
    unsigned int packed[256];        // (length << 24) | reversed codeword, valid when all_short
    unsigned char len[256];
    int all_short;                   // no codeword of the row is longer than 24 bits
};

__device__ __forceinline__ void fill_zencode_table(ZEncodeTable &tab, const uint8_t *__restrict__ lengths,
                                                   const unsigned long long *__restrict__ codewords, int symbols)
{
    if (threadIdx.x == 0) tab.all_short = 1;
    __syncthreads();
    for (int c = threadIdx.x; c < 256; c += blockDim.x) {
        int l = c < symbols ? lengths[c] : 0;
        l = l > kZMaxLen ? kZMaxLen : l;
        unsigned long long cw = (c < symbols && l) ? codewords[c] : 0ull;
        cw &= (1ull << l) - 1ull;
        const unsigned long long rev = l ? (__brevll(cw) >> (64 - l)) : 0ull;
        tab.rev[c] = rev;
        tab.len[c] = (unsigned char)l;
        tab.packed[c] = ((unsigned int)l << 24) | (unsigned int)(rev & 0xFFFFFFull);
        if (l > 24) tab.all_short = 0;                         // benign race: every writer stores 0
    }
    __syncthreads();
}

template <int R>
__global__ void __launch_bounds__(256) k_zrun_write(const Args a, const uint8_t *__restrict__ lengths,
                                                   const unsigned long long *__restrict__ codewords,
                                                   const int64_t table_stride, const int64_t tiles,
                                                   const uint32_t *__restrict__ tile_bits, const int64_t tile_stride,
                                                   const unsigned long long *__restrict__ group_offsets,
                                                   const int64_t group_stride, uint32_t *__restrict__ streams,
                                                   const int64_t stream_words, const int64_t stream_stride_words)
{
    __shared__ ZEncodeTable tab;
    __shared__ unsigned int step_buf[4][kZBufWords];
    const ZrunShape z = zrun_shape(a.s);
    const uint32_t p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t first = (int64_t)blockIdx.x * kZBlockTiles + wave * kZWaveTiles;
    const int64_t group = ((int64_t)blockIdx.x * kZBlockTiles) / kZGroup;
    unsigned int *__restrict__ mine = step_buf[wave];
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    uint32_t *__restrict__ out = streams + (int64_t)p * stream_stride_words;
    // Where the wave's range starts: the group's offset plus the sizes of the group's tiles before it.
    const int64_t my_tile = group * kZGroup + lane;
    const unsigned int my_bits = my_tile < tiles ? tile_bits[(int64_t)p * tile_stride + my_tile] : 0u;
    const unsigned long long group_start = group_offsets[(int64_t)p * group_stride + group];
    // (the first step's codes are requested before the table is built; a wave that goes by whole
    // tiles does not use them)
    Codes16<R> cd, cd_next;
    int valid, valid_next = load_step_codes<R>(crow, a.row_bytes, a.n, first * kZTile + lane * 16, cd_next);
    fill_zencode_table(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, z.zz + 1);
    if (first >= tiles) return;                                // wave-uniform; no block barrier follows
    const unsigned int incl = wave_inclusive_scan(my_bits);
    const unsigned int excl_tile = incl - my_bits;
    const unsigned long long range_start =
        group_start + (unsigned int)__builtin_amdgcn_readlane((int)excl_tile, (int)(first - group * kZGroup));
    // Sparse tiles (at most one bit per element) go a whole tile at a time; see below.
    bool whole_tiles = true;
    for (int i = 0; i < kZWaveTiles; ++i) {
        const unsigned int bits_i =
            (unsigned int)__builtin_amdgcn_readlane((int)my_bits, (int)((first - group * kZGroup + i) & 63));
        whole_tiles = whole_tiles && bits_i <= kZSparseTileBits;
    }
    // The buffer's words that codewords are ORed into start out as zeros (and are cleared again
    // as they leave): all of them, or only the few a sparse tile can fill.
    for (int j = lane; j < (whole_tiles ? kZListAt : kZBufWords); j += 64) mine[j] = 0u;
    wave_lds_sync();

    unsigned long long pos = range_start;                      // bit offset of the current piece
    unsigned int carry = 0;                                    // partial last word of the piece before
    int64_t last_tile = first + kZWaveTiles - 1;
    if (last_tile > tiles - 1) last_tile = tiles - 1;
    const bool all_short = tab.all_short != 0;
    // A piece (a step of 1024 elements, or a whole tile): every lane has `nbits` bits for it; a
    // wave prefix sum places them, `walk(put)` appends the lane's codewords with put(bits,
    // length) into the wave's LDS buffer, which is aligned with the 32-bit words of the stream.
    // Words wholly inside the wave's range then leave with plain stores and their buffer word is
    // cleared for the next piece.  The last word of a piece, when partial, is carried into the
    // first word of the next; only the two ends of the wave's range use atomic ORs.
    // (write_piece in three parts, so that a piece can also be placed token by token.)
    unsigned int piece_shift = 0;
    unsigned long long piece_word0 = 0, piece_end = 0;
    int piece_words = 0;
    auto begin_piece = [&](unsigned int total) {
        piece_shift = (unsigned int)(pos & 31ull);
        piece_word0 = pos >> 5;
        piece_end = pos + total;
        const unsigned int span = (total + piece_shift + 31u) >> 5;
        piece_words = (int)(span < (unsigned int)kZBufWords ? span : (unsigned int)kZBufWords);
    };
    // Appends a lane's bits from bit `at` of the buffer on: put(bits, length) with length <= 32.
    auto place = [&](unsigned int at, auto &&walk) {
        int w = (int)(at >> 5);
        unsigned long long acc = 0;
        unsigned int held = at & 31u;                          // bits of acc below the next free one
        auto put = [&](unsigned int piece, unsigned int l) {   // l <= 32, held < 32
            acc |= (unsigned long long)piece << held;
            held += l;
            if (held >= 32u) {
                if (w < piece_words) atomicOr(&mine[w], (unsigned int)acc);
                ++w;
                acc >>= 32;
                held -= 32u;
            }
        };
        walk(put);
        if (held > 0u && acc != 0ull && w < piece_words) atomicOr(&mine[w], (unsigned int)acc);
    };
    auto end_piece = [&](bool final_piece) {
        const int words = piece_words;
        const unsigned long long word0 = piece_word0, end = piece_end;
        wave_lds_sync();
        const bool has_tail = (end & 31ull) != 0ull;
        if (words > 0) {
            unsigned int tail = mine[words - 1];               // same address for all lanes
            if (words == 1) tail |= carry;
            for (int j = lane; j < words; j += 64) {
                unsigned int value = mine[j];
                mine[j] = 0u;
                if (j == 0) value |= carry;
                const unsigned long long gw = word0 + (unsigned long long)j;
                if (gw >= (unsigned long long)stream_words) continue;
                const bool lower_ok = gw * 32ull >= range_start;
                const bool upper_ok = (gw + 1ull) * 32ull <= end;
                if (lower_ok && upper_ok) out[gw] = value;
                else if (!upper_ok && !final_piece) continue;  // carried below
                else if (value) atomicOr(&out[gw], value);
            }
            carry = has_tail && !final_piece ? tail : 0u;
        }
        wave_lds_sync();                                       // the buffer is clear again for the next piece
        pos = end;
    };
    auto write_piece = [&](unsigned int nbits, auto &&walk, bool final_piece) {
        const unsigned int incl_bits = wave_inclusive_scan(nbits);
        begin_piece((unsigned int)__builtin_amdgcn_readlane((int)incl_bits, 63));
        place(piece_shift + (incl_bits - nbits), walk);
        end_piece(final_piece);
    };
    // One token's codeword, in at most two parts of at most 32 bits.
    auto put_token = [&](auto &put, int token) {
        if (all_short) {
            const unsigned int e = tab.packed[token & 255];
            put(e & 0xFFFFFFu, e >> 24);
        } else {
            unsigned int l = tab.len[token & 255];
            unsigned long long bits = tab.rev[token & 255];
            if (l > 32u) {
                put((unsigned int)bits, 32u);
                bits >>= 32;
                l -= 32u;
            }
            put((unsigned int)bits, l);
        }
    };

    // Sparse tiles (at most one bit per element) go a whole tile at a time, 64 consecutive
    // elements per lane: with few tokens the cost of a piece is its scans and its bookkeeping,
    // and a tile pays them once instead of four times; and the tokens are placed from the list
    // of the tile's non-zero levels, a token per lane, instead of by two walks that cost the wave
    // as many rounds as its busiest lane has levels.  Denser tiles go in steps of 1024 elements,
    // whose bits fit the buffer whatever the code is, and whose tokens' table entries can be kept
    // between the two walks.
    if (whole_tiles) {
        TileCodes<R> tc, tc_next;
        load_tile_codes<R>(crow, a.row_bytes, a.n, first * kZTile + lane * 64, tc_next);
#pragma unroll 1
        for (int i = 0; i < kZWaveTiles; ++i) {
            const int64_t tile = first + i;
            if (tile > last_tile) break;                       // wave-uniform
            tc = tc_next;
            load_tile_codes<R>(crow, a.row_bytes, a.n, (tile + 1) * kZTile + lane * 64, tc_next);
            const int64_t rest = a.n - tile * kZTile;
            const int tile_elems = rest < kZTile ? (int)rest : kZTile;
            unsigned int *__restrict__ list = mine + kZListAt;
            const int levels = tile_list_build<R>(tc, lane, tile_elems, z, list);
            if (levels >= 0) {
                // By the position list: the tile's size is known from pass 1, a wave prefix sum
                // per 64 entries places every lane's token (with the "Z zeros" before it).
                const unsigned int tile_total = (unsigned int)__builtin_amdgcn_readlane(
                    (int)my_bits, (int)((first - group * kZGroup + i) & 63));
                begin_piece(tile_total);
                unsigned int placed = piece_shift;
                const unsigned int len_zeros = tab.len[z.zz];
                tile_list_tokens(list, levels, lane, z, [&](bool have, bool closing, int token, unsigned int zs) {
                    const unsigned int own = closing ? 0u : (unsigned int)tab.len[token & 255];
                    const unsigned int nbits = have ? zs * len_zeros + own : 0u;
                    const unsigned int incl_bits = wave_inclusive_scan(nbits);
                    place(placed + (incl_bits - nbits), [&](auto &put) {
                        if (have) {
                            for (unsigned int k = 0; k < zs; ++k) put_token(put, z.zz);
                            if (!closing) put_token(put, token);
                        }
                    });
                    placed += (unsigned int)__builtin_amdgcn_readlane((int)incl_bits, 63);
                });
                end_piece(tile == last_tile);
                continue;
            }
            const int run = tile_run_in<R>(tc, lane, z);
            unsigned int nbits = 0;
            tile_walk<R>(tc, lane, tile_elems, run, z, [&](int token) { nbits += tab.packed[token & 255] >> 24; });
            write_piece(nbits, [&](auto &put) {
                tile_walk<R>(tc, lane, tile_elems, run, z, [&](int token) { put_token(put, token); });
            }, tile == last_tile);
        }
        return;
    }
    int since = 0;
#pragma unroll 1
    for (int i = 0; i < kZWaveSteps; ++i) {
        const int64_t tile = first + (i / kZSteps);
        const int step = i % kZSteps;
        const int64_t step_first = first * kZTile + (int64_t)i * kZStep;
        const int step_valid = step_elements(a.n, step_first);
        if (tile > last_tile || step_valid == 0) break;        // wave-uniform
        cd = cd_next;
        valid = valid_next;
        valid_next = load_step_codes<R>(crow, a.row_bytes, a.n, step_first + kZStep + lane * 16, cd_next);
        if (step == 0) since = 0;
        const int64_t elem = step_first + lane * 16;
        const int run = lane_run_in<R>(cd, valid, lane, step_valid, since, z);
        const bool close = closes_tile(a.n, tile, elem, valid);
        // First walk: the lane's bits; while no codeword is longer than 24 bits the tokens'
        // table entries are kept (entry k of lane t at [k][t], behind the part of the buffer
        // such codewords can fill), so the second walk need not find the tokens again.
        unsigned int nbits = 0;
        int kept = 0;
        lane_tokens<R>(cd, valid, run, close, z, [&](int token) {
            const unsigned int e = tab.packed[token & 255];
            nbits += e >> 24;
            if (all_short && kept < kZKeepMax) mine[kZKeepAt + kept * 64 + lane] = e;
            ++kept;
        });
        const bool final_step = tile == last_tile && (step == kZSteps - 1 || step_first + kZStep >= a.n);
        write_piece(nbits, [&](auto &put) {
            if (all_short) {
                for (int k = 0; k < kept; ++k) {
                    const unsigned int e = mine[kZKeepAt + k * 64 + lane];
                    put(e & 0xFFFFFFu, e >> 24);
                }
            } else {
                lane_tokens<R>(cd, valid, run, close, z, [&](int token) { put_token(put, token); });
            }
        }, final_step);
    }
}

// ---------------------------------------------------------------------------------------------
// Decoder: one lane per tile, a wave per group of 64 tiles, four groups per block.
// ---------------------------------------------------------------------------------------------
// Decoding a tile is a chain (a token's position is known only once the one before it has been
// decoded), so the work per token is kept small:
//  - `fast` maps the next 12 stream bits to the token whose codeword they begin with, together
//    with what the token stands for: length | zeros << 4 | d << 11 in 16 bits, where d is the
//    XOR of the level's code with the code of level 0 (0 = the token has no level); 0 = the
//    codeword is longer than 12 bits.  Up to 4-bit codes the upper 16 bits describe, in the same
//    form, the token that follows when its codeword also ends inside the 12 bits (0 = none): one
//    lookup then yields two tokens; wider codes keep d in the upper half (8 bits) and get one
//    token per lookup.  (16-bit entries with a second lookup of what the token stands for free
//    LDS for two more blocks per compute unit, but the second lookup lengthens every token's
//    chain: 6-8 % slower at 8 and 16 workers, 8 % faster at 32.)  In a canonical code the
//    codewords, left-aligned,
//    grow with their length, so the length of a longer codeword is 13 plus the number of
//    lengths l >= 13 whose last left-aligned codeword lies below the next 32 stream bits: a
//    count over 20 bounds that every lane keeps in registers (in a wave of 64 tiles some lane
//    meets a rare, long codeword in most rounds, so this route has to be short); beyond 32 bits
//    one bit at a time;
//  - the output is a window of W = 16 or 32 words per lane in LDS that starts out as codes of level 0
//    (a message is mostly zeros); a token moves the output position past its zeros and XORs
//    its level's code into the window.  The lanes of a wave go through their tiles window by
//    window together, so a window leaves with one store sequence for all 64 tiles (lanes that
//    moved theirs on their own made the wave run that sequence for a few lanes at a time,
//    nearly once per token); a token whose level falls beyond the window is held for the next.
struct ZDecodeTable {
    unsigned long long first_code[64];       // canonical: first codeword of each length
    unsigned int fast[1 << kZFastBits];
    unsigned int count[64];                  // codewords of each length
    unsigned int zero_words[8];              // the output's words when every level is 0 (they repeat
                                             // after R / gcd(R, 32) words)
    unsigned int last[33];                   // last left-aligned 32-bit codeword of lengths <= l (wraps to ~0 when none)
    unsigned int delta[33];                  // index into sorted[] minus the codeword, per length
    unsigned short base[64];                 // index into sorted[] of the first one
    unsigned short info[256];                // token -> (zeros << 8) | d (d: see above)
    unsigned short sorted_info[256];         // info of the tokens in the order (length, token)
    unsigned char sorted[256];               // tokens in the order (length, token)
    unsigned char len[256];                  // codeword length of every token (0: does not occur)
};

template <int R>
__device__ __forceinline__ void fill_zdecode_table(ZDecodeTable &tab, const uint8_t *__restrict__ lengths,
                                                   const unsigned long long *__restrict__ codewords,
                                                   const ZrunShape &z)
{
    const int tid = threadIdx.x, symbols = z.zz + 1;
    // The lengths go to LDS first: the loops below read them many times, and a read from global
    // memory inside a loop that every thread of the block walks costs its full latency each time.
    for (int c = tid; c < 256; c += blockDim.x)
        tab.len[c] = (unsigned char)(c < symbols ? (lengths[c] > kZMaxLen ? kZMaxLen : lengths[c]) : 0);
    auto len_of = [&](int c) -> int { return tab.len[c & 255]; };
    for (int l = tid; l < 64; l += blockDim.x) {
        tab.count[l] = 0;
        tab.first_code[l] = 0ull;
    }
    for (int c = tid; c < 256; c += blockDim.x) {
        tab.sorted[c] = (unsigned char)z.zz;
        if (c >= z.zz) {                                       // "Z zeros" (entries beyond it are never reached)
            tab.info[c] = (unsigned short)(z.Z << 8);
        } else {
            const int rank = c % z.two_s, code = rank < z.s ? rank : rank + 1;
            tab.info[c] = (unsigned short)(((c / z.two_s) << 8) | ((code ^ z.s) & ((1 << R) - 1)));
        }
    }
    if (tid < 8) {                                             // bits [32 tid, 32 tid + 32) of the all-zero-level stream
        unsigned int word = 0;
        for (int k = (32 * tid) / R; k * R < 32 * tid + 32; ++k) {
            const int at = k * R - 32 * tid;                   // where field k starts, relative to the word
            word |= at >= 0 ? (unsigned int)z.s << at : (unsigned int)z.s >> -at;
        }
        tab.zero_words[tid] = word;
    }
    __syncthreads();
    for (int c = tid; c < symbols; c += blockDim.x) {
        const int l = len_of(c);
        if (l) atomicAdd(&tab.count[l], 1u);
    }
    __syncthreads();
    for (int l = tid; l < 64; l += blockDim.x) {
        unsigned int at = 0;
        for (int j = 1; j < l; ++j) at += tab.count[j];
        tab.base[l] = (unsigned short)at;
    }
    __syncthreads();
    for (int c = tid; c < symbols; c += blockDim.x) {
        const int l = len_of(c);
        if (!l) continue;
        int rank = 0;
        for (int j = 0; j < c; ++j) rank += len_of(j) == l ? 1 : 0;
        const unsigned long long cw = codewords[c] & ((1ull << l) - 1ull);
        if (rank == 0) tab.first_code[l] = cw;
        const int slot = tab.base[l] + rank;
        if (slot < 256) tab.sorted[slot] = (unsigned char)c;
    }
    for (int c = tid; c < 256; c += blockDim.x) tab.sorted_info[c] = tab.info[z.zz];
    __syncthreads();
    for (int c = tid; c < 256; c += blockDim.x) tab.sorted_info[c] = tab.info[tab.sorted[c]];
    for (int l = tid; l <= 32; l += blockDim.x) {
        // (first codeword of the next occupied length, left-aligned) - 1 = the last codeword of lengths <= l
        unsigned long long bound = 0;                          // left-aligned end of the codewords of lengths <= l
        for (int j = 1; j <= l; ++j)
            if (tab.count[j]) bound = (tab.first_code[j] + tab.count[j]) << (32 - j);
        tab.last[l] = (unsigned int)(bound - 1ull);
        tab.delta[l] = (unsigned int)tab.base[l] - (unsigned int)tab.first_code[l];
    }
    __syncthreads();
    // Every window of kZFastBits stream bits that begins with a codeword of at most that length: in
    // a canonical code the left-aligned codewords grow with their length, so the length is one
    // plus the number of lengths whose last codeword lies below the window (its unknown bits
    // taken as zeros: exact up to kZFastBits bits), and the token follows from the codeword's
    // distance to the first one of its length.  One thread per entry, no walk over the tokens.
    int shortest = 1;                                          // (lengths below it have no last codeword)
    while (shortest <= kZFastBits && tab.count[shortest] == 0u) ++shortest;
    for (unsigned int i = tid; i < (1u << kZFastBits); i += blockDim.x) {
        const unsigned int top = __brev(i);                    // first stream bit on top
        int l = 1;
#pragma unroll
        for (int j = 1; j <= kZFastBits; ++j) l += (j < shortest || top > tab.last[j]) ? 1 : 0;
        unsigned int entry = 0u;
        if (l <= kZFastBits) {
            const unsigned int info = tab.sorted_info[((top >> (32 - l)) + tab.delta[l]) & 255u];
            entry = (unsigned int)l | ((info >> 8) << 4) | ((info & 255u) << (R <= 4 ? 11 : 16));
        }
        tab.fast[i] = entry;
    }
    __syncthreads();
    if constexpr (R <= 4) {
        // The token that follows inside the window: the entry of the window shifted by the first
        // codeword, when both lengths fit 12 bits (then it did not depend on the bits shifted in).
        constexpr int kMine = (1 << kZFastBits) / 256;
        unsigned int second[kMine];
#pragma unroll
        for (int q = 0; q < kMine; ++q) {
            const unsigned int i = (unsigned int)tid + 256u * q;
            const unsigned int first = tab.fast[i];
            const unsigned int next = first ? tab.fast[i >> (first & 15u)] & 0xFFFFu : 0u;
            second[q] = (next && (first & 15u) + (next & 15u) <= (unsigned int)kZFastBits) ? next : 0u;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kMine; ++q) tab.fast[tid + 256 * q] |= second[q] << 16;
        __syncthreads();
    }
}

template <int R, int W>
__global__ void __launch_bounds__(256) k_zrun_decode(const Args a, const uint8_t *__restrict__ lengths,
                                                    const unsigned long long *__restrict__ codewords,
                                                    const int64_t table_stride, const int64_t tiles,
                                                    const uint32_t *__restrict__ tile_bits, const int64_t tile_stride,
                                                    const unsigned long long *__restrict__ group_offsets,
                                                    const int64_t group_stride, const uint32_t *__restrict__ streams,
                                                    const int64_t stream_words, const int64_t stream_stride_words,
                                                    const int lanes_shift)
{
    constexpr int kPeriod = R == 2 || R == 4 || R == 8 ? 1 : (R == 6 ? 3 : R);   // words after which zero_words repeat
    __shared__ ZDecodeTable tab;
    __shared__ unsigned int out_ring[(W + 1) * 256];
    const ZrunShape z = zrun_shape(a.s);
    const uint32_t p = blockIdx.y;
    fill_zdecode_table<R>(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, z);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // A wave takes 64 >> lanes_shift tiles of a group, one per lane of its first lanes: decoding
    // is a chain of dependent instructions, so while the message has too few tiles to fill the
    // chip with whole waves, more waves with idle lanes finish sooner (and a wave waits for the
    // slowest of fewer tiles at every window).
    const int64_t part = (int64_t)blockIdx.x * 4 + wave;       // index of the wave's part of a group
    const int64_t group = part >> lanes_shift;
    if (group * kZGroup >= tiles) return;                      // wave-uniform, after the last barrier
    const int lanes = kZGroup >> lanes_shift;
    const int first = (int)(part & ((1 << lanes_shift) - 1)) * lanes;   // its first tile inside the group
    // All 64 lanes add up the group's tile sizes; lane i then takes the start of tile first + i.
    const int64_t scan_tile = group * kZGroup + lane;
    const unsigned int scan_bits = scan_tile < tiles ? tile_bits[(int64_t)p * tile_stride + scan_tile] : 0u;
    const unsigned int before = wave_inclusive_scan(scan_bits) - scan_bits;
    const unsigned int mine_before = (unsigned int)__shfl((int)before, (first + lane) & 63, 64);
    const int64_t tile = group * kZGroup + first + lane;
    const unsigned long long start = group_offsets[(int64_t)p * group_stride + group] + mine_before;
    if (lane >= lanes || tile >= tiles) return;
    const int64_t elem0 = tile * kZTile;
    const int tile_elems = (int)((a.n - elem0) < kZTile ? (a.n - elem0) : (int64_t)kZTile);
    const uint32_t *__restrict__ in = streams + (int64_t)p * stream_stride_words;
    uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    int64_t out_byte = (elem0 >> 3) * R;                       // a multiple of 512*R: 4-byte aligned in the row

    // Stream words arrive four at a time and a whole batch ahead of their use.  They are addressed
    // by a 32-bit byte offset from the word in which the wave's group starts (one pointer for the
    // wave, no 64-bit arithmetic per lane: the tiles of a group span far less than 2^32 bits).
    // Near the row's end the offsets are clamped to its last word instead of being tested one by
    // one: a message never reads past its own end, and anything else only has to stay inside the
    // row.
    const unsigned long long last_word = (unsigned long long)stream_words - 1ull;
    unsigned long long group_word = group_offsets[(int64_t)p * group_stride + group] >> 5;
    group_word = group_word < last_word ? group_word : last_word;
    group_word = ((unsigned long long)(unsigned int)__builtin_amdgcn_readfirstlane((int)(group_word >> 32)) << 32) |
                 (unsigned int)__builtin_amdgcn_readfirstlane((int)(unsigned int)group_word);
    const char *__restrict__ in_group = reinterpret_cast<const char *>(in + group_word);
    constexpr unsigned int kFarthest = 0x3FFFFFF0u;           // keeps every offset below 2^32
    const unsigned int last_at =
        last_word - group_word < (kFarthest >> 2) ? (unsigned int)(last_word - group_word) << 2 : kFarthest;
    unsigned int next_at =
        (start >> 5) - group_word < (kFarthest >> 2) ? (unsigned int)((start >> 5) - group_word) << 2 : kFarthest;
    auto word_at = [&](unsigned int byte) -> uint32_t { return *reinterpret_cast<const uint32_t *>(in_group + byte); };
    auto fetch4 = [&]() -> uint4 {
        uint4 b;
        if (next_at + 12u <= last_at) {
            b.x = word_at(next_at);
            b.y = word_at(next_at + 4u);
            b.z = word_at(next_at + 8u);
            b.w = word_at(next_at + 12u);
        } else {
            b.x = word_at(next_at + 0u < last_at ? next_at + 0u : last_at);
            b.y = word_at(next_at + 4u < last_at ? next_at + 4u : last_at);
            b.z = word_at(next_at + 8u < last_at ? next_at + 8u : last_at);
            b.w = word_at(next_at + 12u < last_at ? next_at + 12u : last_at);
        }
        next_at += 16u;
        return b;
    };
    uint4 batch = fetch4(), batch_ahead = fetch4();
    int in_batch = 4;
    // The batch in flight becomes the current one and the next is requested.  The hand-over is
    // written as moves that cannot sink below the new loads (the loads' address passes through
    // them): the registers of the old batch are then free to receive the loads.  Left to the
    // compiler, the old values stay live across the loads, the new ones land in other registers
    // and are copied into place at once, which waits for them to arrive: a memory round trip in
    // most token steps of a wave, since its lanes run out of words at different times.
    auto next_batch = [&]() {
        asm volatile("v_mov_b32 %0, %5\n\tv_mov_b32 %1, %6\n\tv_mov_b32 %2, %7\n\tv_mov_b32 %3, %8"
                     : "=&v"(batch.x), "=&v"(batch.y), "=&v"(batch.z), "=&v"(batch.w), "+v"(next_at)
                     : "v"(batch_ahead.x), "v"(batch_ahead.y), "v"(batch_ahead.z), "v"(batch_ahead.w));
        batch_ahead = fetch4();
        in_batch = 4;
    };

    // The output window: words [w0, w0 + W) of the tile's part of the row, the same w0
    // for every lane of the wave.  Word k of lane t at [k][t]: whatever words the lanes of a wave
    // touch, they lie in 64 different banks.  When codes can straddle two words the window has
    // one more word, the first of the next window: an element belongs to the window in which it
    // begins, and what it leaves in that extra word moves on to the next window's word 0.
    constexpr bool kStraddle = (32 % R) != 0;
    unsigned int *__restrict__ ring = out_ring + threadIdx.x;
    auto start_window = [&](int w0) {                          // w0 is the same for the whole wave
        if constexpr (kStraddle) {
            ring[0] = w0 > 0 ? ring[W * 256] : tab.zero_words[0];
#pragma unroll
            for (int k = 1; k <= W; ++k) ring[k * 256] = tab.zero_words[(w0 + k) % kPeriod];
        } else {
#pragma unroll
            for (int k = 0; k < W; ++k)
                ring[k * 256] = tab.zero_words[kPeriod == 1 ? 0 : (w0 + k) % kPeriod];
        }
    };
    // XORs d into element e's field (d == 0: no change).  Only the row within the window is
    // formed from e, so an element outside the window (always with d == 0) touches some row of
    // the lane's own.
    auto put = [&](unsigned int e, unsigned int d) {
        const unsigned int bit = e * R, row = (bit >> 5) & (unsigned int)(W - 1);
        if constexpr (kStraddle) {
            const unsigned long long v = (unsigned long long)d << (bit & 31u);
            atomicXor(&ring[row * 256], (unsigned int)v);
            atomicXor(&ring[(row + 1) * 256], (unsigned int)(v >> 32));
        } else {
            atomicXor(&ring[row * 256], d << (bit & 31u));
        }
    };
    // The bounds of the lengths 13..31 and of length 32, in registers.
    unsigned int last[32 - (kZFastBits + 1)];
#pragma unroll
    for (int j = 0; j < 32 - (kZFastBits + 1); ++j) last[j] = tab.last[kZFastBits + 1 + j];
    const unsigned int last32 = tab.last[32];

    const int tile_bits_out = tile_elems * R;
    const int tile_words = (tile_bits_out + 31) >> 5;
    const bool rows_on_16 = (reinterpret_cast<uintptr_t>(crow) & 15u) == 0u;   // block-uniform
    auto leave_window = [&](const int w0) {
        // The window leaves: whole, or the last words of a ragged tile with its pad bits zero.
        const int count = tile_words - w0 < W ? tile_words - w0 : W;
        if (count > 0) {
            if (w0 + count == tile_words && (tile_bits_out & 31))
                ring[(count - 1) * 256] &= (1u << (tile_bits_out & 31)) - 1u;
            if (count == W && out_byte + 4 * W <= a.row_bytes) {
                if (rows_on_16) {
#pragma unroll
                    for (int q = 0; q < W / 4; ++q) {
                        uint4 v;
                        v.x = ring[(4 * q + 0) * 256];
                        v.y = ring[(4 * q + 1) * 256];
                        v.z = ring[(4 * q + 2) * 256];
                        v.w = ring[(4 * q + 3) * 256];
                        reinterpret_cast<uint4 *>(crow + out_byte)[q] = v;
                    }
                } else {
#pragma unroll
                    for (int k = 0; k < W; ++k)
                        reinterpret_cast<uint32_t *>(crow + out_byte)[k] = ring[k * 256];
                }
            } else {
                for (int k = 0; k < count; ++k)
                    store_code_bytes(crow + out_byte + 4 * k, ring[k * 256], 4, a.row_bytes - (out_byte + 4 * k));
            }
            out_byte += 4 * count;
        }
    };
    // The steps of a token are written without branches: the lanes of a wave are at different
    // tokens, so a branch that one lane takes costs all of them, and decoding is bound by the
    // number of instructions issued.
    //  - the next 32 stream bits are bits [bp, bp + 32) of nxt:cur, bp < 32; a lookup consumes at
    //    most 12 bits (32 for a long codeword), then the pair moves on by a word where due;
    //  - a token whose level begins beyond the window is not taken: it stays in the stream and is
    //    looked up again in the next window (runs are shorter than a window, so it fits there);
    //  - the second token of an entry is taken when its zeros and one more element fit the
    //    window and the tile;
    //  - words that get no level are XORed with 0.
    unsigned int cur = batch.x, nxt = batch.y, bp = (unsigned int)(start & 31ull);
    batch.x = batch.z;
    batch.y = batch.w;
    in_batch = 2;
    auto advance = [&]() {
        const bool step = bp >= 32u;
        cur = step ? nxt : cur;
        nxt = step ? batch.x : nxt;
        batch.x = step ? batch.y : batch.x;
        batch.y = step ? batch.z : batch.y;
        batch.z = step ? batch.w : batch.z;
        in_batch -= step ? 1 : 0;
        bp &= 31u;
        if (in_batch == 0) next_batch();
    };
    unsigned int at = 0;                                       // elements decoded so far
    int held_word = -1;                                        // only codewords beyond 32 bits leave a level behind
    unsigned long long held_bits = 0ull;
    start_window(0);
#pragma unroll 1
    for (int w0 = 0; w0 < kZTile * R / 32; w0 += W) {
        const int w_end = w0 + W;
        const int begin_here = (w_end * 32 + R - 1) / R;     // elements that begin before the window's end
        const unsigned int limit = (unsigned int)(begin_here < tile_elems ? begin_here : tile_elems);
        if (held_word >= 0 && held_word < w_end) {
            atomicXor(&ring[(held_word - w0) * 256], (unsigned int)held_bits);
            if constexpr (kStraddle) atomicXor(&ring[(held_word - w0 + 1) * 256], (unsigned int)(held_bits >> 32));
            held_word = -1;
        }
        bool blocked = false;
        while (at < limit && !blocked) {
            const unsigned int bits = __builtin_amdgcn_alignbit(nxt, cur, bp);
            const unsigned int hit = tab.fast[bits & ((1u << kZFastBits) - 1u)];
            unsigned int len1 = hit & 15u, zeros1 = (hit >> 4) & 127u;
            unsigned int d1 = R <= 4 ? (hit >> 11) & 15u : (hit >> 16) & 255u;
            const unsigned int second = R <= 4 ? hit >> 16 : 0u;
            if (hit == 0u) {
                // Longer than the table covers: its length from the bounds, then its place among the
                // codewords of that length.
                const unsigned int top = __brev(bits);
                int l = kZFastBits + 1;
#pragma unroll
                for (int j = 0; j < 32 - (kZFastBits + 1); ++j) l += top > last[j] ? 1 : 0;
                if (top <= last32) {
                    const unsigned int info = tab.sorted_info[((top >> (32 - l)) + tab.delta[l]) & 255u];
                    len1 = (unsigned int)l;
                    zeros1 = info >> 8;
                    d1 = info & 255u;
                } else {
                    // Beyond 32 bits: one bit at a time, the token applied here.  (A stream that is not of
                    // this code may end up here as well and comes out as "Z zeros" tokens.)
                    unsigned int token = (unsigned int)z.zz;
                    unsigned long long word = top;
                    bp += 32u;
                    advance();
                    for (l = 33; l <= kZMaxLen; ++l) {
                        word = (word << 1) | (unsigned long long)((cur >> bp) & 1u);
                        ++bp;
                        advance();
                        const unsigned long long idx = word - tab.first_code[l];
                        if (tab.count[l] && word >= tab.first_code[l] && idx < tab.count[l]) {
                            token = tab.sorted[(tab.base[l] + (unsigned int)idx) & 255u];
                            break;
                        }
                    }
                    const unsigned int info = tab.info[token];
                    const unsigned int room = (unsigned int)tile_elems - at;   // > 0 inside this loop
                    at += (info >> 8) < room ? (info >> 8) : room;
                    if ((info & 255u) != 0u && at < (unsigned int)tile_elems) {
                        const int bit = (int)at * R, level_word = bit >> 5;
                        if (level_word < w_end) {
                            put(at, info & 255u);
                        } else {
                            held_word = level_word;
                            held_bits = (unsigned long long)(info & 255u) << (bit & 31);
                        }
                        ++at;
                    }
                    continue;
                }
            }
            // (A token that closes a tile has its level beyond the tile's end: it is never taken, and
            // nothing follows it.  An entry without a second token has zeros there: taking it changes
            // nothing.  After a blocked token the test of the second one fails by itself.)
            const unsigned int end1 = at + zeros1;             // where the token's level goes
            const bool put1 = d1 != 0u && end1 < limit;
            blocked = d1 != 0u && end1 >= limit;
            put(end1, put1 ? d1 : 0u);
            const unsigned int at1 = end1 + (put1 ? 1u : 0u);
            const unsigned int zeros2 = (second >> 4) & 127u, d2 = (second >> 11) & 15u;
            const unsigned int end2 = at1 + zeros2;
            const bool take2 = end2 < limit;
            put(end2, take2 ? d2 : 0u);
            const unsigned int at2 = end2 + (d2 != 0u ? 1u : 0u);
            at = blocked ? at : (take2 ? at2 : at1);
            bp += (blocked ? 0u : len1) + (take2 ? second & 15u : 0u);
            advance();
        }
        leave_window(w0);
        start_window(w_end);
    }
}

// ---------------------------------------------------------------------------------------------
// Launchers.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) k_zrun_zero_counts(unsigned long long *counts, int64_t count_stride, int bins)
{
    if ((int)threadIdx.x < bins) counts[(int64_t)blockIdx.x * count_stride + threadIdx.x] = 0ull;
}

hipError_t launch_zrun_histogram(const Args &a, unsigned long long *counts, int64_t count_stride, hipStream_t stream)
{
    const int symbols = 2 * a.s * (127 / a.s) + 1;
    hipLaunchKernelGGL(k_zrun_zero_counts, dim3((unsigned)a.workers), dim3(256), 0, stream, counts, count_stride, symbols);
    const int64_t tiles = (a.n + kZTile - 1) / kZTile;
    unsigned per_row = cdiv(tiles, kZBlockTiles);
    const unsigned want = cdiv(kZHistBlocks, a.workers);
    if (per_row > want) per_row = want;
    const dim3 grid(per_row, (unsigned)a.workers);
#define CALL(RR) hipLaunchKernelGGL((k_zrun_histogram<RR>), grid, dim3(256), 0, stream, a, tiles, counts, count_stride)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_zrun_encode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                              int64_t table_stride, uint32_t *streams, int64_t stream_stride_words,
                              uint32_t *tile_bits, int64_t tile_stride, unsigned long long *group_offsets,
                              int64_t group_stride, hipStream_t stream)
{
    const int64_t tiles = (a.n + kZTile - 1) / kZTile;
    const dim3 grid(cdiv(tiles, kZBlockTiles), (unsigned)a.workers);
#define CALL(RR)                                                                                                  \
    hipLaunchKernelGGL((k_zrun_tile_bits<RR>), grid, dim3(256), 0, stream, a, lengths, table_stride, tiles, tile_bits, \
                       tile_stride)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    hipLaunchKernelGGL(k_zrun_scan, dim3((unsigned)a.workers), dim3(1024), 0, stream, tile_bits, tile_stride, tiles,
                       group_offsets, group_stride, streams, stream_stride_words, stream_stride_words);
#define CALL(RR)                                                                                                   \
    hipLaunchKernelGGL((k_zrun_write<RR>), grid, dim3(256), 0, stream, a, lengths, codewords, table_stride, tiles, \
                       tile_bits, tile_stride, group_offsets, group_stride, streams, stream_stride_words,          \
                       stream_stride_words)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_zrun_decode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                              int64_t table_stride, const uint32_t *streams, int64_t stream_stride_words,
                              const uint32_t *tile_bits, int64_t tile_stride, const unsigned long long *group_offsets,
                              int64_t group_stride, hipStream_t stream)
{
    const int64_t tiles = (a.n + kZTile - 1) / kZTile;
    // Tiles per wave: 64, halved while that still gives every SIMD at most two waves, down to 8:
    // decoding is bound by the instructions a SIMD issues, and a wave costs the same whether 8 or
    // 64 of its lanes decode; only a message too small to give every SIMD work gains from more
    // waves (each a shorter wait for the slowest of its tiles).
    const int64_t held = (int64_t)256 * 4 * 2;
    int lanes_shift = 0;
    while (lanes_shift < 3 && cdiv(tiles, kZGroup >> (lanes_shift + 1)) * a.workers <= held) ++lanes_shift;
    const unsigned row_blocks = cdiv(cdiv(tiles, kZGroup) << lanes_shift, 4);
    const dim3 grid(row_blocks, (unsigned)a.workers);
    // Windows of 32 words: half as many store sequences, each a wait for the stores before it
    // (a wave's loads and stores share one counter), but 52 KB of LDS instead of 36: three blocks
    // per compute unit instead of four.  A message that the chip holds at once with four blocks
    // per unit but not with three keeps the windows of 16 words.
    const int64_t blocks = (int64_t)row_blocks * a.workers;
    const bool narrow = blocks > 256 * 3 && blocks <= 256 * 4;
#define CALL(RR)                                                                                                       \
    if (narrow)                                                                                                        \
        hipLaunchKernelGGL((k_zrun_decode<RR, 16>), grid, dim3(256), 0, stream, a, lengths, codewords, table_stride,  \
                           tiles, tile_bits, tile_stride, group_offsets, group_stride, streams, stream_stride_words, \
                           stream_stride_words, lanes_shift);                                                        \
    else                                                                                                               \
        hipLaunchKernelGGL((k_zrun_decode<RR, 32>), grid, dim3(256), 0, stream, a, lengths, codewords, table_stride,  \
                           tiles, tile_bits, tile_stride, group_offsets, group_stride, streams, stream_stride_words, \
                           stream_stride_words, lanes_shift)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

}  // namespace ecq
