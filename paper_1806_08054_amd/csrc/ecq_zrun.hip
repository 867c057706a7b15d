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
constexpr int kZGroup = ECQ_ZRUN_GROUP;                        // tiles per group = per block of the coders
constexpr int kZStep = 1024;                                   // elements a wave takes at a time (16 per lane)
constexpr int kZSteps = kZTile / kZStep;
constexpr int kZWaveTiles = kZGroup / 4;                       // consecutive tiles per wave
constexpr int kZMaxLen = 63;                                   // longest codeword handled
constexpr int kZFastBits = 10;                                 // decode: direct table on 10 stream bits
constexpr int kZRingWords = 16;                                // decode: words a lane collects before storing
constexpr int kZRingStride = 20;                               // ... and the distance between lanes' rings
// Words of LDS a wave needs for one step: 1024 elements send at most 1025 tokens (every element
// at most one, plus the tile's closing token) of at most 63 bits, plus the up-to-31-bit shift
// that aligns the buffer with the stream's words.
constexpr int kZBufWords = ((kZStep + 1) * kZMaxLen + 31 + 31) / 32 + 1;

static_assert(kZTile == 4096 && kZGroup == 64, "a block of four waves takes one group, a wave 16 tiles");

struct ZrunShape {
    int s, two_s, Z, zz;                                       // zz = 2sZ: the token "Z zeros"
};

__device__ __forceinline__ ZrunShape zrun_shape(int s)
{
    ZrunShape z;
    z.s = s;
    z.two_s = 2 * s;
    z.Z = 127 / s;
    z.zz = 2 * s * z.Z;
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
    int incl = last;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int below = __shfl_up(incl, d, 64);
        if (lane >= d) incl = below > incl ? below : incl;
    }
    int before = __shfl_up(incl, 1, 64);
    if (lane == 0) before = -1;
    const int zeros = before >= 0 ? lane * 16 - before - 1 : since + lane * 16;
    const int wave_last = __builtin_amdgcn_readlane(incl, 63);
    since = wave_last >= 0 ? step_valid - wave_last - 1 : since + step_valid;
    return zeros % z.Z;
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
// Token counts of every worker row.  A block walks groups of 64 tiles of one row (a wave 16
// consecutive tiles of each), counts into one LDS histogram per wave and adds its totals to the
// row's counters once: few, long-lived blocks, because all blocks of a row end in the same
// global counters.
// ---------------------------------------------------------------------------------------------
constexpr int kZHistBlocks = 768;                              // target for the whole grid: three per CU

template <int R>
__global__ void __launch_bounds__(256) k_zrun_histogram(const Args a, const int64_t tiles,
                                                       unsigned long long *__restrict__ counts,
                                                       const int64_t count_stride)
{
    __shared__ unsigned int hist[4][256];
    for (int c = threadIdx.x; c < 4 * 256; c += blockDim.x) (&hist[0][0])[c] = 0u;
    __syncthreads();
    const ZrunShape z = zrun_shape(a.s);
    const uint32_t p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    unsigned int *__restrict__ mine = hist[wave];
    const int64_t groups = (tiles + kZGroup - 1) / kZGroup;
    for (int64_t group = blockIdx.x; group < groups; group += gridDim.x) {
        const int64_t first = group * kZGroup + wave * kZWaveTiles;
#pragma unroll 1
        for (int t = 0; t < kZWaveTiles; ++t) {
            const int64_t tile = first + t;
            if (tile >= tiles) break;                          // wave-uniform
            int since = 0;
#pragma unroll 1
            for (int step = 0; step < kZSteps; ++step) {
                const int64_t step_first = tile * kZTile + (int64_t)step * kZStep;
                const int step_valid = step_elements(a.n, step_first);
                if (step_valid == 0) break;                    // wave-uniform
                const int64_t elem = step_first + lane * 16;
                Codes16<R> cd;
                const int valid = load_step_codes<R>(crow, a.row_bytes, a.n, elem, cd);
                const int run = lane_run_in<R>(cd, valid, lane, step_valid, since, z);
                lane_tokens<R>(cd, valid, run, closes_tile(a.n, tile, elem, valid), z,
                               [&](int token) { atomicAdd(&mine[token & 255], 1u); });
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
// Encoder, pass 1: the number of stream bits of every tile.  One block per group of 64 tiles, a
// wave 16 consecutive tiles.
// ---------------------------------------------------------------------------------------------
template <int R>
__global__ void __launch_bounds__(256) k_zrun_tile_bits(const Args a, const uint8_t *__restrict__ lengths,
                                                       const int64_t table_stride, const int64_t tiles,
                                                       uint32_t *__restrict__ tile_bits, const int64_t tile_stride)
{
    __shared__ unsigned char len[256];
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
    const int64_t first = (int64_t)blockIdx.x * kZGroup + wave * kZWaveTiles;
#pragma unroll 1
    for (int t = 0; t < kZWaveTiles; ++t) {
        const int64_t tile = first + t;
        if (tile >= tiles) break;                              // wave-uniform
        int since = 0;
        unsigned int bits = 0;
#pragma unroll 1
        for (int step = 0; step < kZSteps; ++step) {
            const int64_t step_first = tile * kZTile + (int64_t)step * kZStep;
            const int step_valid = step_elements(a.n, step_first);
            if (step_valid == 0) break;                        // wave-uniform
            const int64_t elem = step_first + lane * 16;
            Codes16<R> cd;
            const int valid = load_step_codes<R>(crow, a.row_bytes, a.n, elem, cd);
            const int run = lane_run_in<R>(cd, valid, lane, step_valid, since, z);
            lane_tokens<R>(cd, valid, run, closes_tile(a.n, tile, elem, valid), z,
                           [&](int token) { bits += len[token & 255]; });
        }
        const unsigned int incl = wave_inclusive_scan(bits);   // a tile has fewer than 2^32 bits
        if (lane == 63) tile_bits[(int64_t)p * tile_stride + tile] = incl;
    }
}

// ---------------------------------------------------------------------------------------------
// Encoder, pass 2: one block per row walks the tile sizes and leaves the stream bit at which
// every group of 64 tiles starts (entry `groups`: the row's total).  It also clears the 32-bit
// stream word in which every wave of pass 3 starts (every 16th tile) and the one that holds the
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
// Encoder, pass 3: one block per group of 64 tiles, a wave 16 consecutive tiles, taken in steps
// of 1024 elements.  Per step a lane walks its tokens twice: once for the sum of their codeword
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
    const int64_t group = blockIdx.x;
    const int64_t first = group * kZGroup + wave * kZWaveTiles;
    unsigned int *__restrict__ mine = step_buf[wave];
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    uint32_t *__restrict__ out = streams + (int64_t)p * stream_stride_words;
    // Where the wave's range starts: the group's offset plus the sizes of the group's tiles before it.
    const int64_t my_tile = group * kZGroup + lane;
    const unsigned int my_bits = my_tile < tiles ? tile_bits[(int64_t)p * tile_stride + my_tile] : 0u;
    const unsigned long long group_start = group_offsets[(int64_t)p * group_stride + group];
    fill_zencode_table(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, z.zz + 1);
    if (first >= tiles) return;                                // wave-uniform; no block barrier follows
    const unsigned int incl = wave_inclusive_scan(my_bits);
    const unsigned int excl_tile = incl - my_bits;
    const unsigned long long range_start =
        group_start + (unsigned int)__builtin_amdgcn_readlane((int)excl_tile, wave * kZWaveTiles);
    for (int j = lane; j < kZBufWords; j += 64) mine[j] = 0u;
    wave_lds_sync();

    unsigned long long pos = range_start;                      // bit offset of the current step
    unsigned int carry = 0;                                    // partial last word of the step before
    int64_t last_tile = first + kZWaveTiles - 1;
    if (last_tile > tiles - 1) last_tile = tiles - 1;
#pragma unroll 1
    for (int64_t tile = first; tile <= last_tile; ++tile) {
        int since = 0;
#pragma unroll 1
        for (int step = 0; step < kZSteps; ++step) {
            const int64_t step_first = tile * kZTile + (int64_t)step * kZStep;
            const int step_valid = step_elements(a.n, step_first);
            if (step_valid == 0) break;                        // wave-uniform
            const int64_t elem = step_first + lane * 16;
            Codes16<R> cd;
            const int valid = load_step_codes<R>(crow, a.row_bytes, a.n, elem, cd);
            const int run = lane_run_in<R>(cd, valid, lane, step_valid, since, z);
            const bool close = closes_tile(a.n, tile, elem, valid);
            unsigned int nbits = 0;
            lane_tokens<R>(cd, valid, run, close, z, [&](int token) { nbits += tab.len[token & 255]; });
            const unsigned int incl_bits = wave_inclusive_scan(nbits);
            const unsigned int total = (unsigned int)__builtin_amdgcn_readlane((int)incl_bits, 63);
            const unsigned int shift = (unsigned int)(pos & 31ull);
            const unsigned long long word0 = pos >> 5;
            const unsigned long long end = pos + total;
            const unsigned int span = (total + shift + 31u) >> 5;
            const int words = (int)(span < (unsigned int)kZBufWords ? span : (unsigned int)kZBufWords);

            // The lane's codewords, from buffer bit shift + (bits of the lanes before it).
            {
                const unsigned int at = shift + (incl_bits - nbits);
                int w = (int)(at >> 5);
                unsigned long long acc = 0;
                unsigned int held = at & 31u;                  // bits of acc below the next free one
                auto put = [&](unsigned int piece, unsigned int l) {   // l <= 32, held < 32
                    acc |= (unsigned long long)piece << held;
                    held += l;
                    if (held >= 32u) {
                        if (w < words) atomicOr(&mine[w], (unsigned int)acc);
                        ++w;
                        acc >>= 32;
                        held -= 32u;
                    }
                };
                const bool all_short = tab.all_short != 0;
                lane_tokens<R>(cd, valid, run, close, z, [&](int token) {
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
                });
                if (held > 0u && acc != 0ull && w < words) atomicOr(&mine[w], (unsigned int)acc);
            }
            wave_lds_sync();

            // Words wholly inside the wave's range leave with plain stores and their buffer word
            // is cleared for the next step.  The last word of a step, when partial, is carried
            // into the first word of the next step; only the two ends of the range use atomic ORs.
            const bool final_step = tile == last_tile && (step == kZSteps - 1 || step_first + kZStep >= a.n);
            const bool has_tail = (end & 31ull) != 0ull;
            if (words > 0) {
                unsigned int tail = mine[words - 1];           // same address for all lanes
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
                    else if (!upper_ok && !final_step) continue;   // carried below
                    else if (value) atomicOr(&out[gw], value);
                }
                carry = has_tail && !final_step ? tail : 0u;
            }
            wave_lds_sync();                                   // the buffer is clear again for the next step
            pos = end;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Decoder: one lane per tile, a wave per group of 64 tiles, four groups per block.
// ---------------------------------------------------------------------------------------------
// `fast` maps the next 10 stream bits to the token whose codeword they begin with (length in
// the high byte; 0 = longer than 10 bits); longer codewords are found by the canonical
// first-code / count test on the next 32 stream bits, and one bit at a time beyond that.
struct ZDecodeTable {
    unsigned long long first_code[64];       // canonical: first codeword of each length
    unsigned int count[64];                  // codewords of each length
    unsigned short base[64];                 // index into sorted[] of the first one
    unsigned short fast[1 << kZFastBits];    // (length << 8) | token
    unsigned char sorted[256];               // tokens in the order (length, token)
    unsigned char zeros[256];                // zeros a token stands for
    unsigned char code[256];                 // the code (level + s) that follows them; 255: none
};

__device__ __forceinline__ void fill_zdecode_table(ZDecodeTable &tab, const uint8_t *__restrict__ lengths,
                                                   const unsigned long long *__restrict__ codewords,
                                                   const ZrunShape &z)
{
    const int tid = threadIdx.x, symbols = z.zz + 1;
    auto len_of = [&](int c) -> int { return c < symbols ? (lengths[c] > kZMaxLen ? kZMaxLen : lengths[c]) : 0; };
    for (int l = tid; l < 64; l += blockDim.x) {
        tab.count[l] = 0;
        tab.first_code[l] = 0ull;
    }
    for (int i = tid; i < (1 << kZFastBits); i += blockDim.x) tab.fast[i] = 0;
    for (int c = tid; c < 256; c += blockDim.x) {
        tab.sorted[c] = (unsigned char)z.zz;
        if (c >= z.zz) {                                       // "Z zeros" (entries beyond it are never reached)
            tab.zeros[c] = (unsigned char)z.Z;
            tab.code[c] = 255;
        } else {
            const int rank = c % z.two_s;
            tab.zeros[c] = (unsigned char)(c / z.two_s);
            tab.code[c] = (unsigned char)(rank < z.s ? rank : rank + 1);
        }
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
    // Every window whose low bits are a codeword of at most kZFastBits bits.
    for (int c = 0; c < symbols; ++c) {
        const int l = len_of(c);
        if (!l || l > kZFastBits) continue;                    // block-uniform
        const unsigned long long cw = codewords[c] & ((1ull << l) - 1ull);
        const unsigned int rev = (unsigned int)(__brevll(cw) >> (64 - l));
        for (unsigned int hi = tid; hi < (1u << (kZFastBits - l)); hi += blockDim.x)
            tab.fast[rev | (hi << l)] = (unsigned short)((l << 8) | c);
    }
    __syncthreads();
}

template <int R>
__global__ void __launch_bounds__(256) k_zrun_decode(const Args a, const uint8_t *__restrict__ lengths,
                                                    const unsigned long long *__restrict__ codewords,
                                                    const int64_t table_stride, const int64_t tiles,
                                                    const uint32_t *__restrict__ tile_bits, const int64_t tile_stride,
                                                    const unsigned long long *__restrict__ group_offsets,
                                                    const int64_t group_stride, const uint32_t *__restrict__ streams,
                                                    const int64_t stream_words, const int64_t stream_stride_words)
{
    __shared__ ZDecodeTable tab;
    __shared__ __attribute__((aligned(16))) unsigned int out_ring[256 * kZRingStride];
    const ZrunShape z = zrun_shape(a.s);
    const uint32_t p = blockIdx.y;
    fill_zdecode_table(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, z);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t group = (int64_t)blockIdx.x * 4 + wave;
    if (group * kZGroup >= tiles) return;                      // wave-uniform, after the last barrier
    const int64_t tile = group * kZGroup + lane;
    const unsigned int my_bits = tile < tiles ? tile_bits[(int64_t)p * tile_stride + tile] : 0u;
    const unsigned int incl = wave_inclusive_scan(my_bits);
    const unsigned long long start = group_offsets[(int64_t)p * group_stride + group] + (incl - my_bits);
    if (tile >= tiles) return;
    const int64_t elem0 = tile * kZTile;
    int remaining = (int)((a.n - elem0) < kZTile ? (a.n - elem0) : (int64_t)kZTile);
    const uint32_t *__restrict__ in = streams + (int64_t)p * stream_stride_words;
    uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    int64_t out_byte = (elem0 >> 3) * R;                       // a multiple of 512*R: 4-byte aligned in the row

    // Bit reservoir: `have` valid bits, the next stream bit is bit 0.  Stream words arrive four
    // at a time and a whole batch ahead of their use.  Indices are clamped to the row's last word
    // instead of being tested one by one: a message never reads past its own end, and anything
    // else only has to stay inside the row.
    unsigned long long next_word = start >> 5;
    const unsigned long long last_word = (unsigned long long)stream_words - 1ull;
    auto fetch4 = [&]() -> uint4 {
        uint4 b;
        b.x = in[next_word + 0 < last_word ? next_word + 0 : last_word];
        b.y = in[next_word + 1 < last_word ? next_word + 1 : last_word];
        b.z = in[next_word + 2 < last_word ? next_word + 2 : last_word];
        b.w = in[next_word + 3 < last_word ? next_word + 3 : last_word];
        next_word += 4;
        return b;
    };
    uint4 batch = fetch4(), batch_ahead = fetch4();
    int in_batch = 4;
    auto take = [&]() -> unsigned int {
        if (in_batch == 0) {
            batch = batch_ahead;
            batch_ahead = fetch4();
            in_batch = 4;
        }
        const unsigned int wv = batch.x;
        batch.x = batch.y; batch.y = batch.z; batch.z = batch.w;
        --in_batch;
        return wv;
    };
    unsigned long long res = take();
    unsigned int have = 32u;
    auto refill = [&]() {
        if (have <= 32u) {
            res |= (unsigned long long)take() << have;
            have += 32u;
        }
    };
    {
        const unsigned int skip = (unsigned int)(start & 31ull);
        res >>= skip;
        have -= skip;
    }

    // Decoded codes collect in a 64-bit accumulator, whole words go to a per-lane LDS ring and
    // leave 64 bytes at a time.
    unsigned long long out_acc = 0;
    unsigned int out_held = 0;
    unsigned int *__restrict__ ring = out_ring + threadIdx.x * kZRingStride;
    int ring_at = 0;
    auto flush_ring = [&](int count) {
        if (count == kZRingWords && out_byte + 4 * kZRingWords <= a.row_bytes) {
#pragma unroll
            for (int q = 0; q < kZRingWords / 4; ++q) {
                const uint4 v = *reinterpret_cast<const uint4 *>(&ring[4 * q]);
                uint32_t *dst = reinterpret_cast<uint32_t *>(crow + out_byte) + 4 * q;
                dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
            }
        } else {
            for (int k = 0; k < count; ++k)
                store_code_bytes(crow + out_byte + 4 * k, ring[k], 4, a.row_bytes - (out_byte + 4 * k));
        }
        out_byte += 4 * count;
    };
    auto push_words = [&]() {                                  // move whole words of out_acc to the ring
        while (out_held >= 32u) {
            ring[ring_at++] = (unsigned int)out_acc;
            out_acc >>= 32;
            out_held -= 32u;
            if (ring_at == kZRingWords) {
                flush_ring(kZRingWords);
                ring_at = 0;
            }
        }
    };
    // A 64-bit word full of codes of level 0 (c = s in every R-bit field that fits whole).
    constexpr int kFieldsPerWord = 32 / R;                     // zeros appended per round: they fit 32 bits
    unsigned int zero_fields = 0;
#pragma unroll
    for (int k = 0; k < kFieldsPerWord; ++k) zero_fields |= (unsigned int)a.s << (R * k);

    while (remaining > 0) {
        refill();
        unsigned int token;
        const unsigned int hit = tab.fast[(unsigned int)res & ((1u << kZFastBits) - 1u)];
        if (hit) {
            token = hit & 0xFFu;
            res >>= (hit >> 8);
            have -= (hit >> 8);
        } else {
            // Longer than the table covers.  Up to 32 bits: the next 32 stream bits, first one on
            // top, give the candidate codeword of every length by one shift; the canonical code
            // says which length holds it.
            token = (unsigned int)z.zz;
            if (have < 32u) refill();
            const unsigned int top = __brev((unsigned int)res);
            int l = kZFastBits + 1;
            bool found = false;
            for (; l <= 32; ++l) {
                const unsigned long long cand = top >> (32 - l);
                const unsigned long long idx = cand - tab.first_code[l];
                if (tab.count[l] && cand >= tab.first_code[l] && idx < tab.count[l]) {
                    token = tab.sorted[(tab.base[l] + (unsigned int)idx) & 255u];
                    res >>= l;
                    have -= (unsigned int)l;
                    found = true;
                    break;
                }
            }
            if (!found) {
                // Beyond 32 bits: one bit at a time.  (A stream that is not of this code ends up
                // here as well and comes out as "Z zeros" tokens.)
                unsigned long long word = top;
                res >>= 32;
                have -= 32u;
                for (l = 33; l <= kZMaxLen; ++l) {
                    if (have == 0u) refill();
                    word = (word << 1) | (res & 1ull);
                    res >>= 1;
                    --have;
                    const unsigned long long idx = word - tab.first_code[l];
                    if (tab.count[l] && word >= tab.first_code[l] && idx < tab.count[l]) {
                        token = tab.sorted[(tab.base[l] + (unsigned int)idx) & 255u];
                        break;
                    }
                }
            }
        }
        int zeros = tab.zeros[token];
        const unsigned int code = tab.code[token];
        zeros = zeros < remaining ? zeros : remaining;
        remaining -= zeros;
        while (zeros > 0) {                                    // up to 32 / R zeros per round
            const int m = zeros < kFieldsPerWord ? zeros : kFieldsPerWord;
            const unsigned int fields = (R * m) >= 32 ? zero_fields : (zero_fields & ((1u << (R * m)) - 1u));
            out_acc |= (unsigned long long)fields << out_held;
            out_held += (unsigned int)(R * m);
            zeros -= m;
            push_words();
        }
        if (code != 255u && remaining > 0) {
            out_acc |= (unsigned long long)(code & ((1u << R) - 1u)) << out_held;
            out_held += R;
            --remaining;
            push_words();
        }
    }
    // What is left of a ragged last tile: whole words, then fewer than 32 bits (pad bits zero).
    flush_ring(ring_at);
    if (out_held > 0u && out_byte < a.row_bytes)
        store_code_bytes(crow + out_byte, out_acc, (int)((out_held + 7u) >> 3), a.row_bytes - out_byte);
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
    unsigned per_row = cdiv(tiles, kZGroup);
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
    const dim3 grid(cdiv(tiles, kZGroup), (unsigned)a.workers);
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
    const dim3 grid(cdiv(cdiv(tiles, kZGroup), 4), (unsigned)a.workers);
#define CALL(RR)                                                                                                    \
    hipLaunchKernelGGL((k_zrun_decode<RR>), grid, dim3(256), 0, stream, a, lengths, codewords, table_stride, tiles, \
                       tile_bits, tile_stride, group_offsets, group_stride, streams, stream_stride_words,           \
                       stream_stride_words)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

}  // namespace ecq
