// Huffman coding of the quantised levels on gfx950 (MI355X), wave64.
//
// Section 4 of Wu et al. (ICML 2018) names Huffman encoding as the way to spend fewer than
// r = ceil(log2(2s+1)) bits per element: the levels of one worker's message are far from
// uniform (most are 0), and all of the paper's communication-cost figures assume such a code.
// This file builds the code of every worker row from its level counts d_k, turns the
// fixed-length message into the variable-length one and back.
//
// Conventions (the paper fixes none of them; they are the ones documented in ecq.h):
//   construction  leaves = levels with d_k > 0 numbered by their code c = level + s; the two
//                 live nodes that come first in the order (weight, number) are merged into a
//                 node with the next free number; codeword length = depth (a single occupied
//                 level gets length 1);
//   codewords     canonical: levels sorted by (length, c), first codeword 0, each next one is
//                 (previous + 1) shifted left by the growth in length;
//   stream        LSB-first (stream bit j is bit (j & 7) of byte (j >> 3)), a codeword is
//                 written most significant bit first, pad bits are zero;
//   tiles         a row is cut into tiles of 1024 elements; the bit offset of every tile is
//                 kept so that tiles encode and decode independently.
#include "ecq_device.hpp"
#include "ecq_internal.hpp"

namespace ecq {

constexpr int kTile = ECQ_HUFFMAN_TILE;
constexpr int kMaxLen = 63;                                    // longest codeword handled
// Words of LDS a wave needs to assemble one tile: 1024 codewords of up to 63 bits plus the
// up-to-31-bit shift that aligns the buffer with the 32-bit words of the stream.
constexpr int kTileWords = (kTile * kMaxLen + 31 + 31) / 32 + 1;
constexpr int kFastBits = 10;                                  // decode: direct table on 10 stream bits

static_assert(kTile == 1024, "a wave encodes one tile: 64 lanes x 16 elements");

// ---------------------------------------------------------------------------------------------
// Code construction: one wave per worker row.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_huffman_build(const unsigned long long *__restrict__ counts,
                                                     const int64_t table_stride, const int bins,
                                                     uint8_t *__restrict__ lengths,
                                                     unsigned long long *__restrict__ codewords)
{
    __shared__ unsigned long long weight[512];
    __shared__ unsigned long long first_code[64];
    __shared__ unsigned int len_count[64];
    __shared__ short parent[512];
    __shared__ unsigned char live[512];
    __shared__ unsigned char len_of[256];

    const int lane = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * table_stride;
    for (int i = lane; i < 512; i += 64) {
        const unsigned long long w = i < bins ? counts[row + i] : 0ull;
        weight[i] = w;
        parent[i] = -1;
        live[i] = w > 0 ? 1 : 0;
    }
    len_count[lane] = 0u;
    __syncthreads();

    int alive = 0;
    for (int i = lane; i < bins; i += 64) alive += live[i];
    for (int d = 1; d < 64; d <<= 1) alive += __shfl_xor(alive, d, 64);
    const bool single = alive == 1;

    // alive - 1 merges; node numbers stay below bins + alive - 1 <= 509.
    int nodes = bins;
    while (alive > 1) {
        int pick[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            // First live node in the order (weight, number): lanes scan their nodes in
            // ascending number, so "<" keeps the lowest number among equal weights.
            unsigned long long bw = ~0ull;
            int bi = 0x7FFFFFFF;
            for (int i = lane; i < nodes; i += 64)
                if (live[i] && (bi == 0x7FFFFFFF || weight[i] < bw)) {
                    bw = weight[i];
                    bi = i;
                }
            for (int d = 1; d < 64; d <<= 1) {
                const unsigned long long ow = __shfl_xor(bw, d, 64);
                const int oi = __shfl_xor(bi, d, 64);
                const bool take = oi != 0x7FFFFFFF && (bi == 0x7FFFFFFF || ow < bw || (ow == bw && oi < bi));
                if (take) {
                    bw = ow;
                    bi = oi;
                }
            }
            pick[k] = bi;                                      // the same in every lane
            if (lane == 0 && bi < nodes) live[bi] = 0;
            __syncthreads();
        }
        if (pick[0] >= nodes || pick[1] >= nodes) break;       // cannot happen: alive counts the live nodes
        if (lane == 0) {
            weight[nodes] = weight[pick[0]] + weight[pick[1]];
            parent[pick[0]] = (short)nodes;
            parent[pick[1]] = (short)nodes;
            live[nodes] = 1;
        }
        ++nodes;
        --alive;
        __syncthreads();
    }

    for (int c = lane; c < 256; c += 64) {
        int depth = 0;
        if (c < bins && weight[c] > 0) {
            if (single) depth = 1;
            else
                for (int i = c; parent[i] >= 0; i = parent[i]) ++depth;
        }
        depth = depth > kMaxLen ? kMaxLen : depth;             // cannot happen for counts that sum to <= 2^34
        len_of[c] = (unsigned char)depth;
        if (depth) atomicAdd(&len_count[depth], 1u);
    }
    __syncthreads();
    if (lane == 0) {
        unsigned long long next = 0;
        first_code[0] = 0;
        for (int l = 1; l < 64; ++l) {
            first_code[l] = next;
            next = (next + len_count[l]) << 1;
        }
    }
    __syncthreads();
    for (int c = lane; c < bins; c += 64) {
        const int l = len_of[c];
        unsigned int rank = 0;
        for (int j = 0; j < c; ++j) rank += len_of[j] == l ? 1u : 0u;
        lengths[row + c] = (uint8_t)l;
        codewords[row + c] = l ? first_code[l] + rank : 0ull;
    }
}

// ---------------------------------------------------------------------------------------------
// Encoder.
// ---------------------------------------------------------------------------------------------

// Per-row code table in LDS: length and the codeword with its bits reversed, i.e. in the
// order in which they enter the LSB-first stream.
struct EncodeTable {
    unsigned long long rev[256];
    unsigned char len[256];
};

__device__ __forceinline__ void fill_encode_table(EncodeTable &tab, const uint8_t *__restrict__ lengths,
                                                  const unsigned long long *__restrict__ codewords, int bins)
{
    for (int c = threadIdx.x; c < 256; c += blockDim.x) {
        int l = c < bins ? lengths[c] : 0;
        l = l > kMaxLen ? kMaxLen : l;
        unsigned long long cw = (c < bins && l) ? codewords[c] : 0ull;
        cw &= (1ull << l) - 1ull;
        tab.rev[c] = l ? (__brevll(cw) >> (64 - l)) : 0ull;
        tab.len[c] = (unsigned char)l;
    }
    __syncthreads();
}

// The fixed-length codes of the 16 elements a lane owns inside its tile, as two groups of 8.
template <int R>
__device__ __forceinline__ int load_lane_codes(const uint8_t *__restrict__ crow, int64_t row_bytes, int64_t n,
                                               int64_t elem, uint64_t (&grp)[2])
{
    int64_t rest = n - elem;
    const int valid = rest < 0 ? 0 : (rest > 16 ? 16 : (int)rest);
    grp[0] = valid > 0 ? load_code_group<R>(crow, row_bytes, elem) : 0ull;
    grp[1] = valid > 8 ? load_code_group<R>(crow, row_bytes, elem + 8) : 0ull;
    return valid;
}

template <int R>
__device__ __forceinline__ unsigned int code_at(const uint64_t (&grp)[2], int e)
{
    return (unsigned int)((grp[e >> 3] >> (R * (e & 7))) & ((1u << R) - 1u));
}

// Pass 1: number of stream bits of every tile (a wave per tile, a lane per 16 elements).
template <int R>
__global__ void __launch_bounds__(256) k_huffman_tile_bits(const Args a, const uint8_t *__restrict__ lengths,
                                                          const unsigned long long *__restrict__ codewords,
                                                          const int64_t table_stride, const int64_t tiles,
                                                          unsigned long long *__restrict__ tile_offsets,
                                                          const int64_t offset_stride)
{
    __shared__ EncodeTable tab;
    const uint32_t p = blockIdx.y;
    fill_encode_table(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, 2 * a.s + 1);
    const int lane = threadIdx.x & 63;
    const int64_t tile = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (tile >= tiles) return;                                 // wave-uniform, after the only barrier
    uint64_t grp[2];
    const int valid = load_lane_codes<R>(a.codes + (int64_t)p * a.code_stride, a.row_bytes, a.n,
                                         tile * kTile + lane * 16, grp);
    unsigned int bits = 0;
#pragma unroll
    for (int e = 0; e < 16; ++e) bits += e < valid ? tab.len[code_at<R>(grp, e)] : 0u;
    for (int d = 1; d < 64; d <<= 1) bits += __shfl_xor(bits, d, 64);
    if (lane == 0) tile_offsets[(int64_t)p * offset_stride + tile] = bits;
}

// Pass 2: exclusive prefix sum of the tile sizes of one row (one block per row), in place;
// entry `tiles` receives the total.  Also clears the 32-bit stream word in which each tile
// starts and the one that holds the end of the row: those are the words two tiles may share
// and pass 3 fills them with atomic ORs.
__global__ void __launch_bounds__(1024) k_huffman_scan(unsigned long long *__restrict__ tile_offsets,
                                                      const int64_t offset_stride, const int64_t tiles,
                                                      uint32_t *__restrict__ streams, const int64_t stream_words,
                                                      const int64_t stream_stride_words)
{
    __shared__ unsigned long long wave_total[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    unsigned long long *__restrict__ row = tile_offsets + (int64_t)blockIdx.x * offset_stride;
    uint32_t *__restrict__ out = streams + (int64_t)blockIdx.x * stream_stride_words;
    unsigned long long carry = 0;
    for (int64_t base = 0; base < tiles; base += 4096) {
        const int64_t i0 = base + (int64_t)tid * 4;
        unsigned long long v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = i0 + k < tiles ? row[i0 + k] : 0ull;
        const unsigned long long mine = (v[0] + v[1]) + (v[2] + v[3]);
        unsigned long long incl = mine;
        for (int d = 1; d < 64; d <<= 1) {
            const unsigned long long up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wave_total[wave] = incl;
        __syncthreads();
        unsigned long long before = carry, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const unsigned long long t = wave_total[w];
            before += w < wave ? t : 0ull;
            all += t;
        }
        unsigned long long off = before + (incl - mine);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < tiles) {
                row[i0 + k] = off;
                const unsigned long long word = off >> 5;
                if (word < (unsigned long long)stream_words) out[word] = 0u;
            }
            off += v[k];
        }
        carry += all;
        __syncthreads();                                       // wave_total is reused by the next chunk
    }
    if (tid == 0) {
        row[tiles] = carry;
        const unsigned long long word = carry >> 5;
        if ((carry & 31ull) && word < (unsigned long long)stream_words) out[word] = 0u;
    }
}

// Pass 3: a wave assembles the bits of its tile in LDS, aligned with the 32-bit words of the
// stream, then stores the words: those that lie wholly inside the tile with plain coalesced
// stores, the first and last (which neighbouring tiles may share) with atomic ORs.
template <int R>
__global__ void __launch_bounds__(256) k_huffman_write(const Args a, const uint8_t *__restrict__ lengths,
                                                      const unsigned long long *__restrict__ codewords,
                                                      const int64_t table_stride, const int64_t tiles,
                                                      const unsigned long long *__restrict__ tile_offsets,
                                                      const int64_t offset_stride, uint32_t *__restrict__ streams,
                                                      const int64_t stream_words, const int64_t stream_stride_words)
{
    __shared__ EncodeTable tab;
    __shared__ unsigned int buf[4][kTileWords];
    const uint32_t p = blockIdx.y;
    fill_encode_table(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, 2 * a.s + 1);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t tile = (int64_t)blockIdx.x * 4 + wave;
    const bool active = tile < tiles;                          // wave-uniform

    unsigned long long start = 0, end = 0;
    if (active) {
        start = tile_offsets[(int64_t)p * offset_stride + tile];
        end = tile_offsets[(int64_t)p * offset_stride + tile + 1];
        if (end < start) end = start;
    }
    const unsigned int shift = (unsigned int)(start & 31ull);
    const unsigned long long word0 = start >> 5;
    unsigned long long span = ((end - start) + shift + 31ull) >> 5;
    const int words = (int)(span < (unsigned long long)kTileWords ? span : (unsigned long long)kTileWords);
    unsigned int *__restrict__ mine = buf[wave];
    for (int j = lane; j < words; j += 64) mine[j] = 0u;
    __syncthreads();

    if (active) {
        uint64_t grp[2];
        const int valid = load_lane_codes<R>(a.codes + (int64_t)p * a.code_stride, a.row_bytes, a.n,
                                             tile * kTile + lane * 16, grp);
        unsigned int nbits = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e) nbits += e < valid ? tab.len[code_at<R>(grp, e)] : 0u;
        unsigned int incl = nbits;
        for (int d = 1; d < 64; d <<= 1) {
            const unsigned int up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        // Bit position of this lane's first codeword in the wave's buffer.
        const unsigned int pos = shift + (incl - nbits);
        int w = (int)(pos >> 5);
        unsigned long long acc = 0;
        unsigned int held = pos & 31u;                         // bits of acc below the next free one
#pragma unroll 1
        for (int e = 0; e < valid; ++e) {
            const unsigned int c = code_at<R>(grp, e);
            unsigned int l = tab.len[c];
            unsigned long long bits = tab.rev[c];
            while (l > 0) {                                    // at most two pieces of <= 32 bits
                const unsigned int piece = l > 32u ? 32u : l;
                acc |= (bits & ((1ull << piece) - 1ull)) << held;
                held += piece;
                bits >>= piece;
                l -= piece;
                if (held >= 32u) {
                    if (w < words) atomicOr(&mine[w], (unsigned int)acc);
                    ++w;
                    acc >>= 32;
                    held -= 32u;
                }
            }
        }
        if (held > 0u && acc != 0ull && w < words) atomicOr(&mine[w], (unsigned int)acc);
    }
    __syncthreads();

    if (active) {
        uint32_t *__restrict__ out = streams + (int64_t)p * stream_stride_words;
        for (int j = lane; j < words; j += 64) {
            const unsigned long long gw = word0 + (unsigned long long)j;
            if (gw >= (unsigned long long)stream_words) continue;
            const unsigned int value = mine[j];
            const bool whole = gw * 32ull >= start && (gw + 1ull) * 32ull <= end;
            if (whole) out[gw] = value;
            else if (value) atomicOr(&out[gw], value);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Decoder: one lane per tile.
// ---------------------------------------------------------------------------------------------
struct DecodeTable {
    unsigned long long first_code[64];       // canonical: first codeword of each length
    unsigned short count[64];                // codewords of each length
    unsigned short base[64];                 // index into sorted[] of the first one
    unsigned short fast[1 << kFastBits];     // next 10 stream bits -> (length << 8) | code, 0 = longer
    unsigned char sorted[256];               // codes c in the order (length, c)
};

__device__ __forceinline__ void fill_decode_table(DecodeTable &tab, const uint8_t *__restrict__ lengths,
                                                  const unsigned long long *__restrict__ codewords, int bins)
{
    const int tid = threadIdx.x;
    for (int l = tid; l < 64; l += blockDim.x) {
        tab.count[l] = 0;
        tab.first_code[l] = 0ull;
    }
    for (int i = tid; i < (1 << kFastBits); i += blockDim.x) tab.fast[i] = 0;
    __syncthreads();
    if (tid == 0) {
        // Canonical order: by (length, c).  bins <= 255, so this small serial pass is cheap.
        for (int c = 0; c < bins; ++c) {
            const int l = lengths[c] > kMaxLen ? kMaxLen : lengths[c];
            if (l) tab.count[l] = (unsigned short)(tab.count[l] + 1);
        }
        unsigned short at = 0;
        for (int l = 1; l < 64; ++l) {
            tab.base[l] = at;
            at = (unsigned short)(at + tab.count[l]);
        }
        tab.base[0] = 0;
    }
    __syncthreads();
    for (int c = tid; c < bins; c += blockDim.x) {
        const int l = lengths[c] > kMaxLen ? kMaxLen : lengths[c];
        if (!l) continue;
        int rank = 0;
        bool lowest = true;
        for (int j = 0; j < c; ++j) {
            const int lj = lengths[j] > kMaxLen ? kMaxLen : lengths[j];
            if (lj == l) {
                ++rank;
                lowest = false;
            }
        }
        const unsigned long long cw = codewords[c] & ((1ull << l) - 1ull);
        if (lowest) tab.first_code[l] = cw;
        const int slot = tab.base[l] + rank;
        if (slot < 256) tab.sorted[slot] = (unsigned char)c;
        if (l <= kFastBits) {
            const unsigned int rev = (unsigned int)(__brevll(cw) >> (64 - l));
            for (unsigned int hi = 0; hi < (1u << (kFastBits - l)); ++hi)
                tab.fast[rev | (hi << l)] = (unsigned short)((l << 8) | c);
        }
    }
    __syncthreads();
}

template <int R>
__global__ void __launch_bounds__(64) k_huffman_decode(const Args a, const uint8_t *__restrict__ lengths,
                                                      const unsigned long long *__restrict__ codewords,
                                                      const int64_t table_stride, const int64_t tiles,
                                                      const unsigned long long *__restrict__ tile_offsets,
                                                      const int64_t offset_stride,
                                                      const uint32_t *__restrict__ streams,
                                                      const int64_t stream_words, const int64_t stream_stride_words)
{
    __shared__ DecodeTable tab;
    const uint32_t p = blockIdx.y;
    fill_decode_table(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, 2 * a.s + 1);
    const int64_t tile = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (tile >= tiles) return;
    const int64_t elem0 = tile * kTile;
    const int count = (int)((a.n - elem0) < kTile ? (a.n - elem0) : (int64_t)kTile);
    const uint32_t *__restrict__ in = streams + (int64_t)p * stream_stride_words;
    uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;

    const unsigned long long start = tile_offsets[(int64_t)p * offset_stride + tile];
    unsigned long long next_word = start >> 5;
    // Bit reservoir: `have` valid bits, the next stream bit is bit 0.
    unsigned long long res = 0;
    unsigned int have = 0;
    auto refill = [&]() {
        while (have <= 32u) {
            const unsigned int wv = next_word < (unsigned long long)stream_words ? in[next_word] : 0u;
            ++next_word;
            res |= (unsigned long long)wv << have;
            have += 32u;
        }
    };
    refill();
    {
        const unsigned int skip = (unsigned int)(start & 31ull);
        res >>= skip;
        have -= skip;
    }

    for (int e0 = 0; e0 < count; e0 += 8) {
        uint64_t group = 0;
        const int in_group = count - e0 < 8 ? count - e0 : 8;
        for (int e = 0; e < in_group; ++e) {
            refill();
            unsigned int c;
            const unsigned int hit = tab.fast[(unsigned int)res & ((1u << kFastBits) - 1u)];
            if (hit) {
                c = hit & 0xFFu;
                res >>= (hit >> 8);
                have -= (hit >> 8);
            } else {
                // Longer than the table covers: walk the canonical code one bit at a time.
                unsigned long long word = 0;
                c = 0;
                for (int l = 1; l <= kMaxLen; ++l) {
                    if (have == 0u) refill();
                    word = (word << 1) | (res & 1ull);
                    res >>= 1;
                    --have;
                    const unsigned long long idx = word - tab.first_code[l];
                    if (tab.count[l] && word >= tab.first_code[l] && idx < tab.count[l]) {
                        c = tab.sorted[(tab.base[l] + (unsigned int)idx) & 255u];
                        break;
                    }
                }
            }
            group |= (uint64_t)(c & ((1u << R) - 1u)) << (R * e);
        }
        const int64_t byte_off = ((elem0 + e0) >> 3) * R;
        store_code_bytes(crow + byte_off, group, R, a.row_bytes - byte_off);
    }
}

// ---------------------------------------------------------------------------------------------
// Launchers.
// ---------------------------------------------------------------------------------------------
hipError_t launch_huffman_build(int workers, int bins, const unsigned long long *counts, int64_t table_stride,
                                uint8_t *lengths, unsigned long long *codewords, hipStream_t stream)
{
    hipLaunchKernelGGL(k_huffman_build, dim3((unsigned)workers), dim3(64), 0, stream, counts, table_stride, bins,
                       lengths, codewords);
    return hipGetLastError();
}

hipError_t launch_huffman_encode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                                 int64_t table_stride, uint32_t *streams, int64_t stream_stride_words,
                                 unsigned long long *tile_offsets, int64_t offset_stride, hipStream_t stream)
{
    const int64_t tiles = (a.n + kTile - 1) / kTile;
    const int64_t stream_words = stream_stride_words;
    const dim3 grid(cdiv(tiles, 4), (unsigned)a.workers);
#define CALL(RR)                                                                                               \
    hipLaunchKernelGGL((k_huffman_tile_bits<RR>), grid, dim3(256), 0, stream, a, lengths, codewords, table_stride, \
                       tiles, tile_offsets, offset_stride)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    hipLaunchKernelGGL(k_huffman_scan, dim3((unsigned)a.workers), dim3(1024), 0, stream, tile_offsets, offset_stride,
                       tiles, streams, stream_words, stream_stride_words);
#define CALL(RR)                                                                                               \
    hipLaunchKernelGGL((k_huffman_write<RR>), grid, dim3(256), 0, stream, a, lengths, codewords, table_stride,   \
                       tiles, tile_offsets, offset_stride, streams, stream_words, stream_stride_words)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_huffman_decode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                                 int64_t table_stride, const uint32_t *streams, int64_t stream_stride_words,
                                 const unsigned long long *tile_offsets, int64_t offset_stride, hipStream_t stream)
{
    const int64_t tiles = (a.n + kTile - 1) / kTile;
    const dim3 grid(cdiv(tiles, 64), (unsigned)a.workers);
#define CALL(RR)                                                                                               \
    hipLaunchKernelGGL((k_huffman_decode<RR>), grid, dim3(64), 0, stream, a, lengths, codewords, table_stride,   \
                       tiles, tile_offsets, offset_stride, streams, stream_stride_words, stream_stride_words)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

}  // namespace ecq
