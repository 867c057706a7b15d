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
constexpr int kFastBits = 10;                                  // decode: direct table on 10 stream bits
constexpr int kRunTiles = 16;                                  // encoder: consecutive tiles (one "run") per wave
constexpr int kRunElems = kRunTiles * ECQ_HUFFMAN_TILE;
constexpr int kDecodeThreads = 256;                            // decode: tiles (lanes) per block
constexpr int kRingWords = 16;                                 // decode: words a lane collects before storing

// The encoder's waves take a run in steps of 64 lanes x 16*Q elements: Q = 4 (four tiles per
// step) while codes have at most 4 bits, fewer for wider codes, whose codewords can be longer,
// so that a step's bits always fit the wave's LDS buffer.
template <int R>
constexpr int kStepGroups = R <= 4 ? 4 : (R == 5 ? 2 : 1);
static inline int step_groups(int r) { return r <= 4 ? 4 : (r == 5 ? 2 : 1); }

// Words of LDS a wave needs for one step when no codeword is longer than max_len bits: the
// step's codewords plus the up-to-31-bit shift that aligns the buffer with the stream's words.
static inline int step_buffer_words(int r, int max_len)
{
    return (kTile * step_groups(r) * max_len + 31 + 31) / 32 + 1;
}

static_assert(kTile == 1024, "a step is 64 lanes x 16*Q elements = Q tiles");

// ---------------------------------------------------------------------------------------------
// Code construction: one wave per worker row.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(64) k_huffman_build(const unsigned long long *__restrict__ counts,
                                                     const int64_t table_stride, const int bins,
                                                     uint8_t *__restrict__ lengths,
                                                     unsigned long long *__restrict__ codewords)
{
    __shared__ unsigned long long weight[256];                 // of the levels
    __shared__ unsigned long long first_code[64];
    __shared__ unsigned long long leaf_key[256 + 4];           // occupied levels in the order (weight, number), then ~0
    __shared__ unsigned long long made_key[256 + 4];           // merged nodes in the order they are made, then ~0
    __shared__ unsigned long long node_key[256];               // every level's key, ~0 when it does not occur
    __shared__ unsigned int len_count[64];
    __shared__ short parent[512];
    __shared__ unsigned char len_of[256];

    const int lane = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * table_stride;
    for (int i = lane; i < 512; i += 64) {
        if (i < 256) weight[i] = i < bins ? counts[row + i] : 0ull;
        parent[i] = -1;
    }
    len_count[lane] = 0u;
    __syncthreads();

    // A node's place in the order (weight, number) as one integer: weights stay below 2^35 (a
    // row sums to at most 2^34), numbers below 2^9.
    auto key_of = [&](int node) -> unsigned long long { return (weight[node] << 9) | (unsigned long long)node; };
    // Sort the occupied levels by counting, for every one, the occupied levels before it: a lane
    // takes up to four levels at once, so every key read from LDS serves four comparisons, and the
    // reads of several steps are in flight together (one wave: nothing else hides their latency).
    for (int i = lane; i < 256; i += 64) node_key[i] = (i < bins && weight[i] != 0ull) ? key_of(i) : ~0ull;
    __syncthreads();
    const int bins_up = (bins + 7) & ~7;                       // the loops over all levels go in steps of 8 (<= 256)
    int alive = 0;
    {
        unsigned long long mine[4];
        int rank[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            mine[q] = node_key[lane + 64 * q];
            rank[q] = 0;
            alive += mine[q] != ~0ull ? 1 : 0;
        }
#pragma unroll 8
        for (int j = 0; j < bins_up; ++j) {
            const unsigned long long other = node_key[j];      // an unoccupied level: the largest key, before nothing
#pragma unroll
            for (int q = 0; q < 4; ++q) rank[q] += other < mine[q] ? 1 : 0;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (mine[q] != ~0ull) leaf_key[rank[q]] = mine[q];
    }
    for (int d = 1; d < 64; d <<= 1) alive += __shfl_xor(alive, d, 64);
    const bool single = alive == 1;
    for (int i = lane; i < 256 + 4; i += 64) {                  // (ranks stay below `alive`: no entry is written twice)
        if (i >= alive) leaf_key[i] = ~0ull;
        made_key[i] = ~0ull;
    }
    __syncthreads();

    // The two nodes that come first in the order (weight, number) are merged into a node with
    // the next free number, alive - 1 times (numbers stay below bins + alive - 1 <= 509).  The
    // merged nodes come into being in that very order (their weights never decrease, their
    // numbers grow), so the first of all live nodes is always the first leaf not yet taken or
    // the first merged node not yet taken: one lane walks the two queues.
    // The walk is a chain of dependent steps of one lane, so it is written without branches and
    // without waits: the first two keys of each queue travel in registers, the third is requested
    // from LDS a pick before it can be needed (both queues, whichever moves), and a node made
    // while such a request is in flight is put in its place from registers.  A key holds the
    // node's weight: nothing else is read back.
    if (lane == 0) {
        int next_leaf = 0, next_made = 0, made = 0;
        unsigned long long l0 = leaf_key[0], l1 = leaf_key[1], l2 = leaf_key[2];
        unsigned long long m0 = ~0ull, m1 = ~0ull, m2 = ~0ull;
        bool m2_new = false;                                   // the third merged node was made after its request:
        unsigned long long m2_key = ~0ull;                     // this is its key
        for (int m = 0; m + 1 < alive; ++m) {
            unsigned long long pick[2];
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const unsigned long long third = m2_new ? m2_key : m2;
                const bool leaf = l0 < m0;
                pick[k] = leaf ? l0 : m0;
                l0 = leaf ? l1 : l0;
                l1 = leaf ? l2 : l1;
                m0 = leaf ? m0 : m1;
                m1 = leaf ? m1 : third;
                next_leaf += leaf ? 1 : 0;
                next_made += leaf ? 0 : 1;
                l2 = leaf_key[next_leaf + 2];
                m2 = made_key[next_made + 2];                  // (requested after the last node was stored)
                m2_new = false;
            }
            const int node = bins + made;
            const unsigned long long sum = (pick[0] >> 9) + (pick[1] >> 9);
            const unsigned long long key = (sum << 9) | (unsigned long long)node;
            made_key[made] = key;
            parent[(int)(pick[0] & 511ull)] = (short)node;
            parent[(int)(pick[1] & 511ull)] = (short)node;
            // The new node is entry `made` of its queue: one of the three that travel in registers?
            const int ahead = made - next_made;
            m0 = ahead == 0 ? key : m0;
            m1 = ahead == 1 ? key : m1;
            m2_new = ahead == 2;
            m2_key = key;
            ++made;
        }
    }
    __syncthreads();

    // A level's codeword length is its depth in the tree.  A lane climbs from its four levels side
    // by side, so that the four chains of LDS reads overlap.
    {
        int at[4], depth[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = lane + 64 * q;
            const bool occurs = c < bins && weight[c] > 0;
            at[q] = occurs && !single ? c : -1;
            depth[q] = occurs && single ? 1 : 0;
        }
        for (;;) {
            bool climbing = false;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int up = at[q] >= 0 ? parent[at[q]] : -1;
                depth[q] += up >= 0 ? 1 : 0;
                at[q] = up;
                climbing = climbing || up >= 0;
            }
            if (!climbing) break;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int d = depth[q] > kMaxLen ? kMaxLen : depth[q];   // cannot happen for counts that sum to <= 2^34
            len_of[lane + 64 * q] = (unsigned char)d;
            if (d) atomicAdd(&len_count[d], 1u);
        }
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
    // Canonical codewords: a level's place among the levels of its length, in number order.
    {
        int len[4];
        unsigned int rank[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            len[q] = len_of[lane + 64 * q];                    // 0 beyond `bins`
            rank[q] = 0u;
        }
#pragma unroll 8
        for (int j = 0; j < bins_up; ++j) {
            const int other = len_of[j];
#pragma unroll
            for (int q = 0; q < 4; ++q) rank[q] += (other == len[q] && j < lane + 64 * q) ? 1u : 0u;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = lane + 64 * q;
            if (c >= bins) continue;
            lengths[row + c] = (uint8_t)len[q];
            codewords[row + c] = len[q] ? first_code[len[q]] + rank[q] : 0ull;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Encoder.
// ---------------------------------------------------------------------------------------------

// Per-row code table in LDS.
//   rev/len   every level: codeword with its bits reversed (the order in which they enter the
//             LSB-first stream) and its length;
//   packed    (length << 24) | reversed codeword, valid when no codeword of the row is longer
//             than 24 bits (all_short) -- true unless some level is rarer than about 1 in 2^24;
//   group     the same for GROUPS of group_k consecutive elements, indexed by their group_k*R
//             code bits: total length << 24 | the codewords back to back.  group_k = 4 for
//             2-bit codes whose codewords have at most 6 bits, else 2 while codes have at most
//             4 bits (a pair whose codewords exceed 24 bits together has 255 in the length
//             field and no bits; pair_len holds every pair's true length), else 1: short
//             codes, the common case, cost a quarter or half of the table lookups.
struct EncodeTable {
    unsigned long long rev[256];
    unsigned int packed[256];
    unsigned int group[256];
    unsigned char len[256];
    unsigned char pair_len[256];
    int all_short;
    int group_k;
    unsigned int max_len;
};

template <int R>
__device__ __forceinline__ void fill_encode_table(EncodeTable &tab, const uint8_t *__restrict__ lengths,
                                                  const unsigned long long *__restrict__ codewords, int bins)
{
    if (threadIdx.x == 0) {
        tab.all_short = 1;
        tab.max_len = 0u;
    }
    __syncthreads();
    for (int c = threadIdx.x; c < 256; c += blockDim.x) {
        int l = c < bins ? lengths[c] : 0;
        l = l > kMaxLen ? kMaxLen : l;
        unsigned long long cw = (c < bins && l) ? codewords[c] : 0ull;
        cw &= (1ull << l) - 1ull;
        const unsigned long long rev = l ? (__brevll(cw) >> (64 - l)) : 0ull;
        tab.rev[c] = rev;
        tab.len[c] = (unsigned char)l;
        tab.packed[c] = ((unsigned int)l << 24) | (unsigned int)(rev & 0xFFFFFFull);
        if (l > 24) tab.all_short = 0;                         // benign race: every writer stores 0
        if (l) atomicMax(&tab.max_len, (unsigned int)l);
    }
    __syncthreads();
    int k = 1;
    if (4 * R <= 8 && 4u * tab.max_len <= 24u) k = 4;
    else if (2 * R <= 8) k = 2;
    if (threadIdx.x == 0) tab.group_k = k;
    if (k > 1) {
        for (int idx = threadIdx.x; idx < (1 << (k * R)); idx += blockDim.x) {
            unsigned int total = 0;
            unsigned long long bits = 0;
            for (int j = 0; j < k; ++j) {
                const unsigned int c = (idx >> (R * j)) & ((1u << R) - 1u);
                bits |= tab.rev[c] << total;
                total += tab.len[c];
            }
            tab.group[idx] = total <= 24u ? ((total << 24) | (unsigned int)bits) : 0xFF000000u;
            if (k == 2) tab.pair_len[idx] = (unsigned char)total;
        }
    }
    __syncthreads();
}

// The fixed-length codes of the 16 elements a lane owns inside its tile; returns how many exist.
template <int R>
__device__ __forceinline__ int load_lane_codes(const uint8_t *__restrict__ crow, int64_t row_bytes, int64_t n,
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

// The same for the Q consecutive runs of 16 elements a lane owns in one encoder step: when all
// of them exist they are one contiguous piece of 2*R*Q bytes.
template <int R, int Q>
__device__ __forceinline__ void load_lane_step(const uint8_t *__restrict__ crow, int64_t row_bytes, int64_t n,
                                               int64_t elem, Codes16<R> (&cd)[Q], int (&valid)[Q])
{
    if (elem + 16 * Q <= n) {
        const uint8_t *__restrict__ src = crow + ((elem * R) >> 3);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            cd[q].load(src + q * 2 * R);
            valid[q] = 16;
        }
    } else {
#pragma unroll
        for (int q = 0; q < Q; ++q) valid[q] = load_lane_codes<R>(crow, row_bytes, n, elem + 16 * q, cd[q]);
    }
}

// The K*R code bits of group g (elements g*K .. g*K+K-1) of a lane's 16 codes.
template <int R, int K>
__device__ __forceinline__ unsigned int group_index(const Codes16<R> &cd, int g)
{
    const int bit = R * K * g, i = bit >> 5, sh = bit & 31;
    uint32_t v = cd.w[i] >> sh;
    if (sh + R * K > 32) v |= cd.w[i + 1] << (32 - sh);
    return v & ((1u << (R * K)) - 1u);
}

// Sum of the codeword lengths of a lane's codes.
template <int R>
__device__ __forceinline__ unsigned int lane_bits(const EncodeTable &tab, const Codes16<R> &cd, int valid)
{
    unsigned int bits = 0;
    if constexpr (R == 2) {
        // Three levels: count them with bit masks; pad codes (zero bits = code 0) are removed
        // through `valid`.
        const uint32_t x = cd.w[0], lo = x & 0x55555555u, hi = (x >> 1) & 0x55555555u;
        const unsigned int n1 = __popc(lo & ~hi), n2 = __popc(hi & ~lo), n3 = __popc(hi & lo);
        bits = (valid - n1 - n2 - n3) * tab.len[0] + n1 * tab.len[1] + n2 * tab.len[2];
    } else if (R <= 4 && valid == 16 && tab.group_k == 2) {
        if constexpr (R <= 4) {
#pragma unroll
            for (int g = 0; g < 8; ++g) bits += tab.pair_len[group_index<R, 2>(cd, g)];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) bits += e < valid ? tab.len[cd.code(e)] : 0u;
    }
    return bits;
}

// Appends a lane's 16 codewords, K at a time through the group table (K = 1: the per-level
// table, with missing elements skipped), to the wave's buffer starting at buffer bit `pos`.
// Every table entry holds at most 24 bits, so one check of the 64-bit accumulator per entry
// is enough.
template <int R, int K>
__device__ __forceinline__ void emit_groups(const EncodeTable &tab, const Codes16<R> &cd, int valid, unsigned int pos,
                                            unsigned int *__restrict__ mine, int words)
{
    int w = (int)(pos >> 5);
    unsigned long long acc = 0;
    unsigned int held = pos & 31u;                             // bits of acc below the next free one
#pragma unroll
    for (int g = 0; g < 16 / K; ++g) {
        unsigned int entry;
        if constexpr (K == 1) entry = g < valid ? tab.packed[cd.code(g)] : 0u;
        else entry = tab.group[group_index<R, K>(cd, g)];
        acc |= (unsigned long long)(entry & 0xFFFFFFu) << held;
        held += entry >> 24;
        if (held >= 32u) {
            if (w < words) atomicOr(&mine[w], (unsigned int)acc);
            ++w;
            acc >>= 32;
            held -= 32u;
        }
    }
    if (held > 0u && acc != 0ull && w < words) atomicOr(&mine[w], (unsigned int)acc);
}

// Codes of at most 4 bits through the pair table, four pairs at a time: when their codewords
// fit 32 bits together (nearly always: most levels are 0 and have the shortest codeword) they
// are joined in a register and the accumulator is checked once; else pair by pair, and a pair
// without a table entry level by level.
template <int R>
__device__ __forceinline__ void emit_pairs(const EncodeTable &tab, const Codes16<R> &cd, unsigned int pos,
                                           unsigned int *__restrict__ mine, int words)
{
    int w = (int)(pos >> 5);
    unsigned long long acc = 0;
    unsigned int held = pos & 31u;
    auto append = [&](unsigned int bits, unsigned int len) {   // len <= 32, held < 32
        acc |= (unsigned long long)bits << held;
        held += len;
        if (held >= 32u) {
            if (w < words) atomicOr(&mine[w], (unsigned int)acc);
            ++w;
            acc >>= 32;
            held -= 32u;
        }
    };
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        unsigned int e[4], idx[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            idx[j] = group_index<R, 2>(cd, 4 * half + j);
            e[j] = tab.group[idx[j]];
        }
        const unsigned int l0 = e[0] >> 24, l1 = l0 + (e[1] >> 24), l2 = l1 + (e[2] >> 24), l3 = l2 + (e[3] >> 24);
        if (l3 <= 32u) {
            const unsigned int chunk = (e[0] & 0xFFFFFFu) | ((e[1] & 0xFFFFFFu) << l0) | ((e[2] & 0xFFFFFFu) << l1) |
                                       ((e[3] & 0xFFFFFFu) << l2);
            append(chunk, l3);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if ((e[j] >> 24) != 255u) {
                    append(e[j] & 0xFFFFFFu, e[j] >> 24);
                } else {
                    const unsigned int p0 = tab.packed[idx[j] & ((1u << R) - 1u)], p1 = tab.packed[idx[j] >> R];
                    append(p0 & 0xFFFFFFu, p0 >> 24);
                    append(p1 & 0xFFFFFFu, p1 >> 24);
                }
            }
        }
    }
    if (held > 0u && acc != 0ull && w < words) atomicOr(&mine[w], (unsigned int)acc);
}

// Three levels (r = 2) and no codeword longer than 2 bits -- every code built from the counts of
// a ternary message: the 16 codewords of a run fit 32 bits, so four group entries are joined in
// a register and the accumulator is checked once per run instead of once per entry.
template <int Q>
__device__ __forceinline__ void emit_ternary(const EncodeTable &tab, const Codes16<2> (&cd)[Q], unsigned int pos,
                                             unsigned int *__restrict__ mine, int words)
{
    int w = (int)(pos >> 5);
    unsigned long long acc = 0;
    unsigned int held = pos & 31u;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const uint32_t x = cd[q].w[0];
        const unsigned int e0 = tab.group[x & 0xFFu], e1 = tab.group[(x >> 8) & 0xFFu];
        const unsigned int e2 = tab.group[(x >> 16) & 0xFFu], e3 = tab.group[x >> 24];
        const unsigned int l0 = e0 >> 24, l1 = l0 + (e1 >> 24), l2 = l1 + (e2 >> 24), l3 = l2 + (e3 >> 24);
        const unsigned int chunk = (e0 & 0xFFFFFFu) | ((e1 & 0xFFFFFFu) << l0) | ((e2 & 0xFFFFFFu) << l1) |
                                   ((e3 & 0xFFFFFFu) << l2);
        acc |= (unsigned long long)chunk << held;
        held += l3;
        if (held >= 32u) {
            if (w < words) atomicOr(&mine[w], (unsigned int)acc);
            ++w;
            acc >>= 32;
            held -= 32u;
        }
    }
    if (held > 0u && acc != 0ull && w < words) atomicOr(&mine[w], (unsigned int)acc);
}

// The same for rows with a codeword longer than 24 bits: one level at a time from the 63-bit
// table, in at most two pieces of 32 bits.
template <int R>
__device__ __forceinline__ void emit_long(const EncodeTable &tab, const Codes16<R> &cd, int valid, unsigned int pos,
                                          unsigned int *__restrict__ mine, int words)
{
    int w = (int)(pos >> 5);
    unsigned long long acc = 0;
    unsigned int held = pos & 31u;
#pragma unroll 1
    for (int e = 0; e < valid; ++e) {
        unsigned int c = 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) c = k == e ? cd.code(k) : c;
        unsigned int l = tab.len[c];
        unsigned long long bits = tab.rev[c];
        while (l > 0) {
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

// Codeword lengths only, for pass 1: per level, and per PAIR of levels (indexed by their 2*R
// code bits) while codes have at most 4 bits.
struct LengthTable {
    unsigned char len[256];
    unsigned char pair[256];
};

template <int R>
__device__ __forceinline__ void fill_length_table(LengthTable &tab, const uint8_t *__restrict__ lengths, int bins)
{
    for (int c = threadIdx.x; c < 256; c += blockDim.x) {
        const int l = c < bins ? lengths[c] : 0;
        tab.len[c] = (unsigned char)(l > kMaxLen ? kMaxLen : l);
    }
    __syncthreads();
    if constexpr (R <= 4) {
        for (int idx = threadIdx.x; idx < (1 << (2 * R)); idx += blockDim.x)
            tab.pair[idx] = (unsigned char)(tab.len[idx & ((1 << R) - 1)] + tab.len[idx >> R]);
        __syncthreads();
    }
}

// Sum of the codeword lengths of a lane's codes from the length table (the same number that
// lane_bits gives).
template <int R>
__device__ __forceinline__ unsigned int lane_bits_of_lengths(const LengthTable &tab, const unsigned int (&len3)[3],
                                                             const Codes16<R> &cd, int valid)
{
    unsigned int bits = 0;
    if constexpr (R == 2) {
        const uint32_t x = cd.w[0], lo = x & 0x55555555u, hi = (x >> 1) & 0x55555555u;
        const unsigned int n1 = __popc(lo & ~hi), n2 = __popc(hi & ~lo), n3 = __popc(hi & lo);
        bits = (valid - n1 - n2 - n3) * len3[0] + n1 * len3[1] + n2 * len3[2];
    } else if (R <= 4 && valid == 16) {
        if constexpr (R <= 4) {
#pragma unroll
            for (int g = 0; g < 8; ++g) bits += tab.pair[group_index<R, 2>(cd, g)];
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) bits += e < valid ? tab.len[cd.code(e)] : 0u;
    }
    return bits;
}

// Pass 1: number of stream bits of every run of kRunTiles tiles, one wave per run, written to
// the run's first entry of tile_offsets.  A lane owns 16*Q consecutive elements of every step,
// as in pass 3; the loads of several steps are requested before any is used.
template <int R>
__global__ void __launch_bounds__(256) k_huffman_run_bits(const Args a, const uint8_t *__restrict__ lengths,
                                                         const int64_t table_stride, const int64_t tiles,
                                                         unsigned long long *__restrict__ tile_offsets,
                                                         const int64_t offset_stride)
{
    constexpr int Q = kStepGroups<R>;
    constexpr int kStepElems = 64 * 16 * Q;
    constexpr int kSteps = kRunElems / kStepElems;
    constexpr int kWords = Codes16<R>::kWords;
    constexpr int kFit = 32 / (Q * kWords);                    // steps whose codes fit 32 registers
    constexpr int kBatch = kFit >= kSteps ? kSteps : (kFit >= 8 ? 8 : (kFit >= 4 ? 4 : (kFit >= 2 ? 2 : 1)));
    __shared__ LengthTable tab;
    const uint32_t p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t first = ((int64_t)blockIdx.x * 4 + wave) * kRunTiles;
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    Codes16<R> cd[kBatch][Q];
    int valid[kBatch][Q];
    auto request = [&](int s0) {                               // (nothing is read beyond the row's n elements)
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
            load_lane_step<R, Q>(crow, a.row_bytes, a.n, first * kTile + (int64_t)(s0 + i) * kStepElems + lane * (16 * Q),
                                 cd[i], valid[i]);
    };
    request(0);                                                // in flight while the table is made
    fill_length_table<R>(tab, lengths + (int64_t)p * table_stride, 2 * a.s + 1);
    if (first >= tiles) return;                                // wave-uniform; no barrier follows
    const unsigned int len3[3] = {tab.len[0], tab.len[1], tab.len[2]};
    unsigned int bits = 0;
#pragma unroll 1
    for (int s0 = 0; s0 < kSteps; s0 += kBatch) {
        if (s0 > 0) request(s0);
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
#pragma unroll
            for (int q = 0; q < Q; ++q) bits += lane_bits_of_lengths<R>(tab, len3, cd[i][q], valid[i][q]);
    }
    // Sum over the wave; a lane's total stays below 2^32 (16384 elements x 63 bits).
    bits += dpp_u32<0xB1>(bits);                               // quad_perm [1,0,3,2]
    bits += dpp_u32<0x4E>(bits);                               // quad_perm [2,3,0,1]
    bits += dpp_u32<0x141>(bits);                              // row_half_mirror
    bits += dpp_u32<0x140>(bits);                              // row_mirror
    const unsigned int total = (unsigned int)__builtin_amdgcn_readlane((int)bits, 0) +
                               (unsigned int)__builtin_amdgcn_readlane((int)bits, 16) +
                               (unsigned int)__builtin_amdgcn_readlane((int)bits, 32) +
                               (unsigned int)__builtin_amdgcn_readlane((int)bits, 48);
    if (lane == 0) tile_offsets[(int64_t)p * offset_stride + first] = total;
}

// Pass 2: exclusive prefix sum of the run sizes of one row (one block per row), in place in the
// runs' first entries of tile_offsets, 2048 runs at a time with the next chunk's sizes already
// loading; entry `tiles` receives the total.  Also clears the 32-bit stream word in which every
// run starts and the one that holds the end of the row: those are the words two waves of pass 3
// may share, and they fill them with atomic ORs.
__global__ void __launch_bounds__(1024) k_huffman_scan(unsigned long long *__restrict__ tile_offsets,
                                                      const int64_t offset_stride, const int64_t tiles,
                                                      uint32_t *__restrict__ streams, const int64_t stream_words,
                                                      const int64_t stream_stride_words)
{
    constexpr int K = 2;
    __shared__ unsigned long long wave_total[2][16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t runs = (tiles + kRunTiles - 1) / kRunTiles;
    unsigned long long *__restrict__ row = tile_offsets + (int64_t)blockIdx.x * offset_stride;
    uint32_t *__restrict__ out = streams + (int64_t)blockIdx.x * stream_stride_words;
    unsigned long long carry = 0;
    unsigned int v[K], nxt[K];                                 // a run has fewer than 2^32 bits
#pragma unroll
    for (int k = 0; k < K; ++k) nxt[k] = (int64_t)tid * K + k < runs ? (unsigned int)row[((int64_t)tid * K + k) * kRunTiles] : 0u;
    int parity = 0;
    for (int64_t base = 0; base < runs; base += 1024 * K, parity ^= 1) {
        const int64_t i0 = base + (int64_t)tid * K;
        unsigned int mine = 0;                                 // a wave's 128 runs: fewer than 2^32 bits
#pragma unroll
        for (int k = 0; k < K; ++k) {
            v[k] = nxt[k];
            mine += v[k];
            const int64_t ahead = i0 + 1024 * K + k;
            nxt[k] = ahead < runs ? (unsigned int)row[ahead * kRunTiles] : 0u;
        }
        const unsigned int incl = wave_inclusive_scan(mine);
        if (lane == 63) wave_total[parity][wave] = incl;
        __syncthreads();                                       // one barrier per chunk: the totals alternate buffers
        unsigned long long before = carry, all = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const unsigned long long t = wave_total[parity][w];
            before += w < wave ? t : 0ull;
            all += t;
        }
        unsigned long long off = before + (incl - mine);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (i0 + k < runs) {
                row[(i0 + k) * kRunTiles] = off;
                const unsigned long long word = off >> 5;
                if (word < (unsigned long long)stream_words) out[word] = 0u;
            }
            off += v[k];
        }
        carry += all;
    }
    if (tid == 0) {
        row[tiles] = carry;
        const unsigned long long word = carry >> 5;
        if ((carry & 31ull) && word < (unsigned long long)stream_words) out[word] = 0u;
    }
}

// Pass 3: a wave walks one run (kRunTiles consecutive tiles) in steps of Q tiles.  Per step a
// lane sums the codeword lengths of its 16*Q consecutive elements, a wave prefix sum places
// them, the lanes assemble the step's bits in LDS aligned with the 32-bit words of the stream,
// and the words leave with plain coalesced stores; a partial last word is carried into the next
// step, and only the first and last word of the whole run (which a neighbouring wave may share)
// are filled with atomic ORs.  The position inside the run is the wave's own running sum, and
// the lanes at tile boundaries record it as the tile's offset.
// buf_words = LDS words per wave: enough for a step's codewords of the longest length a code
// over 2s+1 levels can have (2s bits); longer steps (only possible with a table that does not
// belong to the message) are cut off.
template <int R>
__global__ void __launch_bounds__(256) k_huffman_write(const Args a, const uint8_t *__restrict__ lengths,
                                                      const unsigned long long *__restrict__ codewords,
                                                      const int64_t table_stride, const int64_t tiles,
                                                      unsigned long long *__restrict__ tile_offsets,
                                                      const int64_t offset_stride, uint32_t *__restrict__ streams,
                                                      const int64_t stream_words, const int64_t stream_stride_words,
                                                      const int buf_words)
{
    constexpr int Q = kStepGroups<R>;
    constexpr int kStepElems = 64 * 16 * Q;
    constexpr int kSteps = kRunElems / kStepElems;
    constexpr int kLanesPerTile = 64 / Q;
    __shared__ EncodeTable tab;
    extern __shared__ unsigned int step_buf[];
    const uint32_t p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t first = ((int64_t)blockIdx.x * 4 + wave) * kRunTiles;
    unsigned int *__restrict__ mine = step_buf + wave * buf_words;
    const uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    unsigned long long *__restrict__ offs = tile_offsets + (int64_t)p * offset_stride;
    uint32_t *__restrict__ out = streams + (int64_t)p * stream_stride_words;
    // The run's offset (pass 2) and the first step's codes are in flight while the table is made.
    const unsigned long long run_start = first < tiles ? offs[first] : 0ull;
    const int64_t elem0 = first * kTile + (int64_t)lane * (16 * Q);
    Codes16<R> cd[Q], cd_next[Q];
    int valid[Q], valid_next[Q];
    load_lane_step<R, Q>(crow, a.row_bytes, a.n, elem0, cd_next, valid_next);
    fill_encode_table<R>(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride, 2 * a.s + 1);
    if (first >= tiles) return;                                // wave-uniform; no block barrier follows
    for (int j = lane; j < buf_words; j += 64) mine[j] = 0u;
    wave_lds_sync();

    unsigned long long pos = run_start;                        // bit offset of the current step
    unsigned int carry = 0;                                    // partial last word of the step before

#pragma unroll 1
    for (int step = 0; step < kSteps; ++step) {
        const int64_t step_first = first * kTile + (int64_t)step * kStepElems;
        if (step_first >= a.n) break;                          // wave-uniform
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            cd[q] = cd_next[q];
            valid[q] = valid_next[q];
        }
        load_lane_step<R, Q>(crow, a.row_bytes, a.n, elem0 + (int64_t)(step + 1) * kStepElems, cd_next, valid_next);
        unsigned int nb[Q], nbits = 0;
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            nb[q] = lane_bits<R>(tab, cd[q], valid[q]);
            nbits += nb[q];
        }
        const unsigned int incl = wave_inclusive_scan(nbits);
        const unsigned int total = (unsigned int)__builtin_amdgcn_readlane((int)incl, 63);
        const unsigned int excl = incl - nbits;
        // Tile offsets inside the run (the run's first one is pass 2's).
        if ((lane & (kLanesPerTile - 1)) == 0 && (step > 0 || lane > 0)) {
            const int64_t tile = first + step * Q + lane / kLanesPerTile;
            if (tile < tiles) offs[tile] = pos + excl;
        }
        const unsigned int shift = (unsigned int)(pos & 31ull);
        const unsigned long long word0 = pos >> 5;
        const unsigned long long end = pos + total;
        const unsigned int span = (total + shift + 31u) >> 5;
        const int words = (int)(span < (unsigned int)buf_words ? span : (unsigned int)buf_words);

        unsigned int at = shift + excl;                        // buffer bit of the lane's next codeword
        bool done = false;
        if constexpr (R == 2) {
            bool whole = true;
#pragma unroll
            for (int q = 0; q < Q; ++q) whole = whole && valid[q] == 16;
            if (tab.max_len <= 2u && whole) {
                emit_ternary<Q>(tab, cd, at, mine, words);
                done = true;
            }
        }
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            if (done) break;
            if (tab.all_short) {
                const int k = valid[q] == 16 ? tab.group_k : 1;
                if (R <= 2 && k == 4) {
                    if constexpr (R <= 2) emit_groups<R, 4>(tab, cd[q], valid[q], at, mine, words);
                } else if (R <= 4 && k == 2) {
                    if constexpr (R <= 4) emit_pairs<R>(tab, cd[q], at, mine, words);
                } else {
                    emit_groups<R, 1>(tab, cd[q], valid[q], at, mine, words);
                }
            } else {
                emit_long<R>(tab, cd[q], valid[q], at, mine, words);
            }
            at += nb[q];
        }
        wave_lds_sync();

        // Words wholly inside the run leave with plain stores and their buffer word is cleared
        // for the next step.  The last word of a step, when partial, is carried into the first
        // word of the next step; only the two ends of the run use atomic ORs.
        const bool final_step = step == kSteps - 1 || step_first + kStepElems >= a.n;
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
                const bool lower_ok = gw * 32ull >= run_start;
                const bool upper_ok = (gw + 1ull) * 32ull <= end;
                if (lower_ok && upper_ok) out[gw] = value;
                else if (!upper_ok && !final_step) continue;   // carried below
                else if (value) atomicOr(&out[gw], value);
            }
            carry = has_tail && !final_step ? tail : 0u;
        }
        wave_lds_sync();                                       // the buffer is clear again for the next step
        pos = end;
    }
}

// ---------------------------------------------------------------------------------------------
// Decoder: one lane per tile.
// ---------------------------------------------------------------------------------------------
// Decoding a tile is a chain: the position of a codeword is known only once the one before it
// has been decoded.  To shorten the chain the main table maps the next 10 stream bits to ALL
// the codewords that end inside them (up to 10, and as many as fit 24 bits of r-bit codes):
//   multi[i] = packed r-bit codes | bits consumed << 24 | symbols << 28      (symbols = 0: none)
// A codeword longer than 10 bits, and the last few symbols of a tile, take the single-symbol
// route: `fast` (first codeword in the 10 bits) or the canonical first-code/count walk.
struct DecodeTable {
    unsigned long long first_code[64];       // canonical: first codeword of each length
    unsigned int multi[1 << kFastBits];
    unsigned int count[64];                  // codewords of each length
    unsigned short base[64];                 // index into sorted[] of the first one
    unsigned short fast[1 << kFastBits];     // next 10 stream bits -> (length << 8) | code, 0 = longer
    unsigned char sorted[256];               // codes c in the order (length, c)
};

template <int R>
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
    // Canonical order: by (length, c).
    for (int c = tid; c < bins; c += blockDim.x) {
        const int l = lengths[c] > kMaxLen ? kMaxLen : lengths[c];
        if (l) atomicAdd(&tab.count[l], 1u);
    }
    __syncthreads();
    for (int l = tid; l < 64; l += blockDim.x) {
        unsigned int at = 0;
        for (int j = 1; j < l; ++j) at += tab.count[j];
        tab.base[l] = (unsigned short)at;
    }
    __syncthreads();
    for (int c = tid; c < bins; c += blockDim.x) {
        const int l = lengths[c] > kMaxLen ? kMaxLen : lengths[c];
        if (!l) continue;
        int rank = 0;
        for (int j = 0; j < c; ++j) {
            const int lj = lengths[j] > kMaxLen ? kMaxLen : lengths[j];
            rank += lj == l ? 1 : 0;
        }
        const unsigned long long cw = codewords[c] & ((1ull << l) - 1ull);
        if (rank == 0) tab.first_code[l] = cw;
        const int slot = tab.base[l] + rank;
        if (slot < 256) tab.sorted[slot] = (unsigned char)c;
    }
    // Every window whose low bits are a codeword of at most kFastBits bits: the block goes
    // through the levels together and shares out each one's 2^(kFastBits - length) windows.
    for (int c = 0; c < bins; ++c) {
        const int l = lengths[c] > kMaxLen ? kMaxLen : lengths[c];
        if (!l || l > kFastBits) continue;                     // block-uniform
        const unsigned long long cw = codewords[c] & ((1ull << l) - 1ull);
        const unsigned int rev = (unsigned int)(__brevll(cw) >> (64 - l));
        for (unsigned int hi = tid; hi < (1u << (kFastBits - l)); hi += blockDim.x)
            tab.fast[rev | (hi << l)] = (unsigned short)((l << 8) | c);
    }
    __syncthreads();
    // Chain single-symbol lookups inside the 10-bit window.  Bits beyond the window read as
    // zeros, so a hit only counts when the whole codeword lies inside the window.
    // A thread walks four windows side by side, so that their table reads overlap.
    constexpr int kMaxSyms = 24 / R < kFastBits ? 24 / R : kFastBits;
    constexpr int kSide = 4;
    for (int i0 = tid; i0 < (1 << kFastBits); i0 += kSide * blockDim.x) {
        unsigned int used[kSide], syms[kSide], packed[kSide];
        bool open[kSide];
#pragma unroll
        for (int e = 0; e < kSide; ++e) {
            used[e] = syms[e] = packed[e] = 0u;
            open[e] = i0 + e * (int)blockDim.x < (1 << kFastBits);
        }
#pragma unroll 1
        for (int step = 0; step < kMaxSyms; ++step) {
            unsigned int hit[kSide];
#pragma unroll
            for (int e = 0; e < kSide; ++e)
                hit[e] = open[e] ? tab.fast[((unsigned int)(i0 + e * (int)blockDim.x) >> used[e]) & ((1u << kFastBits) - 1u)] : 0u;
            bool any = false;
#pragma unroll
            for (int e = 0; e < kSide; ++e) {
                const unsigned int l = hit[e] >> 8;
                open[e] = open[e] && hit[e] != 0u && used[e] + l <= (unsigned int)kFastBits;
                if (open[e]) {
                    packed[e] |= (hit[e] & ((1u << R) - 1u)) << (R * syms[e]);
                    ++syms[e];
                    used[e] += l;
                }
                any = any || open[e];
            }
            if (!any) break;
        }
#pragma unroll
        for (int e = 0; e < kSide; ++e) {
            const int i = i0 + e * (int)blockDim.x;
            if (i < (1 << kFastBits)) tab.multi[i] = syms[e] ? (packed[e] | (used[e] << 24) | (syms[e] << 28)) : 0u;
        }
    }
    __syncthreads();
}

template <int R>
__global__ void __launch_bounds__(kDecodeThreads) k_huffman_decode(const Args a, const uint8_t *__restrict__ lengths,
                                                       const unsigned long long *__restrict__ codewords,
                                                       const int64_t table_stride, const int64_t tiles,
                                                       const unsigned long long *__restrict__ tile_offsets,
                                                       const int64_t offset_stride,
                                                       const uint32_t *__restrict__ streams,
                                                       const int64_t stream_words, const int64_t stream_stride_words,
                                                       const int lanes)
{
    __shared__ DecodeTable tab;
    // Word k of lane t's ring at [k][t]: whatever slots the lanes of a wave are at, they write to
    // 64 different banks.
    __shared__ unsigned int out_ring[kRingWords * kDecodeThreads];
    const uint32_t p = blockIdx.y;
    fill_decode_table<R>(tab, lengths + (int64_t)p * table_stride, codewords + (int64_t)p * table_stride,
                         2 * a.s + 1);
    // A wave takes `lanes` tiles, one per lane of its first `lanes` lanes: decoding is a chain of
    // dependent instructions, so while the message has too few tiles to fill the chip with
    // whole waves, more waves with idle lanes finish sooner.
    const int64_t tile = ((int64_t)blockIdx.x * (kDecodeThreads / 64) + (threadIdx.x >> 6)) * lanes + (threadIdx.x & 63);
    if ((int)(threadIdx.x & 63) >= lanes || tile >= tiles) return;   // after the last barrier
    const int64_t elem0 = tile * kTile;
    int remaining = (int)((a.n - elem0) < kTile ? (a.n - elem0) : (int64_t)kTile);
    const uint32_t *__restrict__ in = streams + (int64_t)p * stream_stride_words;
    uint8_t *__restrict__ crow = a.codes + (int64_t)p * a.code_stride;
    int64_t out_byte = (elem0 >> 3) * R;                       // a multiple of 128*R: 4-byte aligned in the row

    const unsigned long long start = tile_offsets[(int64_t)p * offset_stride + tile];
    unsigned long long next_word = start >> 5;
    // Bit reservoir: `have` valid bits, the next stream bit is bit 0.  Stream words arrive four
    // at a time and a whole batch ahead of their use, so the chain below waits for memory at
    // most once per 128 stream bits, for loads issued 128 bits earlier.
    // Indices are clamped to the row's last word instead of being tested one by one: a message
    // never reads past its own end, and anything else only has to stay inside the row.
    const unsigned long long last_word = (unsigned long long)stream_words - 1ull;
    auto fetch4 = [&]() -> uint4 {
        uint4 b;
        if (next_word + 3 <= last_word) {
            b.x = in[next_word + 0];
            b.y = in[next_word + 1];
            b.z = in[next_word + 2];
            b.w = in[next_word + 3];
        } else {
            b.x = in[next_word + 0 < last_word ? next_word + 0 : last_word];
            b.y = in[next_word + 1 < last_word ? next_word + 1 : last_word];
            b.z = in[next_word + 2 < last_word ? next_word + 2 : last_word];
            b.w = in[next_word + 3 < last_word ? next_word + 3 : last_word];
        }
        next_word += 4;
        return b;
    };
    uint4 batch = fetch4(), batch_ahead = fetch4();
    int in_batch = 4;
    auto take = [&]() -> unsigned int {
        if (in_batch == 0) {
            // The batch in flight becomes the current one through moves that cannot sink below the
            // new loads (the loads' address passes through them), so that its registers are free to
            // receive those loads.  Left to the compiler the old values stay live across the loads,
            // the new ones land in other registers and are copied into place at once, which waits
            // for them to arrive: a memory round trip in most rounds of a wave, since its lanes run
            // out of words at different times.
            asm volatile("v_mov_b32 %0, %5\n\tv_mov_b32 %1, %6\n\tv_mov_b32 %2, %7\n\tv_mov_b32 %3, %8"
                         : "=&v"(batch.x), "=&v"(batch.y), "=&v"(batch.z), "=&v"(batch.w), "+v"(next_word)
                         : "v"(batch_ahead.x), "v"(batch_ahead.y), "v"(batch_ahead.z), "v"(batch_ahead.w));
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
    refill();

    // Decoded codes are collected in a per-lane LDS ring and leave in 64-byte pieces: global
    // stores inside the chain would make every later wait for a stream word also wait for them.
    unsigned long long out_acc = 0;                            // decoded r-bit codes not yet in the ring
    unsigned int out_held = 0;
    unsigned int *__restrict__ ring = out_ring + threadIdx.x;
    int ring_at = 0;
    const bool rows_on_16 = (reinterpret_cast<uintptr_t>(crow) & 15u) == 0u;   // block-uniform
    auto flush_ring = [&](int count) {
        if (count == kRingWords && out_byte + 4 * kRingWords <= a.row_bytes) {
            if (rows_on_16) {                                  // (a tile starts on a multiple of 128 bytes of its row)
#pragma unroll
                for (int q = 0; q < kRingWords / 4; ++q) {
                    uint4 v;
                    v.x = ring[(4 * q + 0) * kDecodeThreads];
                    v.y = ring[(4 * q + 1) * kDecodeThreads];
                    v.z = ring[(4 * q + 2) * kDecodeThreads];
                    v.w = ring[(4 * q + 3) * kDecodeThreads];
                    reinterpret_cast<uint4 *>(crow + out_byte)[q] = v;
                }
            } else {
#pragma unroll
                for (int k = 0; k < kRingWords; ++k)
                    reinterpret_cast<uint32_t *>(crow + out_byte)[k] = ring[k * kDecodeThreads];
            }
        } else {
            for (int k = 0; k < count; ++k)
                store_code_bytes(crow + out_byte + 4 * k, ring[k * kDecodeThreads], 4, a.row_bytes - (out_byte + 4 * k));
        }
        out_byte += 4 * count;
    };
    // The lanes of a wave fill their rings side by side (a tile gives every lane the same number
    // of words) and empty them together: one store sequence per 64 bytes of every tile.  (Each
    // lane emptying its own ring when full made the wave run that sequence for one or two lanes
    // in most rounds.)  A lookup adds at most 24 bits to fewer than 32 held ones, so at most one
    // word per lookup: a lane stops when its ring is full and keeps the rest in `out_acc`.
#pragma unroll 1
    for (int piece = 0; piece < (kTile * R / 32) / kRingWords; ++piece) {
    while (remaining > 0 && ring_at < kRingWords) {
      refill();                                                // have >= 33 here: enough for three lookups
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        if (remaining <= 0 || have < (unsigned int)kFastBits || ring_at >= kRingWords) break;   // (a long codeword may have used more)
        const unsigned int m = tab.multi[(unsigned int)res & ((1u << kFastBits) - 1u)];
        const unsigned int syms = m >> 28;
        if (syms != 0u && (int)syms <= remaining) {
            const unsigned int used = (m >> 24) & 15u;
            out_acc |= (unsigned long long)(m & 0xFFFFFFu) << out_held;
            out_held += syms * R;
            res >>= used;
            have -= used;
            remaining -= (int)syms;
        } else {
            unsigned int c = 0;
            const unsigned int hit = tab.fast[(unsigned int)res & ((1u << kFastBits) - 1u)];
            if (hit) {
                c = hit & 0xFFu;
                res >>= (hit >> 8);
                have -= (hit >> 8);
            } else {
                // Longer than the table covers.  Up to 32 bits: the next 32 stream bits, first one
                // on top, give the candidate codeword of every length by one shift; the canonical
                // code says which length holds it.
                if (have < 32u) refill();
                const unsigned int top = __brev((unsigned int)res);
                int l = kFastBits + 1;
                bool found = false;
                for (; l <= 32; ++l) {
                    const unsigned long long cand = top >> (32 - l);
                    const unsigned long long idx = cand - tab.first_code[l];
                    if (tab.count[l] && cand >= tab.first_code[l] && idx < tab.count[l]) {
                        c = tab.sorted[(tab.base[l] + (unsigned int)idx) & 255u];
                        res >>= l;
                        have -= (unsigned int)l;
                        found = true;
                        break;
                    }
                }
                if (!found) {
                    // Beyond 32 bits (levels rarer than one in 2^32): one bit at a time.
                    unsigned long long word = top;
                    res >>= 32;
                    have -= 32u;
                    for (l = 33; l <= kMaxLen; ++l) {
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
            }
            out_acc |= (unsigned long long)(c & ((1u << R) - 1u)) << out_held;
            out_held += R;
            --remaining;
        }
        // The low word goes to the ring's next slot whether it is complete or not; the slot is
        // only given up once it is.
        const bool full = out_held >= 32u;
        ring[ring_at * kDecodeThreads] = (unsigned int)out_acc;
        out_acc = full ? out_acc >> 32 : out_acc;
        out_held -= full ? 32u : 0u;
        ring_at += full ? 1 : 0;
      }
    }
    if (ring_at == kRingWords) {                                // 64 bytes of codes of every tile of the wave
        flush_ring(kRingWords);
        ring_at = 0;
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
    const dim3 grid_runs(cdiv(tiles, 4 * kRunTiles), (unsigned)a.workers);
#define CALL(RR)                                                                                               \
    hipLaunchKernelGGL((k_huffman_run_bits<RR>), grid_runs, dim3(256), 0, stream, a, lengths, table_stride,      \
                       tiles, tile_offsets, offset_stride)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    hipLaunchKernelGGL(k_huffman_scan, dim3((unsigned)a.workers), dim3(1024), 0, stream, tile_offsets, offset_stride,
                       tiles, streams, stream_words, stream_stride_words);
    // A prefix code over 2s+1 levels has no codeword longer than 2s bits.
    const int max_len = 2 * a.s < kMaxLen ? 2 * a.s : kMaxLen;
    const int buf_words = step_buffer_words(a.r, max_len);
#define CALL(RR)                                                                                               \
    hipLaunchKernelGGL((k_huffman_write<RR>), grid_runs, dim3(256), 4 * buf_words * sizeof(unsigned int),        \
                       stream, a, lengths, codewords, table_stride, tiles, tile_offsets, offset_stride, streams, \
                       stream_words, stream_stride_words, buf_words)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_huffman_decode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                                 int64_t table_stride, const uint32_t *streams, int64_t stream_stride_words,
                                 const unsigned long long *tile_offsets, int64_t offset_stride, hipStream_t stream)
{
    const int64_t tiles = (a.n + kTile - 1) / kTile;
    // Tiles per wave: 64 when that still gives the chip all the waves it can hold at once (six
    // blocks per compute unit), else as few as spreads the tiles over that many waves (8 at least).
    const int64_t held = (int64_t)256 * 6 * (kDecodeThreads / 64);
    int64_t lanes = (tiles * a.workers + held - 1) / held;
    lanes = (lanes + 7) / 8 * 8;
    lanes = lanes < 8 ? 8 : (lanes > 64 ? 64 : lanes);
    const dim3 grid(cdiv(cdiv(tiles, lanes), kDecodeThreads / 64), (unsigned)a.workers);
#define CALL(RR)                                                                                               \
    hipLaunchKernelGGL((k_huffman_decode<RR>), grid, dim3(kDecodeThreads), 0, stream, a, lengths, codewords, table_stride,   \
                       tiles, tile_offsets, offset_stride, streams, stream_stride_words, stream_stride_words, (int)lanes)
    ECQ_DISPATCH_R(a.r, CALL)
#undef CALL
    return hipGetLastError();
}

}  // namespace ecq
