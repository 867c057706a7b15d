/*
 * ecq_oracle.c -- plain, slow, CPU-only statement of what the ECQ-SGD hot path computes.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the HIP library is compared with.  It
 * shares no code, header, table or constant generator with the HIP path and is never linked
 * into or called from it; only tests/, the smoke check and the benchmark's cpu_baseline leg
 * may load it.
 *
 * The method is a randomised encoding, so the oracle is the algorithm taken step by step in
 * the paper's order and notation (Wu et al., ICML 2018):
 *
 *   compensate   v = g + alpha*h                                   Section 4, Eq. (7)
 *   scale        ||v|| taken as the l_inf norm of each bucket      Section 4, text after Eq. (8)
 *   round        xi(|v_i|; ||v||) in {0,1/s,...,1}, sign kept      Section 4, Eq. (8)-(9)
 *   encode       r = ceil(log2(2s+1)) bits per element + 1 scale   Section 4, paragraph on cost
 *   accumulate   h <- beta*h + (g - g~)                            Section 4, Eq. (6)
 *   aggregate    g~ = (1/P) sum_p g~_p                             Section 3/4, Eq. (4); Alg. 1
 *   model update w <- w - eta * g~                                 Eq. (4); Alg. 1, last line
 *
 * Arithmetic: IEEE-754 binary32, round-to-nearest-even, every operation rounded on its own
 * (build with -ffp-contract=off -fno-fast-math; no FMA, denormals kept).  The paper fixes
 * neither the precision nor the operation order; the order below is this repository's
 * convention ("parity unpinned" by the paper for the exact rounding sequence -- it is pinned
 * instead by an exact-rational re-derivation in the tests).
 *
 * Points the paper leaves open and the reading taken here:
 *   - norm: l_inf (max-abs) per bucket by default; a bucket is a run of `bucket` consecutive
 *     elements of the flat per-worker vector, the last one possibly short.  The l_2 norm (the
 *     other choice the paper names, and the one its Lemma 1 covers) is sqrt of the sum of the
 *     squares fl(v_i*v_i), the sum taken over a balanced binary tree by element index (the
 *     bucket padded with zeros to a power of two), then one correctly rounded square root.
 *     (While the squares are normal numbers the computed l_2 norm is never below max|v_i| and
 *     the ratio stays <= 1; a square that underflows can leave the norm below the element, or
 *     at 0: the level is then s, the end of the grid of Eq. (8), or 0 for a zero norm.)
 *   - ||v|| = 0: every level 0, scale 0.
 *   - |v_i| = ||v|| (outside every half-open interval of Eq. (9)): l = s, never rounds up.
 *   - sgn: level is negated iff v_i < 0; level 0 has no sign.
 *   - s*|v_i|/||v|| is evaluated as (|v_i| / ||v||) * s.
 *   - dequantised value is ||v|| * fl(|q|/s) with the sign of q.
 *   - randomness: one 32-bit word per element from Philox4x32-10 (Salmon et al., SC'11), its
 *     top 24 bits give u = k * 2^-24 in [0,1); the level rounds up iff u < frac.
 *   - word for (seed, step, worker p, element i): lane (i & 3) of the block with counter
 *     (low32(i >> 2), p, step_lo, step_hi) and key (seed_lo, seed_hi).
 *   - code = level + s in r bits, fields laid LSB-first in one contiguous bit stream per
 *     worker row (stream bit j is bit (j & 7) of byte (j >> 3)); pad bits are zero.
 *   - Eq. (4): sum over p = 0..P-1 in that order in binary32, then one division by (float)P.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- Philox4x32-10 ---------- */
/* Counter-based generator of Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as
 * 1, 2, 3" (SC'11): ten rounds of two 32x32->64 multiplies and a word permutation, the key
 * bumped by the Weyl constants between rounds. */
void ecq_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The one random word element i of worker p consumes at iteration `step`. */
uint32_t ecq_oracle_word(uint64_t seed, uint64_t step, uint32_t p, uint64_t i)
{
    uint32_t ctr[4], key[2], out[4];
    ctr[0] = (uint32_t)(i >> 2);
    ctr[1] = p;
    ctr[2] = (uint32_t)step;
    ctr[3] = (uint32_t)(step >> 32);
    key[0] = (uint32_t)seed;
    key[1] = (uint32_t)(seed >> 32);
    ecq_oracle_philox4x32_10(ctr, key, out);
    return out[i & 3];
}

void ecq_oracle_words(uint64_t seed, uint64_t step, uint32_t p, uint64_t i0, int64_t count,
                      uint32_t *words)
{
    for (int64_t j = 0; j < count; ++j)
        words[j] = ecq_oracle_word(seed, step, p, i0 + (uint64_t)j);
}

/* ---------------------------------------------------------------- scalar steps ----------- */

/* r = ceil(log2(2s+1)): smallest r with 2^r >= 2s+1 (cost paragraph of Section 4). */
int ecq_oracle_code_bits(int s)
{
    if (s < 1) return -1;
    int r = 0;
    while ((1L << r) < 2L * s + 1L) ++r;
    return r;
}

/* Eq. (7): v = g + alpha*h. */
float ecq_oracle_compensate(float g, float alpha, float h)
{
    float ah = alpha * h;
    return g + ah;
}

/* l_inf norm of one bucket: the largest |v_i| (0 for an empty or all-zero bucket). */
float ecq_oracle_bucket_scale(const float *v, int64_t len)
{
    float m = 0.0f;
    for (int64_t i = 0; i < len; ++i) {
        float a = fabsf(v[i]);
        if (a > m) m = a;
    }
    return m;
}

/* Sum of fl(v_i^2) over indices [lo, lo+width) of a bucket of `len` elements, width a power of
 * two: the two halves are summed on their own and then added; indices >= len count as 0. */
static float sum_squares_tree(const float *v, int64_t lo, int64_t width, int64_t len)
{
    if (lo >= len) return 0.0f;
    if (width == 1) return v[lo] * v[lo];
    float left = sum_squares_tree(v, lo, width / 2, len);
    float right = sum_squares_tree(v, lo + width / 2, width / 2, len);
    return left + right;
}

/* l_2 norm of one bucket, with the summation order stated in the header. */
float ecq_oracle_bucket_scale_l2(const float *v, int64_t len)
{
    int64_t width = 1;
    while (width < len) width *= 2;
    return sqrtf(sum_squares_tree(v, 0, width, len));
}

/* Eq. (8)-(9) for one element: signed level q in [-s, s] given the bucket's scale and the
 * element's random word. */
int ecq_oracle_round(float v, float scale, int s, uint32_t word)
{
    if (scale == 0.0f) return 0;
    float a = fabsf(v) / scale;          /* |v_i| / ||v||  in [0,1]                        */
    float x = a * (float)s;              /* position on the grid {0,1,...,s}               */
    float l = floorf(x);                 /* lower grid point, exact                        */
    float frac = x - l;                  /* = s|v_i|/||v|| - l: probability of rounding up */
    float u = (float)(word >> 8) * 0x1p-24f;   /* uniform on {0,...,2^24-1} * 2^-24, exact */
    int m = (int)l + ((u < frac) ? 1 : 0);
    if (m > s) m = s;
    return (v < 0.0f) ? -m : m;
}

/* Eq. (8): g~_i = ||v|| * sgn * xi with xi = |q|/s. */
float ecq_oracle_dequant(int q, float scale, int s)
{
    int m = q < 0 ? -q : q;
    float xi = (float)m / (float)s;
    float gt = scale * xi;
    return (q < 0) ? -gt : gt;
}

/* Eq. (6): h' = beta*h + (g - g~). */
float ecq_oracle_error(float beta, float h, float g, float gt)
{
    float bh = beta * h;
    float d = g - gt;
    return bh + d;
}

/* Levels for many random words at a fixed (v, scale): lets a test enumerate every outcome. */
void ecq_oracle_round_words(float v, float scale, int s, const uint32_t *words, int64_t count,
                            int8_t *q)
{
    for (int64_t j = 0; j < count; ++j) q[j] = (int8_t)ecq_oracle_round(v, scale, s, words[j]);
}

/* ---------------------------------------------------------------- encoding --------------- */

int64_t ecq_oracle_row_bytes(int64_t n, int s)
{
    int r = ecq_oracle_code_bits(s);
    if (r < 0 || n < 0) return -1;
    return (n * (int64_t)r + 7) / 8;
}

/* Fixed-length encoding: element i's code c = q + s occupies stream bits [i*r, (i+1)*r). */
void ecq_oracle_pack(const int8_t *q, int64_t n, int s, uint8_t *bytes)
{
    int r = ecq_oracle_code_bits(s);
    memset(bytes, 0, (size_t)ecq_oracle_row_bytes(n, s));
    for (int64_t i = 0; i < n; ++i) {
        unsigned c = (unsigned)((int)q[i] + s);
        for (int b = 0; b < r; ++b) {
            int64_t j = i * r + b;
            if ((c >> b) & 1u) bytes[j >> 3] |= (uint8_t)(1u << (j & 7));
        }
    }
}

/* Every worker row encoded on its own; rows of q are n apart, rows of bytes out_stride apart. */
void ecq_oracle_pack_rows(const int8_t *q, int P, int64_t n, int s, uint8_t *bytes, int64_t out_stride)
{
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int p = 0; p < P; ++p) ecq_oracle_pack(q + (int64_t)p * n, n, s, bytes + (int64_t)p * out_stride);
}

void ecq_oracle_unpack(const uint8_t *bytes, int64_t n, int s, int8_t *q)
{
    int r = ecq_oracle_code_bits(s);
    for (int64_t i = 0; i < n; ++i) {
        unsigned c = 0;
        for (int b = 0; b < r; ++b) {
            int64_t j = i * r + b;
            c |= (unsigned)((bytes[j >> 3] >> (j & 7)) & 1u) << b;
        }
        q[i] = (int8_t)((int)c - s);
    }
}

/* ---------------------------------------------------------------- one bucket ------------- */

/* One bucket of worker p at iteration `step` (Alg. 1: quantise g + alpha*h with the current
 * h, then move h to its next value with the same g and g~).  i0 is the index, in the worker's
 * flat vector, of g[0]/h[0].  gt may be NULL.  If update_h is 0, h is left as it is. */
void ecq_oracle_bucket_step(const float *g, float *h, int64_t len, uint64_t i0, uint32_t p,
                            int s, float alpha, float beta, uint64_t seed, uint64_t step,
                            int update_h, int8_t *q, float *scale_out, float *gt, int norm_l2)
{
    float *v = (float *)calloc((size_t)(len > 0 ? len : 1), sizeof(float));
    for (int64_t i = 0; i < len; ++i) v[i] = ecq_oracle_compensate(g[i], alpha, h[i]);
    float scale = norm_l2 ? ecq_oracle_bucket_scale_l2(v, len) : ecq_oracle_bucket_scale(v, len);
    free(v);
    *scale_out = scale;
    for (int64_t i = 0; i < len; ++i) {
        float vi = ecq_oracle_compensate(g[i], alpha, h[i]);
        uint32_t w = ecq_oracle_word(seed, step, p, i0 + (uint64_t)i);
        int qi = ecq_oracle_round(vi, scale, s, w);
        float gti = ecq_oracle_dequant(qi, scale, s);
        q[i] = (int8_t)qi;
        if (gt) gt[i] = gti;
        if (update_h) h[i] = ecq_oracle_error(beta, h[i], g[i], gti);
    }
}

/* ---------------------------------------------------------------- whole batch ------------ */

/* P workers (numbered worker0 .. worker0+P-1), all buckets, one iteration.  g, h:
 * [P][gh_stride]; q: [P][n] signed levels; scales: [P][nb]; gt (optional): [P][n].  Buckets are
 * independent, so the loop over them may be split over threads without changing any result. */
void ecq_oracle_batch_step(const float *g, float *h, int64_t n, int64_t gh_stride, int P,
                           int worker0, int bucket, int s, float alpha, float beta, uint64_t seed,
                           uint64_t step, int update_h, int8_t *q, float *scales, float *gt,
                           int threads, int norm_l2)
{
    int64_t nb = (n + bucket - 1) / bucket;
    int64_t units = (int64_t)P * nb;
#ifdef _OPENMP
    if (threads > 0) omp_set_num_threads(threads);
#pragma omp parallel for schedule(static)
#endif
    for (int64_t unit = 0; unit < units; ++unit) {
        int64_t p = unit / nb, k = unit % nb;
        int64_t e0 = k * (int64_t)bucket;
        int64_t len = (n - e0 < bucket) ? (n - e0) : bucket;
        ecq_oracle_bucket_step(g + p * gh_stride + e0, h + p * gh_stride + e0, len,
                               (uint64_t)e0, (uint32_t)(worker0 + p), s, alpha, beta, seed, step, update_h,
                               q + p * n + e0, scales + p * nb + k,
                               gt ? gt + p * n + e0 : NULL, norm_l2);
    }
    (void)threads;
}

int ecq_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. (6) alone, from an encoded message: h <- beta*h + (g - decode(codes, scales)). */
void ecq_oracle_error_update_row(const float *g, const uint8_t *codes, const float *scales,
                                 int64_t n, int bucket, int s, float beta, float *h)
{
    int r = ecq_oracle_code_bits(s);
    for (int64_t i = 0; i < n; ++i) {
        unsigned c = 0;
        for (int b = 0; b < r; ++b) {
            int64_t j = i * r + b;
            c |= (unsigned)((codes[j >> 3] >> (j & 7)) & 1u) << b;
        }
        float gt = ecq_oracle_dequant((int)c - s, scales[i / bucket], s);
        h[i] = ecq_oracle_error(beta, h[i], g[i], gt);
    }
}

/* Eq. (4) / Alg. 1 "compute global gradients": decode every worker's message and average.
 * codes: [P] rows code_stride BYTES apart; scales: [P] rows scale_stride floats apart. */
void ecq_oracle_aggregate(const uint8_t *codes, int64_t code_stride, const float *scales,
                          int64_t scale_stride, int P, int64_t n, int bucket, int s, float *out)
{
    int r = ecq_oracle_code_bits(s);
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < n; ++i) {
        float acc = 0.0f;
        for (int p = 0; p < P; ++p) {
            const uint8_t *row = codes + (int64_t)p * code_stride;
            unsigned c = 0;
            for (int b = 0; b < r; ++b) {
                int64_t j = i * r + b;
                c |= (unsigned)((row[j >> 3] >> (j & 7)) & 1u) << b;
            }
            float gt = ecq_oracle_dequant((int)c - s, scales[(int64_t)p * scale_stride + i / bucket], s);
            acc = acc + gt;
        }
        out[i] = acc / (float)P;
    }
}

/* Alg. 1 "update model parameters" / Eq. (4): w <- w - eta * g~, the product rounded first. */
void ecq_oracle_sgd_step(float *w, const float *gavg, float eta, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        float stepv = eta * gavg[i];
        w[i] = w[i] - stepv;
    }
}

/* d_k of the cost paragraph of Section 4: how many elements sit on each quantisation level.
 * counts[c] for c = level + s in 0..2s. */
void ecq_oracle_level_histogram(const int8_t *q, int64_t n, int s, uint64_t *counts)
{
    for (int c = 0; c <= 2 * s; ++c) counts[c] = 0;
    for (int64_t i = 0; i < n; ++i) counts[(int)q[i] + s] += 1;
}

/* Entropy-coding bound of Section 4: sum_k d_k log2(d / d_k) bits, d = sum_k d_k. */
double ecq_oracle_entropy_bound_bits(const uint64_t *counts, int bins)
{
    double d = 0.0, bits = 0.0;
    for (int k = 0; k < bins; ++k) d += (double)counts[k];
    for (int k = 0; k < bins; ++k)
        if (counts[k] > 0) bits += (double)counts[k] * log2(d / (double)counts[k]);
    return bits;
}

/* ---------------------------------------------------------------- Huffman coding --------- */
/* Section 4 names Huffman encoding (Huffman, 1952) as the way to go below r bits per element.
 * The code is built per worker row from that row's level counts d_k.
 *
 * Conventions of this repository (the paper fixes none of them):
 *  - Construction: leaves are the levels with d_k > 0, numbered by their code c = level + s;
 *    repeatedly the two live nodes that come first in the order (weight, number) are merged
 *    into a new node that takes the next free number (2s+1, 2s+2, ...); a level's codeword
 *    length is its depth.  A row with a single occupied level gives it length 1.
 *  - Codewords are canonical: levels sorted by (length, c); the first codeword is 0, each next
 *    one is (previous + 1) shifted left by the growth in length.
 *  - Bit stream: LSB-first like the fixed-length stream (stream bit j is bit (j & 7) of byte
 *    (j >> 3)); a codeword is written most significant bit first; pad bits are zero.
 *  - The row is cut into tiles of `tile` elements; tile_offsets[t] is the stream bit at which
 *    tile t starts and tile_offsets[number of tiles] the total length, so tiles decode
 *    independently.
 */

void ecq_oracle_huffman_lengths(const uint64_t *counts, int bins, uint8_t *lengths)
{
    enum { MAXN = 512 };
    uint64_t weight[MAXN];
    int parent[MAXN], live[MAXN];
    int nodes = bins, alive = 0;
    for (int c = 0; c < bins; ++c) {
        weight[c] = counts[c];
        parent[c] = -1;
        live[c] = counts[c] > 0;
        alive += live[c];
        lengths[c] = 0;
    }
    if (alive == 1) {
        for (int c = 0; c < bins; ++c) if (live[c]) lengths[c] = 1;
        return;
    }
    while (alive > 1) {
        int pick[2];
        for (int k = 0; k < 2; ++k) {
            int best = -1;
            for (int i = 0; i < nodes; ++i)
                if (live[i] && (best < 0 || weight[i] < weight[best])) best = i;  /* ties: lowest number */
            live[best] = 0;
            pick[k] = best;
        }
        weight[nodes] = weight[pick[0]] + weight[pick[1]];
        parent[nodes] = -1;
        live[nodes] = 1;
        parent[pick[0]] = nodes;
        parent[pick[1]] = nodes;
        ++nodes;
        --alive;
    }
    for (int c = 0; c < bins; ++c) {
        if (!counts[c]) continue;
        int depth = 0;
        for (int i = c; parent[i] >= 0; i = parent[i]) ++depth;
        lengths[c] = (uint8_t)depth;
    }
}

/* Canonical codewords (as integers, most significant bit = first bit) from the lengths. */
void ecq_oracle_huffman_codes(const uint8_t *lengths, int bins, uint64_t *codes)
{
    uint64_t next = 0;
    int prev_len = 0;
    for (int c = 0; c < bins; ++c) codes[c] = 0;
    for (int len = 1; len < 64; ++len)
        for (int c = 0; c < bins; ++c)
            if (lengths[c] == len) {
                if (prev_len) next = (next + 1) << (len - prev_len);
                codes[c] = next;
                prev_len = len;
            }
}

/* Encodes one worker row.  Returns the total number of bits; out must hold them (it is
 * zeroed up to out_bytes first).  tile_offsets gets ceil(n/tile) + 1 entries. */
int64_t ecq_oracle_huffman_encode(const int8_t *q, int64_t n, int s, const uint8_t *lengths,
                                  const uint64_t *codes, uint8_t *out, int64_t out_bytes, int64_t tile,
                                  uint64_t *tile_offsets)
{
    memset(out, 0, (size_t)out_bytes);
    int64_t pos = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (i % tile == 0) tile_offsets[i / tile] = (uint64_t)pos;
        int c = (int)q[i] + s;
        for (int b = lengths[c] - 1; b >= 0; --b) {            /* most significant bit first */
            if ((codes[c] >> b) & 1u) out[pos >> 3] |= (uint8_t)(1u << (pos & 7));
            ++pos;
        }
    }
    tile_offsets[(n + tile - 1) / tile] = (uint64_t)pos;
    return pos;
}

/* Decodes n levels starting at stream bit `start` by walking the canonical code. */
void ecq_oracle_huffman_decode(const uint8_t *stream, uint64_t start, int64_t n, int s, const uint8_t *lengths,
                               const uint64_t *codes, int8_t *q)
{
    int bins = 2 * s + 1;
    uint64_t pos = start;
    for (int64_t i = 0; i < n; ++i) {
        uint64_t word = 0;
        int len = 0, found = -1;
        while (found < 0 && len < 64) {
            word = (word << 1) | (uint64_t)((stream[pos >> 3] >> (pos & 7)) & 1u);
            ++pos;
            ++len;
            for (int c = 0; c < bins; ++c)
                if (lengths[c] == len && codes[c] == word) found = c;
        }
        q[i] = (int8_t)(found - s);
    }
}

/* ---------------------------------------------------------------- zero-run Huffman coding - */
/* Section 4's cost paragraph bounds the entropy-coded length of a message by
 * sum_k d_k log2(d/d_k) bits.  A Huffman code over single levels never spends less than one bit
 * per element, and quantised gradients are mostly zeros (the bound is often far below one bit),
 * so the Huffman code is taken over TOKENS instead: a run of zero levels together with the
 * non-zero level that ends it (the classic run-length source extension; Huffman, 1952, over
 * the extended alphabet).
 *
 * Conventions of this repository (the paper fixes none of them):
 *  - Z = floor(127 / s) is the longest run a token completes.  Tokens are numbered
 *      z * 2s + j   for a run of z zeros (0 <= z < Z) ended by the non-zero level with rank j,
 *                   j = 0..2s-1 in increasing level order (-s..-1, then 1..s);
 *      2s * Z       for Z zeros and no level after them,
 *    2sZ + 1 <= 255 symbols in all.
 *  - A row is cut into tiles of `tile` elements that are tokenised on their own: levels are
 *    taken in order, a zero extends the run, the Z-th zero of a run sends the token "Z zeros"
 *    and restarts the run, a non-zero level sends (run, level) and restarts the run.  A run
 *    still open at the end of the tile is sent as one "Z zeros" token; the decoder knows the
 *    tile's length and drops the zeros beyond it.
 *  - One Huffman code per worker row from the row's token counts, built and made canonical
 *    exactly as the per-level code above; the bit stream has the same layout (LSB-first,
 *    codewords most significant bit first, tiles back to back without padding).
 *  - Kept beside the stream: the number of bits of every tile (32 bits each) and, for every
 *    group of `group` tiles, the stream bit at which the group starts (64 bits each), the
 *    last entry being the row's total.  Tiles then decode independently.
 */

int ecq_oracle_zrun_max_run(int s) { return (s >= 1 && s <= 127) ? 127 / s : -1; }

int ecq_oracle_zrun_symbols(int s)
{
    int z = ecq_oracle_zrun_max_run(s);
    return z < 0 ? -1 : 2 * s * z + 1;
}

/* Tokens of one tile of len levels; `tokens` must hold len + 1 entries.  Returns their number. */
int64_t ecq_oracle_zrun_tokens(const int8_t *q, int64_t len, int s, uint8_t *tokens)
{
    int Z = ecq_oracle_zrun_max_run(s);
    int64_t count = 0;
    int run = 0;
    for (int64_t i = 0; i < len; ++i) {
        if (q[i] == 0) {
            if (++run == Z) {
                tokens[count++] = (uint8_t)(2 * s * Z);
                run = 0;
            }
        } else {
            int rank = q[i] < 0 ? (int)q[i] + s : (int)q[i] + s - 1;
            tokens[count++] = (uint8_t)(run * 2 * s + rank);
            run = 0;
        }
    }
    if (run > 0) tokens[count++] = (uint8_t)(2 * s * Z);
    return count;
}

/* Token counts of one worker row (all its tiles). */
void ecq_oracle_zrun_histogram(const int8_t *q, int64_t n, int s, int64_t tile, uint64_t *counts)
{
    int A = ecq_oracle_zrun_symbols(s);
    uint8_t *tokens = (uint8_t *)malloc((size_t)tile + 1);
    for (int a = 0; a < A; ++a) counts[a] = 0;
    for (int64_t e0 = 0; e0 < n; e0 += tile) {
        int64_t len = n - e0 < tile ? n - e0 : tile;
        int64_t count = ecq_oracle_zrun_tokens(q + e0, len, s, tokens);
        for (int64_t k = 0; k < count; ++k) counts[tokens[k]] += 1;
    }
    free(tokens);
}

/* A stream row never needs more than this many bytes when the code was built from the row's
 * own token counts: the lengths r*(z+1) for (z, level) and r*Z for "Z zeros" satisfy Kraft's
 * inequality and cost r bits per element covered, and only the one closing token a tile may
 * have covers fewer elements than it is charged for. */
int64_t ecq_oracle_zrun_max_bytes(int64_t n, int s, int64_t tile)
{
    int64_t r = ecq_oracle_code_bits(s), Z = ecq_oracle_zrun_max_run(s);
    int64_t tiles = (n + tile - 1) / tile;
    return ((n * r + tiles * r * Z + 7) / 8 + 3) / 4 * 4;
}

/* Encodes one worker row; returns the total number of bits.  out is zeroed up to out_bytes
 * first and must hold the stream; tile_bits gets ceil(n/tile) entries, group_offsets
 * ceil(tiles/group) + 1. */
int64_t ecq_oracle_zrun_encode(const int8_t *q, int64_t n, int s, const uint8_t *lengths,
                               const uint64_t *codes, uint8_t *out, int64_t out_bytes, int64_t tile,
                               int64_t group, uint32_t *tile_bits, uint64_t *group_offsets)
{
    uint8_t *tokens = (uint8_t *)malloc((size_t)tile + 1);
    memset(out, 0, (size_t)out_bytes);
    int64_t pos = 0, t = 0;
    for (int64_t e0 = 0; e0 < n; e0 += tile, ++t) {
        int64_t len = n - e0 < tile ? n - e0 : tile;
        if (t % group == 0) group_offsets[t / group] = (uint64_t)pos;
        int64_t begin = pos;
        int64_t count = ecq_oracle_zrun_tokens(q + e0, len, s, tokens);
        for (int64_t k = 0; k < count; ++k) {
            int a = tokens[k];
            for (int b = lengths[a] - 1; b >= 0; --b) {        /* most significant bit first */
                if ((codes[a] >> b) & 1u) out[pos >> 3] |= (uint8_t)(1u << (pos & 7));
                ++pos;
            }
        }
        tile_bits[t] = (uint32_t)(pos - begin);
    }
    group_offsets[(t + group - 1) / group] = (uint64_t)pos;
    free(tokens);
    return pos;
}

/* Decodes one tile of len levels whose tokens start at stream bit `start`. */
void ecq_oracle_zrun_decode(const uint8_t *stream, uint64_t start, int64_t len, int s,
                            const uint8_t *lengths, const uint64_t *codes, int8_t *q)
{
    int Z = ecq_oracle_zrun_max_run(s), A = ecq_oracle_zrun_symbols(s);
    uint64_t pos = start;
    int64_t i = 0;
    while (i < len) {
        uint64_t word = 0;
        int bits = 0, found = -1;
        while (found < 0 && bits < 64) {
            word = (word << 1) | (uint64_t)((stream[pos >> 3] >> (pos & 7)) & 1u);
            ++pos;
            ++bits;
            for (int a = 0; a < A; ++a)
                if (lengths[a] == bits && codes[a] == word) found = a;
        }
        if (found < 0) break;                                   /* not a stream of this code */
        int zeros = found == 2 * s * Z ? Z : found / (2 * s);
        for (int k = 0; k < zeros && i < len; ++k) q[i++] = 0;
        if (found != 2 * s * Z && i < len) {
            int rank = found % (2 * s);
            q[i++] = (int8_t)(rank < s ? rank - s : rank - s + 1);
        }
    }
}
