/*
 * ecq.h -- C ABI of the ECQ-SGD hot path for AMD MI355X (gfx950).
 *
 * The library implements, on one GPU and with the P data-parallel workers laid out as a
 * resident batch, the per-iteration compression codec of Error Compensated Quantized SGD
 * (Wu, Huang, Huang, Zhang, ICML 2018), Section 4:
 *
 *     v   = g + alpha*h                          compensate             Eq. (7)
 *     g~  = ||v|| * sgn(v) * xi(|v|; ||v||)      stochastic quantiser   Eq. (8)-(9)
 *     encode g~ as r = ceil(log2(2s+1)) bits per element + one fp32 scale per bucket
 *     h  <- beta*h + (g - g~)                    error accumulator      Eq. (6)
 *     g~_avg = (1/P) sum_p g~_p                  aggregation            Eq. (4), Alg. 1
 *
 * General conventions
 *  - Every data pointer is a DEVICE pointer owned by the caller.  The library allocates
 *    nothing, frees nothing and keeps no state between calls: the state of the method is the
 *    caller's `h` plus the (seed, step) pair; the caller passes step = t at iteration t.
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream) and returns without synchronising.
 *  - Return value: ECQ_OK (0) or a negative ecq_status.  Argument errors are found on the
 *    host before anything is launched and leave all outputs untouched.
 *  - Non-finite inputs give undefined results (no error).
 *
 * Data layout (P = workers, N = n elements per worker, b = bucket, nb = ceil(N/b))
 *  - g, h   : float32 [P][gh_stride], row p = worker p's flat gradient / accumulated error.
 *  - scales : float32 [P][scale_stride]; scales[p][k] = norm ||v|| of bucket k of worker p,
 *             bucket k = elements [k*b, min((k+1)*b, N)).
 *  - codes  : bytes [P][code_stride]; row p is one contiguous bit stream, element i's code
 *             c = level + s (0..2s) in stream bits [i*r, (i+1)*r), stream bit j = bit (j & 7)
 *             of byte (j >> 3).  The first ecq_row_bytes() bytes of every row are written in
 *             full (pad bits zero); bytes from there to code_stride are never touched.
 *  - Strides only have to satisfy the divisibility stated with ecq_shape, but rows that start
 *    on 128-byte boundaries (gh_stride and scale_stride multiples of 32 floats, code_stride a
 *    multiple of 128 bytes, 128-byte aligned base pointers) let every wave load and store
 *    whole cache lines: measured 4-5 % more bandwidth on MI355X.
 *
 * Arithmetic: IEEE binary32, round to nearest even, one rounding per operation (no fused
 * multiply-add), denormals kept.  Randomness: one word per element of Philox4x32-10
 * (Salmon et al., SC'11): word (i & 3) of the block with counter
 * (low32(i >> 2), p, step_lo, step_hi) and key (seed_lo, seed_hi); its top 24 bits form the
 * uniform u in [0,1) that decides the rounding direction of Eq. (9).  Results therefore do
 * not depend on launch geometry.
 */
#ifndef ECQ_H
#define ECQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ECQ_OK = 0,
    ECQ_ERR_NULL = -1,    /* a required pointer is NULL                                   */
    ECQ_ERR_SHAPE = -2,   /* n <= 0, n > ECQ_MAX_N or workers <= 0 or workers > 65535      */
    ECQ_ERR_LEVELS = -3,  /* s outside 1..127                                             */
    ECQ_ERR_BUCKET = -4,  /* bucket not a positive multiple of 8                           */
    ECQ_ERR_STRIDE = -5,  /* a row stride too small for its row or not suitably divisible */
    ECQ_ERR_ALIGN = -6,   /* a base pointer is not aligned as documented                  */
    ECQ_ERR_LAUNCH = -7,  /* the HIP runtime refused a launch                             */
    ECQ_ERR_PARAM = -8    /* alpha, beta or norm out of range, or an unknown tuning value  */
} ecq_status;

/* Largest n: element index i enters the Philox counter as low32(i >> 2). */
#define ECQ_MAX_N (((int64_t)1) << 34)

/* The scaling factor ||v|| of Eq. (8); the paper names both choices (text after Eq. (8)).
 *   ECQ_NORM_LINF  max |v_i| over the bucket (order-free).
 *   ECQ_NORM_L2    sqrt of the sum of fl(v_i^2), the sum taken over a balanced binary tree by
 *                  element index (the bucket padded with zeros to a power of two), then one
 *                  correctly rounded square root.  Squares must not overflow binary32.  Squares
 *                  that underflow are handled as Eq. (8)-(9) read: a computed norm of 0 gives
 *                  level 0 everywhere, and an element that exceeds the computed norm (possible
 *                  when its square is denormal) takes level s, the end of the grid.
 * Either norm takes any bucket that is a positive multiple of 8, up to one that holds the whole
 * row (n <= bucket: one norm per worker, Eq. (8) without buckets).
 * Buckets beyond 32768 elements take two passes over g and h (20 instead of 12 bytes per
 * element); with ECQ_NORM_L2 the first pass borrows a few bytes per 8192 elements of the
 * worker's row of `codes`, which the second pass then overwrites as documented. */
#define ECQ_NORM_LINF 0
#define ECQ_NORM_L2 1

typedef struct {
    int64_t n;            /* N: elements per worker, 1..ECQ_MAX_N                           */
    int32_t workers;      /* P: 1..65535                                                   */
    int32_t bucket;       /* b: positive multiple of 8 (every bucket starts on a byte)      */
    int32_t s;            /* non-zero quantisation levels, 1..127 (r = 2..8 bits)          */
    int32_t norm;         /* scaling factor ||v||: ECQ_NORM_LINF (0) or ECQ_NORM_L2 (1)     */
    int64_t gh_stride;    /* floats between worker rows of g and of h: >= n, multiple of 4 */
    int64_t code_stride;  /* BYTES between worker rows of codes: >= row bytes, mult. of 4  */
    int64_t scale_stride; /* floats between worker rows of scales: >= nb                   */
} ecq_shape;

/* Optional launch tuning; pass NULL for the defaults.  Results never depend on it. */
typedef struct {
    int32_t path;          /* 0 = choose; 1 = bucket-in-registers single pass;
                              2 = two-pass (norm kernel, then quantise kernel)             */
    int32_t waves_per_bucket; /* 0 = choose; else 1,2,4,8,16 (path 1, buckets >= 256)      */
    int32_t block_threads; /* 0 = choose; else 64..1024, multiple of 64                    */
    int32_t block_order;   /* path 1, buckets >= 256.  0 = choose; 1 = blocks in address order,
                              worker rows issued in launches of about 2^28 elements; 2 = the
                              same with one contiguous region of blocks per XCD; 3 = address
                              order, all rows in one launch                               */
} ecq_tuning;

/* r = ceil(log2(2s+1)) bits per encoded element (Section 4, cost paragraph);
 * negative ecq_status for s outside 1..127. */
int ecq_code_bits(int s);

/* *bytes = ceil(n*r/8), the encoded length of one worker row without its scales. */
int ecq_row_bytes(int64_t n, int s, int64_t *bytes);

/* *nb = ceil(n / bucket). */
int ecq_num_buckets(int64_t n, int bucket, int64_t *nb);

/* Host-side check of a shape; what every entry point runs first. */
int ecq_check_shape(const ecq_shape *shape);

/*
 * Eq. (7)-(9) and the fixed-length encoding: quantise v = g + alpha*h of every worker.
 *   g, h   in   device, [P][gh_stride] float32, 16-byte aligned; neither is written.
 *   alpha  in   compensation coefficient, finite, >= 0.
 *   seed, step  select the random stream; use step = iteration number.
 *   codes  out  device, [P][code_stride] bytes, 4-byte aligned.
 *   scales out  device, [P][scale_stride] float32.
 */
int ecq_quantize(const ecq_shape *shape, const float *g, const float *h, float alpha,
                 uint64_t seed, uint64_t step, uint8_t *codes, float *scales, void *stream);

/*
 * Eq. (6): h <- beta*h + (g - g~), with g~ decoded from (codes, scales) as
 * scales[p][i/b] * fl(|q|/s) carrying the sign of q = code - s (Eq. (8)).
 *   g      in      device, [P][gh_stride] float32, 16-byte aligned.
 *   codes, scales  in, as written by ecq_quantize.  A code beyond 2s (no message written by
 *                  this library holds one) decodes as level 0 here and in the aggregation.
 *   beta   in      time-decaying factor, 0 <= beta <= 1.
 *   h      in/out  device, [P][gh_stride] float32, 16-byte aligned, updated in place.
 */
int ecq_error_update(const ecq_shape *shape, const float *g, const uint8_t *codes,
                     const float *scales, float beta, float *h, void *stream);

/*
 * The per-worker part of one iteration of Alg. 1 in a single pass over g and h: quantise
 * g + alpha*h with the current h (Eq. (7)-(9)), encode, and move h to its next value
 * (Eq. (6)).  Bit-identical to ecq_quantize followed by ecq_error_update.  h is updated in
 * place; g is not written.
 */
int ecq_quantize_update(const ecq_shape *shape, const float *g, float *h, float alpha,
                        float beta, uint64_t seed, uint64_t step, uint8_t *codes, float *scales,
                        void *stream);

/* The same with explicit launch tuning (NULL = defaults); used to show that results do not
 * depend on launch geometry and to sweep configurations. */
int ecq_quantize_update_ex(const ecq_shape *shape, const float *g, float *h, float alpha,
                           float beta, uint64_t seed, uint64_t step, uint8_t *codes,
                           float *scales, const ecq_tuning *tuning, void *stream);

/*
 * Eq. (4) / Alg. 1 "compute global gradients": out[i] = (sum_{p=0}^{P-1} g~_p[i]) / P, the
 * sum taken in the order p = 0, 1, ..., P-1 in binary32, followed by one division by
 * (float)P.  gh_stride of the shape is not used.
 *   codes, scales  in   all P workers' messages.
 *   out            out  device, [n] float32, 16-byte aligned.
 */
int ecq_dequant_aggregate(const ecq_shape *shape, const uint8_t *codes, const float *scales,
                          float *out, void *stream);

/*
 * Eq. (4) in full, i.e. Alg. 1 "compute global gradients" followed by "update model
 * parameters": g~avg as in ecq_dequant_aggregate, then w[i] <- w[i] - fl(eta * g~avg[i]),
 * fused so the averaged gradient need not travel through memory.
 *   eta  in      learning rate, finite.
 *   w    in/out  device, [n] float32, 16-byte aligned: the model replica, updated in place.
 *   out  out     device, [n] float32, 16-byte aligned, or NULL: g~avg is also stored there.
 */
int ecq_dequant_aggregate_sgd(const ecq_shape *shape, const uint8_t *codes, const float *scales,
                              float eta, float *w, float *out, void *stream);

/*
 * d_k of Section 4's cost paragraph: counts[p][c] = number of elements of worker p whose code
 * is c (c = level + s, 0..2s).  Entropy coding of worker p's message then needs at most
 * sum_k d_k log2(d/d_k) bits (see ecq_entropy_bound_bits).
 *   codes   in   as written by ecq_quantize / ecq_quantize_update.
 *   counts  out  device, uint64 [P][count_stride], count_stride >= 2s+1, 8-byte aligned; the
 *                first 2s+1 counters of every row are overwritten, the rest left alone.
 */
int ecq_level_histogram(const ecq_shape *shape, const uint8_t *codes, uint64_t *counts,
                        int64_t count_stride, void *stream);

/*
 * HOST function on HOST memory: *bits = sum_k d_k log2(d / d_k) over one histogram row of
 * `bins` counters (d = sum_k d_k; empty levels contribute nothing), in float64.
 */
int ecq_entropy_bound_bits(const uint64_t *counts_host, int bins, double *bits);

/*
 * Huffman coding of the quantised levels.  Section 4's cost paragraph names Huffman encoding
 * as the way to go below r bits per element, and the paper's communication-cost figures assume
 * it.  One code per worker row, built from that row's counts d_k.  Conventions (the paper
 * fixes none of them):
 *  - construction: leaves are the levels with d_k > 0, numbered by their code c = level + s;
 *    the two live nodes that come first in the order (weight, number) are merged into a new
 *    node that takes the next free number (2s+1, 2s+2, ...); a level's codeword length is its
 *    depth; a row with a single occupied level gives it length 1; unused levels get length 0;
 *  - codewords are canonical: levels sorted by (length, c), first codeword 0, each next one
 *    is (previous + 1) shifted left by the growth in length;
 *  - the stream is LSB-first like the fixed-length one (stream bit j is bit (j & 7) of byte
 *    (j >> 3)); a codeword is written most significant bit first; pad bits are zero;
 *  - a row is cut into tiles of ECQ_HUFFMAN_TILE elements whose bit offsets are kept, so
 *    tiles encode and decode independently.
 * A code built from a row's own counts never needs more than n*r bits for that row, so a
 * stream row of ecq_row_bytes() bytes (rounded up to 4) always suffices.
 */
#define ECQ_HUFFMAN_TILE 1024

/* *tiles = ceil(n / ECQ_HUFFMAN_TILE). */
int ecq_huffman_num_tiles(int64_t n, int64_t *tiles);

/*
 * Codeword lengths and canonical codewords of every worker row from its level counts.
 *   counts     in   device, uint64 [workers][table_stride], as written by ecq_level_histogram
 *                   (each row must sum to at most ECQ_MAX_N: no codeword then exceeds 63 bits).
 *   lengths    out  device, uint8  [workers][table_stride]: bits of level c's codeword, 0 = unused.
 *   codewords  out  device, uint64 [workers][table_stride]: the codeword as an integer whose
 *                   most significant of `length` bits is sent first.  8-byte aligned.
 * table_stride >= 2s+1; only the first 2s+1 entries of each row are written.
 */
int ecq_huffman_build(int workers, int s, const uint64_t *counts, int64_t table_stride,
                      uint8_t *lengths, uint64_t *codewords, void *stream);

/*
 * Re-encodes every worker's fixed-length message with its row's Huffman code.
 *   codes         in   as written by ecq_quantize / ecq_quantize_update (shape describes it).
 *   lengths, codewords  in  as written by ecq_huffman_build (same table_stride).
 *   streams       out  device, bytes [workers][stream_stride], 4-byte aligned, stream_stride a
 *                      multiple of 4 and >= ecq_row_bytes() rounded up to 4.  Row p receives
 *                      tile_offsets[p][tiles] bits; the bytes that hold them, rounded up to a
 *                      multiple of 4, are written in full (pad bits zero), the rest of the row
 *                      is left alone.
 *   tile_offsets  out  device, uint64 [workers][offset_stride], offset_stride >= tiles + 1:
 *                      entry t is the stream bit at which tile t of the row starts, entry
 *                      `tiles` the row's total number of bits.
 * Tables that do not belong to the codes (a level present in the message but with length 0,
 * or a total beyond the stream row) give a meaningless stream, never an out-of-range access.
 */
int ecq_huffman_encode(const ecq_shape *shape, const uint8_t *codes, const uint8_t *lengths,
                       const uint64_t *codewords, int64_t table_stride, uint8_t *streams,
                       int64_t stream_stride, uint64_t *tile_offsets, int64_t offset_stride,
                       void *stream);

/*
 * Inverse of ecq_huffman_encode: rebuilds the fixed-length message (which
 * ecq_dequant_aggregate and ecq_error_update read) from streams, tile offsets and tables.
 *   codes  out  device, [workers][code_stride] bytes; the first ecq_row_bytes() bytes of every
 *               row are written in full (pad bits zero).
 */
int ecq_huffman_decode(const ecq_shape *shape, const uint8_t *streams, int64_t stream_stride,
                       const uint64_t *tile_offsets, int64_t offset_stride, const uint8_t *lengths,
                       const uint64_t *codewords, int64_t table_stride, uint8_t *codes,
                       void *stream);

/*
 * Zero-run Huffman coding of the quantised levels: the entropy coding of Section 4's cost
 * paragraph for messages that are mostly zeros.  That paragraph bounds the coded length by
 * sum_k d_k log2(d/d_k) bits, which is often far below one bit per element, while a Huffman code
 * over single levels (above) spends at least one.  Here the Huffman code is taken over TOKENS: a
 * run of zero levels together with the non-zero level that ends it.  Conventions (the paper
 * fixes none of them):
 *  - Z = floor(127 / s).  Token z*2s + j stands for z zeros (0 <= z < Z) followed by the non-zero
 *    level of rank j (levels -s..-1, 1..s in increasing order); token 2sZ for Z zeros and no level:
 *    2sZ + 1 <= 255 symbols;
 *  - a row is cut into tiles of ECQ_ZRUN_TILE elements that are tokenised on their own: levels
 *    are taken in order, the Z-th zero of a run sends "Z zeros" and restarts the run, a non-zero
 *    level sends (run, level); a run still open at the end of the tile is sent as one "Z zeros"
 *    token, and the decoder drops the zeros beyond the tile's end;
 *  - one Huffman code per worker row from the row's token counts, constructed and made canonical
 *    as for ecq_huffman_build; the stream has the same layout (LSB-first, codewords most
 *    significant bit first), tiles back to back;
 *  - beside the stream travel the number of bits of every tile (32 bits each) and the stream bit
 *    at which every group of ECQ_ZRUN_GROUP tiles starts (64 bits each; one more entry holds the
 *    row's total), so tiles decode independently: 1/128 bit per element in all.
 * Measured on the synthetic workloads: 0.5-1.5 % above the bound (index excluded), where the
 * per-level code needs 1.0-1.25 bits per element.  A code beyond 2s is taken as level 0.
 */
#define ECQ_ZRUN_TILE 4096
#define ECQ_ZRUN_GROUP 64

/* *max_run = Z, *symbols = 2sZ + 1 (either pointer may be NULL). */
int ecq_zrun_symbols(int s, int *max_run, int *symbols);

/* *tiles = ceil(n / ECQ_ZRUN_TILE), *groups = ceil(tiles / ECQ_ZRUN_GROUP) (either may be NULL). */
int ecq_zrun_num_tiles(int64_t n, int64_t *tiles, int64_t *groups);

/*
 * *bytes = a stream row that always suffices when the code was built from the row's own token
 * counts (a multiple of 4): the lengths r*(z+1) for (z, level) and r*Z for "Z zeros" satisfy
 * Kraft's inequality and cost r bits per element covered, and only the closing token of a tile
 * covers fewer elements than it is charged for, so no row needs more than n*r + tiles*r*Z bits.
 */
int ecq_zrun_stream_bytes(int64_t n, int s, int64_t *bytes);

/*
 * counts[p][t] = how often token t occurs in worker p's message.
 *   codes   in   as written by ecq_quantize / ecq_quantize_update.
 *   counts  out  device, uint64 [P][count_stride], count_stride >= 2sZ + 1, 8-byte aligned; the
 *                first 2sZ + 1 counters of every row are overwritten, the rest left alone.
 */
int ecq_zrun_histogram(const ecq_shape *shape, const uint8_t *codes, uint64_t *counts, int64_t count_stride,
                       void *stream);

/* ecq_huffman_build over the token alphabet: lengths and canonical codewords of the 2sZ + 1
 * tokens of every worker row (table_stride >= 2sZ + 1). */
int ecq_zrun_build(int workers, int s, const uint64_t *counts, int64_t table_stride, uint8_t *lengths,
                   uint64_t *codewords, void *stream);

/*
 * Re-encodes every worker's fixed-length message with its row's token code.
 *   codes          in   as written by ecq_quantize / ecq_quantize_update (shape describes it).
 *   lengths, codewords  in  as written by ecq_zrun_build (same table_stride).
 *   streams        out  device, bytes [workers][stream_stride], 4-byte aligned, stream_stride a
 *                       multiple of 4 and >= ecq_zrun_stream_bytes().  The bytes that hold row p's
 *                       bits, rounded up to a multiple of 4, are written in full (pad bits zero),
 *                       the rest of the row is left alone.
 *   tile_bits      out  device, uint32 [workers][tile_stride], tile_stride >= tiles: the number of
 *                       stream bits of every tile.
 *   group_offsets  out  device, uint64 [workers][group_stride], group_stride >= groups + 1: entry
 *                       j is the stream bit at which tile j * ECQ_ZRUN_GROUP starts, entry `groups`
 *                       the row's total.  8-byte aligned.
 * Tables that do not belong to the codes give a meaningless stream, never an out-of-range access.
 */
int ecq_zrun_encode(const ecq_shape *shape, const uint8_t *codes, const uint8_t *lengths, const uint64_t *codewords,
                    int64_t table_stride, uint8_t *streams, int64_t stream_stride, uint32_t *tile_bits,
                    int64_t tile_stride, uint64_t *group_offsets, int64_t group_stride, void *stream);

/*
 * Inverse of ecq_zrun_encode: rebuilds the fixed-length message from streams, index and tables.
 *   codes  out  device, [workers][code_stride] bytes; the first ecq_row_bytes() bytes of every row
 *               are written in full (pad bits zero).
 */
int ecq_zrun_decode(const ecq_shape *shape, const uint8_t *streams, int64_t stream_stride, const uint32_t *tile_bits,
                    int64_t tile_stride, const uint64_t *group_offsets, int64_t group_stride, const uint8_t *lengths,
                    const uint64_t *codewords, int64_t table_stride, uint8_t *codes, void *stream);

/*
 * The random words of Eq. (9)'s rounding decision, for inspection: words[j] is the word
 * element i0 + j of worker p consumes at iteration `step`.  words: device, [count] uint32.
 */
int ecq_philox_words(uint64_t seed, uint64_t step, uint32_t p, uint64_t i0, int64_t count,
                     uint32_t *words, void *stream);

/*
 * Self-check, not part of the method: the kernels obtain |v_i| / ||v|| from a per-bucket
 * reciprocal instead of one full division per element.  This call compares that routine with
 * the plain correctly rounded binary32 division for every divisor significand (2^23 of them,
 * exponents drawn over the whole normal range from `salt`) and `per_divisor` numerators each
 * (same binade, far smaller, denormal, equal, up to an eighth larger), in both of the forms the
 * kernels use, and adds
 * the number of differing results to *mismatches (device, uint64, zeroed by the call).
 * Expected: 0.
 */
int ecq_check_division(int per_divisor, uint32_t salt, uint64_t *mismatches, void *stream);

/*
 * Bandwidth calibration, not part of the method: out[i] = a[i] + b[i] over n floats
 * (two reads and one write of 4 bytes per element, the same traffic mix as the fused pass),
 * and a plain copy out[i] = a[i].  All pointers device, 16-byte aligned.
 */
int ecq_calib_add(const float *a, const float *b, float *out, int64_t n, void *stream);
int ecq_calib_copy(const float *a, float *out, int64_t n, void *stream);

/*
 * Calibration of the aggregation's access pattern, not part of the method: reads every
 * worker's row of `codes` exactly as ecq_dequant_aggregate does (a wave takes 128*r contiguous
 * bytes of each of the P rows for its 1024 outputs), adds the words up and writes n floats,
 * with no decoding and no norms.  codes, out as for ecq_dequant_aggregate; only the whole runs
 * of 1024 outputs are written.
 */
int ecq_calib_gather(const ecq_shape *shape, const uint8_t *codes, float *out, void *stream);

/* Static, human-readable text for a status value. */
const char *ecq_status_string(int status);

/* Library version, major*10000 + minor*100 + patch. */
int ecq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ECQ_H */
