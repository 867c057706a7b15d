// C ABI of the ECQ-SGD codec: argument checks on the host, then kernel launches.
// Declarations and the contract of every entry point are in include/ecq.h.
#include <cmath>
#include <cstdint>

#include "ecq_internal.hpp"

namespace ecq {

static int code_bits(int s)
{
    if (s < 1 || s > 127) return ECQ_ERR_LEVELS;
    int r = 0;
    while ((1 << r) < 2 * s + 1) ++r;                         // r = ceil(log2(2s+1))
    return r;
}

static bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static int check_shape(const ecq_shape *sh)
{
    if (!sh) return ECQ_ERR_NULL;
    if (sh->n <= 0 || sh->n > ECQ_MAX_N || sh->workers <= 0 || sh->workers > 65535) return ECQ_ERR_SHAPE;
    if (sh->s < 1 || sh->s > 127) return ECQ_ERR_LEVELS;
    if (sh->bucket <= 0 || (sh->bucket & 7) != 0) return ECQ_ERR_BUCKET;
    if (sh->norm != ECQ_NORM_LINF && sh->norm != ECQ_NORM_L2) return ECQ_ERR_PARAM;
    const int r = code_bits(sh->s);
    const int64_t row_bytes = (sh->n * r + 7) / 8;
    const int64_t nb = (sh->n + sh->bucket - 1) / sh->bucket;
    if (sh->gh_stride < sh->n || (sh->gh_stride & 3) != 0) return ECQ_ERR_STRIDE;
    if (sh->code_stride < row_bytes || (sh->code_stride & 3) != 0) return ECQ_ERR_STRIDE;
    if (sh->scale_stride < nb) return ECQ_ERR_STRIDE;
    return ECQ_OK;
}

static Args make_args(const ecq_shape &sh)
{
    Args a{};
    a.n = sh.n;
    a.nb = (sh.n + sh.bucket - 1) / sh.bucket;
    a.gh_stride = sh.gh_stride;
    a.code_stride = sh.code_stride;
    a.scale_stride = sh.scale_stride;
    a.r = code_bits(sh.s);
    a.row_bytes = (sh.n * a.r + 7) / 8;
    a.workers = sh.workers;
    a.bucket = sh.bucket;
    a.s = sh.s;
    a.norm_l2 = sh.norm == ECQ_NORM_L2;
    return a;
}

static void set_stream_key(Args &a, uint64_t seed, uint64_t step)
{
    a.key0 = (uint32_t)seed;
    a.key1 = (uint32_t)(seed >> 32);
    a.step_lo = (uint32_t)step;
    a.step_hi = (uint32_t)(step >> 32);
}

// Chooses how a bucket is mapped to lanes.  Single pass when the bucket has fewer than 256
// elements (a group of lanes inside one wave) or at most 32768 (a team of up to 16 waves holding
// up to 8 float4 per lane); two passes beyond that.
int make_plan(const ecq_shape &sh, const ecq_tuning *tu, Plan *plan)
{
    Plan pl{};
    const int b = sh.bucket;
    int path = 0, waves = 0, threads = 0;
    if (tu) {
        if (tu->block_order < 0 || tu->block_order > 3) return ECQ_ERR_PARAM;
        path = tu->path;
        waves = tu->waves_per_bucket;
        threads = tu->block_threads;
        if (path < 0 || path > 2) return ECQ_ERR_PARAM;
        if (waves != 0 && waves != 1 && waves != 2 && waves != 4 && waves != 8 && waves != 16) return ECQ_ERR_PARAM;
        if (threads != 0 && (threads < 64 || threads > 1024 || (threads & 63) != 0)) return ECQ_ERR_PARAM;
    }
    const bool small_ok = b >= 8 && b < 256;
    const bool team_ok = b >= 256 && b <= 32768;
    // The l2 sum has a fixed tree order: the single-pass mappings reproduce it, and so does the
    // two-pass route for buckets beyond 32768 (sums of 8192-element pieces, then a tree over the
    // pieces), but not the two-pass route forced on a shorter bucket.
    if (sh.norm == ECQ_NORM_L2 && path == 2 && b <= 32768) return ECQ_ERR_PARAM;
    if (path == 0) path = (small_ok || team_ok) ? 1 : 2;
    if (path == 1 && !(small_ok || team_ok)) return ECQ_ERR_PARAM;
    pl.path = path;
    pl.block_threads = 256;
    if (path == 1 && small_ok) {
        pl.lanes_per_bucket = b / 4;
    } else if (path == 1) {
        const int chunks = (b + 255) / 256;                    // float4-per-lane wave loads per bucket
        // Measured on MI355X: two float4 of g and of h per lane stream best; one wave keeps up to
        // four per lane before a second wave (and with it an LDS exchange and a barrier) pays.
        if (waves == 0) {
            waves = 1;
            if (chunks > 4)
                while (waves * 2 < chunks && waves < 16) waves *= 2;
            // 33..64 chunks: eight waves with eight float4 per lane leave room for a second block on
            // the CU (77 % of peak at 16384 elements against 62 % for sixteen waves with four).
            if (chunks > 32 && chunks <= 64) waves = 8;
            // A message with fewer single-wave buckets than the chip holds waves (4 per SIMD) is
            // bound by latency, not by bandwidth: two waves per bucket, half the chain each
            // (21.1 -> 19.1 us at 8 rows of 1 M elements in buckets of 1024).
            if (waves == 1 && chunks >= 3 && threads == 0 && (int64_t)sh.workers * ((sh.n + b - 1) / b) < 16384) {
                waves = 2;
                threads = 128;
            }
        }
        int vec = 1;
        while (vec * waves < chunks) vec *= 2;
        if (vec > 8) return ECQ_ERR_PARAM;                     // the bucket would not fit the team's registers
        if (threads == 0) {
            threads = (waves == 1 && vec == 4) ? 256 : 512;
            if (waves * 64 > threads) threads = waves * 64;
        }
        if (threads % (waves * 64) != 0) return ECQ_ERR_PARAM;
        pl.waves_per_bucket = waves;
        pl.vec_per_lane = vec;
        pl.block_threads = threads;
        const int order = tu ? tu->block_order : 0;
        pl.xcd_striped = order == 2;
        if (pl.xcd_striped && (((int64_t)sh.workers * ((sh.n + b - 1) / b)) >> 28) > 0) pl.xcd_striped = 0;
        // About 2^28 elements per launch (order 3: everything in one launch).
        const int64_t rows = (((int64_t)1 << 28) + sh.n / 2) / sh.n;
        pl.rows_per_launch = order == 3 ? 0 : (int)(rows < 1 ? 1 : (rows > sh.workers ? sh.workers : rows));
    }
    *plan = pl;
    return ECQ_OK;
}

static int run_quantize(const ecq_shape *sh, const float *g, const float *h, float alpha, float beta,
                        uint64_t seed, uint64_t step, uint8_t *codes, float *scales,
                        const ecq_tuning *tuning, bool update_h, void *stream)
{
    const int st = check_shape(sh);
    if (st != ECQ_OK) return st;
    if (!g || !h || !codes || !scales) return ECQ_ERR_NULL;
    if (!aligned(g, 16) || !aligned(h, 16) || !aligned(codes, 4) || !aligned(scales, 4)) return ECQ_ERR_ALIGN;
    if (!std::isfinite(alpha) || alpha < 0.0f) return ECQ_ERR_PARAM;
    if (update_h && !(beta >= 0.0f && beta <= 1.0f)) return ECQ_ERR_PARAM;
    // A bucket that holds the whole row (Eq. (8) without buckets) is the same as any other that
    // does: one norm, zeros beyond the row's end change neither norm.  Take the tightest size a
    // single-pass mapping accepts, so that the cost follows the row and not the bucket.
    ecq_shape shape = *sh;
    if ((int64_t)shape.bucket >= shape.n) {
        const int64_t n8 = (shape.n + 7) / 8 * 8;
        int64_t b = n8;
        if (n8 <= 128) {
            b = 8;
            while (b < n8) b *= 2;
        } else if (n8 < 256) {
            b = 256;
        }
        shape.bucket = (int32_t)b;
    }
    Plan plan;
    const int ps = make_plan(shape, tuning, &plan);
    if (ps != ECQ_OK) return ps;
    Args a = make_args(shape);
    a.g = g;
    a.h = const_cast<float *>(h);
    a.codes = codes;
    a.scales = scales;
    a.alpha = alpha;
    a.beta = beta;
    set_stream_key(a, seed, step);
    return launch_quantize(a, plan, update_h, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

}  // namespace ecq

extern "C" {

int ecq_code_bits(int s) { return ecq::code_bits(s); }

int ecq_row_bytes(int64_t n, int s, int64_t *bytes)
{
    if (!bytes) return ECQ_ERR_NULL;
    const int r = ecq::code_bits(s);
    if (r < 0) return r;
    if (n < 0 || n > ECQ_MAX_N) return ECQ_ERR_SHAPE;
    *bytes = (n * r + 7) / 8;
    return ECQ_OK;
}

int ecq_num_buckets(int64_t n, int bucket, int64_t *nb)
{
    if (!nb) return ECQ_ERR_NULL;
    if (n < 0 || n > ECQ_MAX_N) return ECQ_ERR_SHAPE;
    if (bucket <= 0 || (bucket & 7) != 0) return ECQ_ERR_BUCKET;
    *nb = (n + bucket - 1) / bucket;
    return ECQ_OK;
}

int ecq_check_shape(const ecq_shape *shape) { return ecq::check_shape(shape); }

int ecq_quantize(const ecq_shape *shape, const float *g, const float *h, float alpha, uint64_t seed,
                 uint64_t step, uint8_t *codes, float *scales, void *stream)
{
    return ecq::run_quantize(shape, g, h, alpha, 0.0f, seed, step, codes, scales, nullptr, false, stream);
}

int ecq_quantize_update(const ecq_shape *shape, const float *g, float *h, float alpha, float beta,
                        uint64_t seed, uint64_t step, uint8_t *codes, float *scales, void *stream)
{
    return ecq::run_quantize(shape, g, h, alpha, beta, seed, step, codes, scales, nullptr, true, stream);
}

int ecq_quantize_update_ex(const ecq_shape *shape, const float *g, float *h, float alpha, float beta,
                           uint64_t seed, uint64_t step, uint8_t *codes, float *scales,
                           const ecq_tuning *tuning, void *stream)
{
    return ecq::run_quantize(shape, g, h, alpha, beta, seed, step, codes, scales, tuning, true, stream);
}

int ecq_error_update(const ecq_shape *shape, const float *g, const uint8_t *codes, const float *scales,
                     float beta, float *h, void *stream)
{
    const int st = ecq::check_shape(shape);
    if (st != ECQ_OK) return st;
    if (!g || !h || !codes || !scales) return ECQ_ERR_NULL;
    if (!ecq::aligned(g, 16) || !ecq::aligned(h, 16) || !ecq::aligned(codes, 4) || !ecq::aligned(scales, 4))
        return ECQ_ERR_ALIGN;
    if (!(beta >= 0.0f && beta <= 1.0f)) return ECQ_ERR_PARAM;
    ecq::Args a = ecq::make_args(*shape);
    a.g = g;
    a.h = h;
    a.codes = const_cast<uint8_t *>(codes);
    a.scales = const_cast<float *>(scales);
    a.beta = beta;
    return ecq::launch_error_update(a, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

int ecq_dequant_aggregate(const ecq_shape *shape, const uint8_t *codes, const float *scales, float *out,
                          void *stream)
{
    const int st = ecq::check_shape(shape);
    if (st != ECQ_OK) return st;
    if (!codes || !scales || !out) return ECQ_ERR_NULL;
    if (!ecq::aligned(out, 16) || !ecq::aligned(codes, 4) || !ecq::aligned(scales, 4)) return ECQ_ERR_ALIGN;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    a.scales = const_cast<float *>(scales);
    a.out = out;
    return ecq::launch_dequant_aggregate(a, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

int ecq_dequant_aggregate_sgd(const ecq_shape *shape, const uint8_t *codes, const float *scales, float eta,
                              float *w, float *out, void *stream)
{
    const int st = ecq::check_shape(shape);
    if (st != ECQ_OK) return st;
    if (!codes || !scales || !w) return ECQ_ERR_NULL;
    if (!ecq::aligned(w, 16) || !ecq::aligned(out, 16) || !ecq::aligned(codes, 4) || !ecq::aligned(scales, 4))
        return ECQ_ERR_ALIGN;
    if (!std::isfinite(eta)) return ECQ_ERR_PARAM;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    a.scales = const_cast<float *>(scales);
    a.out = out;
    a.w = w;
    a.eta = eta;
    return ecq::launch_dequant_aggregate(a, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

int ecq_level_histogram(const ecq_shape *shape, const uint8_t *codes, uint64_t *counts, int64_t count_stride,
                        void *stream)
{
    const int st = ecq::check_shape(shape);
    if (st != ECQ_OK) return st;
    if (!codes || !counts) return ECQ_ERR_NULL;
    if (count_stride < 2 * (int64_t)shape->s + 1) return ECQ_ERR_STRIDE;
    if (!ecq::aligned(codes, 4) || !ecq::aligned(counts, 8)) return ECQ_ERR_ALIGN;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    return ecq::launch_level_histogram(a, reinterpret_cast<unsigned long long *>(counts), count_stride,
                                       static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_entropy_bound_bits(const uint64_t *counts_host, int bins, double *bits)
{
    if (!counts_host || !bits) return ECQ_ERR_NULL;
    if (bins < 1 || bins > 255) return ECQ_ERR_LEVELS;
    double d = 0.0, sum = 0.0;
    for (int k = 0; k < bins; ++k) d += (double)counts_host[k];
    for (int k = 0; k < bins; ++k)
        if (counts_host[k]) sum += (double)counts_host[k] * std::log2(d / (double)counts_host[k]);
    *bits = sum;
    return ECQ_OK;
}

int ecq_huffman_num_tiles(int64_t n, int64_t *tiles)
{
    if (!tiles) return ECQ_ERR_NULL;
    if (n < 0 || n > ECQ_MAX_N) return ECQ_ERR_SHAPE;
    *tiles = (n + ECQ_HUFFMAN_TILE - 1) / ECQ_HUFFMAN_TILE;
    return ECQ_OK;
}

int ecq_huffman_build(int workers, int s, const uint64_t *counts, int64_t table_stride, uint8_t *lengths,
                      uint64_t *codewords, void *stream)
{
    if (workers <= 0 || workers > 65535) return ECQ_ERR_SHAPE;
    if (s < 1 || s > 127) return ECQ_ERR_LEVELS;
    if (!counts || !lengths || !codewords) return ECQ_ERR_NULL;
    if (table_stride < 2 * (int64_t)s + 1) return ECQ_ERR_STRIDE;
    if (!ecq::aligned(counts, 8) || !ecq::aligned(codewords, 8)) return ECQ_ERR_ALIGN;
    return ecq::launch_huffman_build(workers, 2 * s + 1, reinterpret_cast<const unsigned long long *>(counts),
                                     table_stride, lengths, reinterpret_cast<unsigned long long *>(codewords),
                                     static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

namespace ecq {
// Checks shared by the two Huffman stream entry points.
static int check_huffman(const ecq_shape *sh, const void *codes, const void *lengths, const void *codewords,
                         int64_t table_stride, const void *streams, int64_t stream_stride,
                         const void *tile_offsets, int64_t offset_stride)
{
    const int st = check_shape(sh);
    if (st != ECQ_OK) return st;
    if (!codes || !lengths || !codewords || !streams || !tile_offsets) return ECQ_ERR_NULL;
    const int r = code_bits(sh->s);
    const int64_t row_bytes = (sh->n * r + 7) / 8;
    const int64_t tiles = (sh->n + ECQ_HUFFMAN_TILE - 1) / ECQ_HUFFMAN_TILE;
    if (table_stride < 2 * (int64_t)sh->s + 1) return ECQ_ERR_STRIDE;
    if ((stream_stride & 3) != 0 || stream_stride < (row_bytes + 3) / 4 * 4) return ECQ_ERR_STRIDE;
    if (offset_stride < tiles + 1) return ECQ_ERR_STRIDE;
    if (!aligned(codes, 4) || !aligned(streams, 4) || !aligned(tile_offsets, 8) || !aligned(codewords, 8))
        return ECQ_ERR_ALIGN;
    return ECQ_OK;
}
}  // namespace ecq

int ecq_huffman_encode(const ecq_shape *shape, const uint8_t *codes, const uint8_t *lengths,
                       const uint64_t *codewords, int64_t table_stride, uint8_t *streams, int64_t stream_stride,
                       uint64_t *tile_offsets, int64_t offset_stride, void *stream)
{
    const int st = ecq::check_huffman(shape, codes, lengths, codewords, table_stride, streams, stream_stride,
                                      tile_offsets, offset_stride);
    if (st != ECQ_OK) return st;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    return ecq::launch_huffman_encode(a, lengths, reinterpret_cast<const unsigned long long *>(codewords),
                                      table_stride, reinterpret_cast<uint32_t *>(streams), stream_stride / 4,
                                      reinterpret_cast<unsigned long long *>(tile_offsets), offset_stride,
                                      static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_huffman_decode(const ecq_shape *shape, const uint8_t *streams, int64_t stream_stride,
                       const uint64_t *tile_offsets, int64_t offset_stride, const uint8_t *lengths,
                       const uint64_t *codewords, int64_t table_stride, uint8_t *codes, void *stream)
{
    const int st = ecq::check_huffman(shape, codes, lengths, codewords, table_stride, streams, stream_stride,
                                      tile_offsets, offset_stride);
    if (st != ECQ_OK) return st;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = codes;
    return ecq::launch_huffman_decode(a, lengths, reinterpret_cast<const unsigned long long *>(codewords),
                                      table_stride, reinterpret_cast<const uint32_t *>(streams), stream_stride / 4,
                                      reinterpret_cast<const unsigned long long *>(tile_offsets), offset_stride,
                                      static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

namespace ecq {
static int64_t zrun_stream_bytes(int64_t n, int s)
{
    const int64_t r = code_bits(s), Z = 127 / s;
    const int64_t tiles = (n + ECQ_ZRUN_TILE - 1) / ECQ_ZRUN_TILE;
    return ((n * r + tiles * r * Z + 7) / 8 + 3) / 4 * 4;
}

// Checks shared by the two zero-run stream entry points.
static int check_zrun(const ecq_shape *sh, const void *codes, const void *lengths, const void *codewords,
                      int64_t table_stride, const void *streams, int64_t stream_stride, const void *tile_bits,
                      int64_t tile_stride, const void *group_offsets, int64_t group_stride)
{
    const int st = check_shape(sh);
    if (st != ECQ_OK) return st;
    if (!codes || !lengths || !codewords || !streams || !tile_bits || !group_offsets) return ECQ_ERR_NULL;
    const int64_t tiles = (sh->n + ECQ_ZRUN_TILE - 1) / ECQ_ZRUN_TILE;
    const int64_t groups = (tiles + ECQ_ZRUN_GROUP - 1) / ECQ_ZRUN_GROUP;
    if (table_stride < 2 * (int64_t)sh->s * (127 / sh->s) + 1) return ECQ_ERR_STRIDE;
    if ((stream_stride & 3) != 0 || stream_stride < zrun_stream_bytes(sh->n, sh->s)) return ECQ_ERR_STRIDE;
    if (tile_stride < tiles || group_stride < groups + 1) return ECQ_ERR_STRIDE;
    if (!aligned(codes, 4) || !aligned(streams, 4) || !aligned(tile_bits, 4) || !aligned(group_offsets, 8) ||
        !aligned(codewords, 8))
        return ECQ_ERR_ALIGN;
    return ECQ_OK;
}
}  // namespace ecq

int ecq_zrun_symbols(int s, int *max_run, int *symbols)
{
    if (s < 1 || s > 127) return ECQ_ERR_LEVELS;
    if (max_run) *max_run = 127 / s;
    if (symbols) *symbols = 2 * s * (127 / s) + 1;
    return ECQ_OK;
}

int ecq_zrun_num_tiles(int64_t n, int64_t *tiles, int64_t *groups)
{
    if (n < 0 || n > ECQ_MAX_N) return ECQ_ERR_SHAPE;
    const int64_t t = (n + ECQ_ZRUN_TILE - 1) / ECQ_ZRUN_TILE;
    if (tiles) *tiles = t;
    if (groups) *groups = (t + ECQ_ZRUN_GROUP - 1) / ECQ_ZRUN_GROUP;
    return ECQ_OK;
}

int ecq_zrun_stream_bytes(int64_t n, int s, int64_t *bytes)
{
    if (!bytes) return ECQ_ERR_NULL;
    if (s < 1 || s > 127) return ECQ_ERR_LEVELS;
    if (n < 0 || n > ECQ_MAX_N) return ECQ_ERR_SHAPE;
    *bytes = ecq::zrun_stream_bytes(n, s);
    return ECQ_OK;
}

int ecq_zrun_histogram(const ecq_shape *shape, const uint8_t *codes, uint64_t *counts, int64_t count_stride,
                       void *stream)
{
    const int st = ecq::check_shape(shape);
    if (st != ECQ_OK) return st;
    if (!codes || !counts) return ECQ_ERR_NULL;
    if (count_stride < 2 * (int64_t)shape->s * (127 / shape->s) + 1) return ECQ_ERR_STRIDE;
    if (!ecq::aligned(codes, 4) || !ecq::aligned(counts, 8)) return ECQ_ERR_ALIGN;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    return ecq::launch_zrun_histogram(a, reinterpret_cast<unsigned long long *>(counts), count_stride,
                                      static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_zrun_build(int workers, int s, const uint64_t *counts, int64_t table_stride, uint8_t *lengths,
                   uint64_t *codewords, void *stream)
{
    if (workers <= 0 || workers > 65535) return ECQ_ERR_SHAPE;
    if (s < 1 || s > 127) return ECQ_ERR_LEVELS;
    if (!counts || !lengths || !codewords) return ECQ_ERR_NULL;
    const int symbols = 2 * s * (127 / s) + 1;
    if (table_stride < symbols) return ECQ_ERR_STRIDE;
    if (!ecq::aligned(counts, 8) || !ecq::aligned(codewords, 8)) return ECQ_ERR_ALIGN;
    return ecq::launch_huffman_build(workers, symbols, reinterpret_cast<const unsigned long long *>(counts),
                                     table_stride, lengths, reinterpret_cast<unsigned long long *>(codewords),
                                     static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_zrun_encode(const ecq_shape *shape, const uint8_t *codes, const uint8_t *lengths, const uint64_t *codewords,
                    int64_t table_stride, uint8_t *streams, int64_t stream_stride, uint32_t *tile_bits,
                    int64_t tile_stride, uint64_t *group_offsets, int64_t group_stride, void *stream)
{
    const int st = ecq::check_zrun(shape, codes, lengths, codewords, table_stride, streams, stream_stride, tile_bits,
                                   tile_stride, group_offsets, group_stride);
    if (st != ECQ_OK) return st;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    return ecq::launch_zrun_encode(a, lengths, reinterpret_cast<const unsigned long long *>(codewords), table_stride,
                                   reinterpret_cast<uint32_t *>(streams), stream_stride / 4, tile_bits, tile_stride,
                                   reinterpret_cast<unsigned long long *>(group_offsets), group_stride,
                                   static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_zrun_decode(const ecq_shape *shape, const uint8_t *streams, int64_t stream_stride, const uint32_t *tile_bits,
                    int64_t tile_stride, const uint64_t *group_offsets, int64_t group_stride, const uint8_t *lengths,
                    const uint64_t *codewords, int64_t table_stride, uint8_t *codes, void *stream)
{
    const int st = ecq::check_zrun(shape, codes, lengths, codewords, table_stride, streams, stream_stride, tile_bits,
                                   tile_stride, group_offsets, group_stride);
    if (st != ECQ_OK) return st;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = codes;
    return ecq::launch_zrun_decode(a, lengths, reinterpret_cast<const unsigned long long *>(codewords), table_stride,
                                   reinterpret_cast<const uint32_t *>(streams), stream_stride / 4, tile_bits,
                                   tile_stride, reinterpret_cast<const unsigned long long *>(group_offsets),
                                   group_stride, static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_check_division(int per_divisor, uint32_t salt, uint64_t *mismatches, void *stream)
{
    if (!mismatches) return ECQ_ERR_NULL;
    if (per_divisor < 1 || per_divisor > 65536) return ECQ_ERR_SHAPE;
    if (!ecq::aligned(mismatches, 8)) return ECQ_ERR_ALIGN;
    return ecq::launch_check_division(per_divisor, salt, reinterpret_cast<unsigned long long *>(mismatches),
                                      static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_philox_words(uint64_t seed, uint64_t step, uint32_t p, uint64_t i0, int64_t count, uint32_t *words,
                     void *stream)
{
    if (!words) return ECQ_ERR_NULL;
    if (count <= 0 || count > ECQ_MAX_N) return ECQ_ERR_SHAPE;
    if (!ecq::aligned(words, 4)) return ECQ_ERR_ALIGN;
    return ecq::launch_philox_words((uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)step,
                                    (uint32_t)(step >> 32), p, i0, count, words,
                                    static_cast<hipStream_t>(stream)) == hipSuccess
               ? ECQ_OK
               : ECQ_ERR_LAUNCH;
}

int ecq_calib_add(const float *a, const float *b, float *out, int64_t n, void *stream)
{
    if (!a || !b || !out) return ECQ_ERR_NULL;
    if (n <= 0) return ECQ_ERR_SHAPE;
    if (!ecq::aligned(a, 16) || !ecq::aligned(b, 16) || !ecq::aligned(out, 16)) return ECQ_ERR_ALIGN;
    return ecq::launch_calib_add(a, b, out, n, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

int ecq_calib_copy(const float *a, float *out, int64_t n, void *stream)
{
    if (!a || !out) return ECQ_ERR_NULL;
    if (n <= 0) return ECQ_ERR_SHAPE;
    if (!ecq::aligned(a, 16) || !ecq::aligned(out, 16)) return ECQ_ERR_ALIGN;
    return ecq::launch_calib_copy(a, out, n, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

int ecq_calib_gather(const ecq_shape *shape, const uint8_t *codes, float *out, void *stream)
{
    const int st = ecq::check_shape(shape);
    if (st != ECQ_OK) return st;
    if (!codes || !out) return ECQ_ERR_NULL;
    if (!ecq::aligned(out, 16) || !ecq::aligned(codes, 4)) return ECQ_ERR_ALIGN;
    ecq::Args a = ecq::make_args(*shape);
    a.codes = const_cast<uint8_t *>(codes);
    a.out = out;
    return ecq::launch_calib_gather(a, static_cast<hipStream_t>(stream)) == hipSuccess ? ECQ_OK : ECQ_ERR_LAUNCH;
}

const char *ecq_status_string(int status)
{
    switch (status) {
    case ECQ_OK: return "ok";
    case ECQ_ERR_NULL: return "a required pointer is NULL";
    case ECQ_ERR_SHAPE: return "n or workers out of range";
    case ECQ_ERR_LEVELS: return "s must be in 1..127";
    case ECQ_ERR_BUCKET: return "bucket must be a positive multiple of 8";
    case ECQ_ERR_STRIDE: return "a row stride is too small or not suitably divisible";
    case ECQ_ERR_ALIGN: return "a base pointer is not aligned as documented";
    case ECQ_ERR_LAUNCH: return "the HIP runtime refused a launch";
    case ECQ_ERR_PARAM: return "alpha, beta, norm or a tuning value is out of range";
    default: return "unknown status";
    }
}

int ecq_version(void) { return 100; }

}  // extern "C"
