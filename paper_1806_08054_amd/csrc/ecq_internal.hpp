// Host-side declarations shared by the C ABI layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ecq.h"

namespace ecq {

// Everything a kernel needs, passed by value.
struct Args {
    const float *g;
    float *h;              // read-only unless the kernel updates the accumulator
    uint8_t *codes;
    float *scales;
    float *out;            // aggregation output (may be null when w is given)
    float *w;              // model replica updated by the aggregation kernel, or null
    int64_t n;
    int64_t nb;
    int64_t gh_stride;
    int64_t code_stride;
    int64_t scale_stride;
    int64_t row_bytes;
    int32_t workers;
    int32_t bucket;
    int32_t s;
    int32_t r;
    int32_t norm_l2;       // 1: l2 scaling, 0: l_inf
    float alpha;
    float beta;
    float eta;
    uint32_t key0, key1;   // seed
    uint32_t step_lo, step_hi;
};

// Resolved launch plan for the quantise(+update) entry points.
struct Plan {
    int path;              // 1 = bucket in registers, 2 = two-pass
    int lanes_per_bucket;  // path 1, bucket < 256: lanes sharing a bucket (bucket / 4)
    int waves_per_bucket;  // path 1, bucket >= 256
    int vec_per_lane;      // path 1: float4 per lane (1, 2, 4, 8)
    int block_threads;
    int rows_per_launch;   // path 1, bucket >= 256: worker rows per kernel launch (0 = all)
    int xcd_striped;       // path 1, bucket >= 256: one contiguous region of blocks per XCD
};

int make_plan(const ecq_shape &shape, const ecq_tuning *tuning, Plan *plan);

hipError_t launch_quantize(const Args &a, const Plan &plan, bool update_h, hipStream_t stream);
hipError_t launch_error_update(const Args &a, hipStream_t stream);
hipError_t launch_dequant_aggregate(const Args &a, hipStream_t stream);
hipError_t launch_level_histogram(const Args &a, unsigned long long *counts, int64_t count_stride,
                                  hipStream_t stream);
hipError_t launch_huffman_build(int workers, int bins, const unsigned long long *counts, int64_t table_stride,
                                uint8_t *lengths, unsigned long long *codewords, hipStream_t stream);
// a.codes = the fixed-length message (read by encode, written by decode).
hipError_t launch_huffman_encode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                                 int64_t table_stride, uint32_t *streams, int64_t stream_stride_words,
                                 unsigned long long *tile_offsets, int64_t offset_stride, hipStream_t stream);
hipError_t launch_huffman_decode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                                 int64_t table_stride, const uint32_t *streams, int64_t stream_stride_words,
                                 const unsigned long long *tile_offsets, int64_t offset_stride, hipStream_t stream);
// Zero-run Huffman coder (ecq_zrun.hip).  a.codes = the fixed-length message.
hipError_t launch_zrun_histogram(const Args &a, unsigned long long *counts, int64_t count_stride, hipStream_t stream);
hipError_t launch_zrun_encode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                              int64_t table_stride, uint32_t *streams, int64_t stream_stride_words,
                              uint32_t *tile_bits, int64_t tile_stride, unsigned long long *group_offsets,
                              int64_t group_stride, hipStream_t stream);
hipError_t launch_zrun_decode(const Args &a, const uint8_t *lengths, const unsigned long long *codewords,
                              int64_t table_stride, const uint32_t *streams, int64_t stream_stride_words,
                              const uint32_t *tile_bits, int64_t tile_stride, const unsigned long long *group_offsets,
                              int64_t group_stride, hipStream_t stream);
hipError_t launch_check_division(int per_divisor, uint32_t salt, unsigned long long *mismatches,
                                 hipStream_t stream);
hipError_t launch_philox_words(uint32_t key0, uint32_t key1, uint32_t step_lo, uint32_t step_hi,
                               uint32_t p, uint64_t i0, int64_t count, uint32_t *words,
                               hipStream_t stream);
hipError_t launch_calib_add(const float *a, const float *b, float *out, int64_t n,
                            hipStream_t stream);
hipError_t launch_calib_copy(const float *a, float *out, int64_t n, hipStream_t stream);
hipError_t launch_calib_gather(const Args &a, hipStream_t stream);

static inline unsigned cdiv(int64_t a, int64_t b) { return (unsigned)((a + b - 1) / b); }

}  // namespace ecq

// Runs CALL(R) with the code width as a compile-time constant.
#define ECQ_DISPATCH_R(r, CALL)      \
    switch (r) {                     \
    case 2: CALL(2); break;          \
    case 3: CALL(3); break;          \
    case 4: CALL(4); break;          \
    case 5: CALL(5); break;          \
    case 6: CALL(6); break;          \
    case 7: CALL(7); break;          \
    default: CALL(8); break;         \
    }

