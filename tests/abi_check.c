/* A C99 program against include/ecq.h: the header has to compile as plain C, and the host-side
 * helpers of the library must be callable from C.  No kernel is launched.
 * Prints one line per call; tests/test_abi.py compares the output. */
#include <inttypes.h>
#include <stdio.h>

#include "ecq.h"

int main(void)
{
    int64_t bytes = 0, nb = 0, tiles = 0, groups = 0, zbytes = 0;
    int max_run = 0, symbols = 0, st;
    ecq_shape sh;
    sh.n = 25557032;
    sh.workers = 8;
    sh.bucket = 512;
    sh.s = 1;
    sh.norm = ECQ_NORM_LINF;
    sh.gh_stride = 25557032;
    sh.scale_stride = 49917;
    printf("code_bits %d %d %d\n", ecq_code_bits(1), ecq_code_bits(4), ecq_code_bits(127));
    st = ecq_row_bytes(sh.n, sh.s, &bytes);
    printf("row_bytes %d %" PRId64 "\n", st, bytes);
    sh.code_stride = (bytes + 3) / 4 * 4;
    st = ecq_num_buckets(sh.n, sh.bucket, &nb);
    printf("num_buckets %d %" PRId64 "\n", st, nb);
    printf("check_shape %d\n", ecq_check_shape(&sh));
    sh.bucket = 12;
    printf("check_shape_bad_bucket %d\n", ecq_check_shape(&sh) == ECQ_ERR_BUCKET);
    st = ecq_zrun_symbols(4, &max_run, &symbols);
    printf("zrun_symbols %d %d %d\n", st, max_run, symbols);
    st = ecq_zrun_num_tiles(sh.n, &tiles, &groups);
    printf("zrun_num_tiles %d %" PRId64 " %" PRId64 "\n", st, tiles, groups);
    st = ecq_zrun_stream_bytes(sh.n, 1, &zbytes);
    printf("zrun_stream_bytes %d %" PRId64 "\n", st, zbytes);
    printf("null_pointer %d\n", ecq_dequant_aggregate(&sh, NULL, NULL, NULL, NULL) < 0);
    printf("status_string %s\n", ecq_status_string(ECQ_ERR_BUCKET)[0] ? "text" : "empty");
    return 0;
}
