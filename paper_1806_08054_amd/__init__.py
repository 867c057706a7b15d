"""ECQ-SGD hot path for AMD MI355X: a thin binding over the C-ABI library ``libecq.so``.

Every step of the path runs in the library's HIP kernels; this package only marshals
arguments.  There is no CPU fallback: importing fails loudly if the library is missing.
"""
from .binding import (  # noqa: F401
    EcqError,
    Shape,
    Tuning,
    code_bits,
    ecq_calib_add,
    ecq_calib_copy,
    ecq_calib_gather,
    ecq_check_division,
    ecq_dequant_aggregate,
    ecq_dequant_aggregate_sgd,
    ecq_entropy_bound_bits,
    ecq_error_update,
    ecq_huffman_build,
    ecq_huffman_decode,
    ecq_huffman_encode,
    huffman_num_tiles,
    ecq_level_histogram,
    ecq_philox_words,
    ecq_quantize,
    ecq_quantize_update,
    ecq_quantize_update_ex,
    lib,
    library_path,
    num_buckets,
    row_bytes,
    status_string,
)
