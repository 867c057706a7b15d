"""ctypes binding of include/ecq.h: same names, argument marshalling only.

Tensors are torch tensors on the GPU (torch is used for device memory and streams, nothing
else); each wrapper passes raw device pointers and the current HIP stream to the library.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG_DIR, "libecq.so")


class EcqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Shape(C.Structure):
    """Mirror of ecq_shape."""
    _fields_ = [("n", C.c_int64), ("workers", C.c_int32), ("bucket", C.c_int32), ("s", C.c_int32),
                ("norm", C.c_int32), ("gh_stride", C.c_int64), ("code_stride", C.c_int64),
                ("scale_stride", C.c_int64)]

    @classmethod
    def packed(cls, n: int, workers: int, bucket: int, s: int, norm: int = 0) -> "Shape":
        """Tightest legal strides: gh rounded up to 4 floats, codes to 4 bytes.
        norm: 0 = l_inf (ECQ_NORM_LINF), 1 = l_2 (ECQ_NORM_L2)."""
        return cls(n=n, workers=workers, bucket=bucket, s=s, norm=norm,
                   gh_stride=(n + 3) // 4 * 4, code_stride=(row_bytes(n, s) + 3) // 4 * 4,
                   scale_stride=num_buckets(n, bucket))

    @classmethod
    def aligned(cls, n: int, workers: int, bucket: int, s: int, norm: int = 0, line: int = 128) -> "Shape":
        """Strides rounded up so that every worker row of g, h, codes and scales starts on a
        `line`-byte boundary (128 = one cache line) when the base pointers do.  A wave's 1 KiB
        loads then cover whole lines; on MI355X this alone is worth 4-5 % of bandwidth."""
        up = lambda x, m: (x + m - 1) // m * m
        return cls(n=n, workers=workers, bucket=bucket, s=s, norm=norm,
                   gh_stride=up(n, line // 4), code_stride=up(row_bytes(n, s), line),
                   scale_stride=up(num_buckets(n, bucket), line // 4))


class Tuning(C.Structure):
    """Mirror of ecq_tuning."""
    _fields_ = [("path", C.c_int32), ("waves_per_bucket", C.c_int32), ("block_threads", C.c_int32),
                ("block_order", C.c_int32)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(
                f"{_LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(_LIB_PATH)
        vp, f, u64, i64 = C.c_void_p, C.c_float, C.c_uint64, C.c_int64
        shp = C.POINTER(Shape)
        L.ecq_code_bits.argtypes = [C.c_int]
        L.ecq_row_bytes.argtypes = [i64, C.c_int, C.POINTER(i64)]
        L.ecq_num_buckets.argtypes = [i64, C.c_int, C.POINTER(i64)]
        L.ecq_check_shape.argtypes = [shp]
        L.ecq_quantize.argtypes = [shp, vp, vp, f, u64, u64, vp, vp, vp]
        L.ecq_error_update.argtypes = [shp, vp, vp, vp, f, vp, vp]
        L.ecq_quantize_update.argtypes = [shp, vp, vp, f, f, u64, u64, vp, vp, vp]
        L.ecq_quantize_update_ex.argtypes = [shp, vp, vp, f, f, u64, u64, vp, vp, C.POINTER(Tuning), vp]
        L.ecq_dequant_aggregate.argtypes = [shp, vp, vp, vp, vp]
        L.ecq_dequant_aggregate_sgd.argtypes = [shp, vp, vp, f, vp, vp, vp]
        L.ecq_level_histogram.argtypes = [shp, vp, vp, i64, vp]
        L.ecq_entropy_bound_bits.argtypes = [C.POINTER(C.c_uint64), C.c_int, C.POINTER(C.c_double)]
        L.ecq_check_division.argtypes = [C.c_int, C.c_uint32, vp, vp]
        L.ecq_huffman_num_tiles.argtypes = [i64, C.POINTER(i64)]
        L.ecq_huffman_build.argtypes = [C.c_int, C.c_int, vp, i64, vp, vp, vp]
        L.ecq_huffman_encode.argtypes = [shp, vp, vp, vp, i64, vp, i64, vp, i64, vp]
        L.ecq_huffman_decode.argtypes = [shp, vp, i64, vp, i64, vp, vp, i64, vp, vp]
        L.ecq_zrun_symbols.argtypes = [C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.ecq_zrun_num_tiles.argtypes = [i64, C.POINTER(i64), C.POINTER(i64)]
        L.ecq_zrun_stream_bytes.argtypes = [i64, C.c_int, C.POINTER(i64)]
        L.ecq_zrun_histogram.argtypes = [shp, vp, vp, i64, vp]
        L.ecq_zrun_build.argtypes = [C.c_int, C.c_int, vp, i64, vp, vp, vp]
        L.ecq_zrun_encode.argtypes = [shp, vp, vp, vp, i64, vp, i64, vp, i64, vp, i64, vp]
        L.ecq_zrun_decode.argtypes = [shp, vp, i64, vp, i64, vp, i64, vp, vp, i64, vp, vp]
        L.ecq_philox_words.argtypes = [u64, u64, C.c_uint32, u64, i64, vp, vp]
        L.ecq_calib_add.argtypes = [vp, vp, vp, i64, vp]
        L.ecq_calib_copy.argtypes = [vp, vp, i64, vp]
        L.ecq_calib_gather.argtypes = [shp, vp, vp, vp]
        L.ecq_status_string.argtypes = [C.c_int]
        L.ecq_status_string.restype = C.c_char_p
        L.ecq_version.argtypes = []
        for name in ("ecq_code_bits", "ecq_row_bytes", "ecq_num_buckets", "ecq_check_shape", "ecq_quantize",
                     "ecq_error_update", "ecq_quantize_update", "ecq_quantize_update_ex",
                     "ecq_dequant_aggregate", "ecq_dequant_aggregate_sgd", "ecq_level_histogram", "ecq_entropy_bound_bits", "ecq_check_division",
                     "ecq_philox_words", "ecq_calib_add", "ecq_calib_copy", "ecq_calib_gather", "ecq_huffman_num_tiles",
                     "ecq_huffman_build", "ecq_huffman_encode", "ecq_huffman_decode",
                     "ecq_zrun_symbols", "ecq_zrun_num_tiles", "ecq_zrun_stream_bytes", "ecq_zrun_histogram",
                     "ecq_zrun_build", "ecq_zrun_encode", "ecq_zrun_decode",
                     "ecq_version"):
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ecq_status_string(status).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise EcqError(status, where)


def code_bits(s: int) -> int:
    r = lib().ecq_code_bits(s)
    if r < 0:
        raise EcqError(r, "ecq_code_bits")
    return r


def row_bytes(n: int, s: int) -> int:
    out = C.c_int64(0)
    _check(lib().ecq_row_bytes(n, s, C.byref(out)), "ecq_row_bytes")
    return out.value


def num_buckets(n: int, bucket: int) -> int:
    out = C.c_int64(0)
    _check(lib().ecq_num_buckets(n, bucket, C.byref(out)), "ecq_num_buckets")
    return out.value


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is not None:
        return C.c_void_p(stream)
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def ecq_quantize(shape: Shape, g, h, alpha: float, seed: int, step: int, codes, scales, stream=None) -> None:
    _check(lib().ecq_quantize(C.byref(shape), _ptr(g), _ptr(h), alpha, seed, step, _ptr(codes), _ptr(scales),
                              _stream(stream)), "ecq_quantize")


def ecq_error_update(shape: Shape, g, codes, scales, beta: float, h, stream=None) -> None:
    _check(lib().ecq_error_update(C.byref(shape), _ptr(g), _ptr(codes), _ptr(scales), beta, _ptr(h),
                                  _stream(stream)), "ecq_error_update")


def ecq_quantize_update(shape: Shape, g, h, alpha: float, beta: float, seed: int, step: int, codes, scales,
                        stream=None) -> None:
    _check(lib().ecq_quantize_update(C.byref(shape), _ptr(g), _ptr(h), alpha, beta, seed, step, _ptr(codes),
                                     _ptr(scales), _stream(stream)), "ecq_quantize_update")


def ecq_quantize_update_ex(shape: Shape, g, h, alpha: float, beta: float, seed: int, step: int, codes, scales,
                           tuning: Tuning | None = None, stream=None) -> None:
    _check(lib().ecq_quantize_update_ex(C.byref(shape), _ptr(g), _ptr(h), alpha, beta, seed, step, _ptr(codes),
                                        _ptr(scales), C.byref(tuning) if tuning is not None else None,
                                        _stream(stream)), "ecq_quantize_update_ex")


def ecq_dequant_aggregate(shape: Shape, codes, scales, out, stream=None) -> None:
    _check(lib().ecq_dequant_aggregate(C.byref(shape), _ptr(codes), _ptr(scales), _ptr(out), _stream(stream)),
           "ecq_dequant_aggregate")


def ecq_dequant_aggregate_sgd(shape: Shape, codes, scales, eta: float, w, out=None, stream=None) -> None:
    _check(lib().ecq_dequant_aggregate_sgd(C.byref(shape), _ptr(codes), _ptr(scales), eta, _ptr(w), _ptr(out),
                                           _stream(stream)), "ecq_dequant_aggregate_sgd")


def ecq_level_histogram(shape: Shape, codes, counts, count_stride: int, stream=None) -> None:
    _check(lib().ecq_level_histogram(C.byref(shape), _ptr(codes), _ptr(counts), count_stride, _stream(stream)),
           "ecq_level_histogram")


def ecq_entropy_bound_bits(counts_host) -> float:
    """counts_host: a sequence of the 2s+1 counters of one worker row, on the host."""
    arr = (C.c_uint64 * len(counts_host))(*[int(c) for c in counts_host])
    bits = C.c_double(0.0)
    _check(lib().ecq_entropy_bound_bits(arr, len(counts_host), C.byref(bits)), "ecq_entropy_bound_bits")
    return bits.value


HUFFMAN_TILE = 1024     # ECQ_HUFFMAN_TILE


def huffman_num_tiles(n: int) -> int:
    out = C.c_int64(0)
    _check(lib().ecq_huffman_num_tiles(n, C.byref(out)), "ecq_huffman_num_tiles")
    return out.value


def ecq_huffman_build(workers: int, s: int, counts, table_stride: int, lengths, codewords, stream=None) -> None:
    _check(lib().ecq_huffman_build(workers, s, _ptr(counts), table_stride, _ptr(lengths), _ptr(codewords),
                                   _stream(stream)), "ecq_huffman_build")


def ecq_huffman_encode(shape: Shape, codes, lengths, codewords, table_stride: int, streams, stream_stride: int,
                       tile_offsets, offset_stride: int, stream=None) -> None:
    _check(lib().ecq_huffman_encode(C.byref(shape), _ptr(codes), _ptr(lengths), _ptr(codewords), table_stride,
                                    _ptr(streams), stream_stride, _ptr(tile_offsets), offset_stride,
                                    _stream(stream)), "ecq_huffman_encode")


def ecq_huffman_decode(shape: Shape, streams, stream_stride: int, tile_offsets, offset_stride: int, lengths,
                       codewords, table_stride: int, codes, stream=None) -> None:
    _check(lib().ecq_huffman_decode(C.byref(shape), _ptr(streams), stream_stride, _ptr(tile_offsets),
                                    offset_stride, _ptr(lengths), _ptr(codewords), table_stride, _ptr(codes),
                                    _stream(stream)), "ecq_huffman_decode")


ZRUN_TILE = 4096        # ECQ_ZRUN_TILE
ZRUN_GROUP = 64         # ECQ_ZRUN_GROUP


def zrun_symbols(s: int) -> tuple[int, int]:
    """(Z, number of tokens) of the zero-run code for s levels."""
    z, a = C.c_int(0), C.c_int(0)
    _check(lib().ecq_zrun_symbols(s, C.byref(z), C.byref(a)), "ecq_zrun_symbols")
    return z.value, a.value


def zrun_num_tiles(n: int) -> tuple[int, int]:
    """(tiles, groups) of a row of n elements."""
    t, g = C.c_int64(0), C.c_int64(0)
    _check(lib().ecq_zrun_num_tiles(n, C.byref(t), C.byref(g)), "ecq_zrun_num_tiles")
    return t.value, g.value


def zrun_stream_bytes(n: int, s: int) -> int:
    out = C.c_int64(0)
    _check(lib().ecq_zrun_stream_bytes(n, s, C.byref(out)), "ecq_zrun_stream_bytes")
    return out.value


def ecq_zrun_histogram(shape: Shape, codes, counts, count_stride: int, stream=None) -> None:
    _check(lib().ecq_zrun_histogram(C.byref(shape), _ptr(codes), _ptr(counts), count_stride, _stream(stream)),
           "ecq_zrun_histogram")


def ecq_zrun_build(workers: int, s: int, counts, table_stride: int, lengths, codewords, stream=None) -> None:
    _check(lib().ecq_zrun_build(workers, s, _ptr(counts), table_stride, _ptr(lengths), _ptr(codewords),
                                _stream(stream)), "ecq_zrun_build")


def ecq_zrun_encode(shape: Shape, codes, lengths, codewords, table_stride: int, streams, stream_stride: int,
                    tile_bits, tile_stride: int, group_offsets, group_stride: int, stream=None) -> None:
    _check(lib().ecq_zrun_encode(C.byref(shape), _ptr(codes), _ptr(lengths), _ptr(codewords), table_stride,
                                 _ptr(streams), stream_stride, _ptr(tile_bits), tile_stride, _ptr(group_offsets),
                                 group_stride, _stream(stream)), "ecq_zrun_encode")


def ecq_zrun_decode(shape: Shape, streams, stream_stride: int, tile_bits, tile_stride: int, group_offsets,
                    group_stride: int, lengths, codewords, table_stride: int, codes, stream=None) -> None:
    _check(lib().ecq_zrun_decode(C.byref(shape), _ptr(streams), stream_stride, _ptr(tile_bits), tile_stride,
                                 _ptr(group_offsets), group_stride, _ptr(lengths), _ptr(codewords), table_stride,
                                 _ptr(codes), _stream(stream)), "ecq_zrun_decode")


def ecq_check_division(per_divisor: int, salt: int, mismatches, stream=None) -> None:
    _check(lib().ecq_check_division(per_divisor, salt, _ptr(mismatches), _stream(stream)), "ecq_check_division")


def ecq_philox_words(seed: int, step: int, p: int, i0: int, count: int, words, stream=None) -> None:
    _check(lib().ecq_philox_words(seed, step, p, i0, count, _ptr(words), _stream(stream)), "ecq_philox_words")


def ecq_calib_add(a, b, out, n: int, stream=None) -> None:
    _check(lib().ecq_calib_add(_ptr(a), _ptr(b), _ptr(out), n, _stream(stream)), "ecq_calib_add")


def ecq_calib_copy(a, out, n: int, stream=None) -> None:
    _check(lib().ecq_calib_copy(_ptr(a), _ptr(out), n, _stream(stream)), "ecq_calib_copy")


def ecq_calib_gather(shape: Shape, codes, out, stream=None) -> None:
    _check(lib().ecq_calib_gather(C.byref(shape), _ptr(codes), _ptr(out), _stream(stream)), "ecq_calib_gather")
