"""CPU oracle for the ECQ-SGD hot path -- TEST INFRASTRUCTURE ONLY.

Loads ``ecq_oracle.c`` (plain C, compiled with gcc, contraction off) through ctypes and wraps
it with numpy array marshalling.  Nothing here is part of the product: only ``tests/``, the
smoke check and the benchmark's ``cpu_baseline`` leg may import this package, and it imports
nothing from the HIP library or its binding.

Each wrapper names the passage of Wu et al. (ICML 2018) its C function follows.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "ecq_oracle.c")
_LIB = os.path.join(_DIR, "libecq_oracle.so")

# Every float operation must be rounded on its own: no contraction, no fast-math.
CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
          "-fopenmp", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _declare(_lib)
    return _lib


_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_i8p = np.ctypeslib.ndpointer(np.int8, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_u64p = np.ctypeslib.ndpointer(np.uint64, flags="C_CONTIGUOUS")


def _declare(L):
    L.ecq_oracle_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
    L.ecq_oracle_philox4x32_10.restype = None
    L.ecq_oracle_word.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64]
    L.ecq_oracle_word.restype = C.c_uint32
    L.ecq_oracle_words.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_int64, _u32p]
    L.ecq_oracle_words.restype = None
    L.ecq_oracle_code_bits.argtypes = [C.c_int]
    L.ecq_oracle_code_bits.restype = C.c_int
    L.ecq_oracle_compensate.argtypes = [C.c_float, C.c_float, C.c_float]
    L.ecq_oracle_compensate.restype = C.c_float
    L.ecq_oracle_bucket_scale.argtypes = [_f32p, C.c_int64]
    L.ecq_oracle_bucket_scale.restype = C.c_float
    L.ecq_oracle_bucket_scale_l2.argtypes = [_f32p, C.c_int64]
    L.ecq_oracle_bucket_scale_l2.restype = C.c_float
    L.ecq_oracle_round.argtypes = [C.c_float, C.c_float, C.c_int, C.c_uint32]
    L.ecq_oracle_round.restype = C.c_int
    L.ecq_oracle_dequant.argtypes = [C.c_int, C.c_float, C.c_int]
    L.ecq_oracle_dequant.restype = C.c_float
    L.ecq_oracle_error.argtypes = [C.c_float, C.c_float, C.c_float, C.c_float]
    L.ecq_oracle_error.restype = C.c_float
    L.ecq_oracle_round_words.argtypes = [C.c_float, C.c_float, C.c_int, _u32p, C.c_int64, _i8p]
    L.ecq_oracle_round_words.restype = None
    L.ecq_oracle_row_bytes.argtypes = [C.c_int64, C.c_int]
    L.ecq_oracle_row_bytes.restype = C.c_int64
    L.ecq_oracle_pack.argtypes = [_i8p, C.c_int64, C.c_int, _u8p]
    L.ecq_oracle_pack.restype = None
    L.ecq_oracle_unpack.argtypes = [_u8p, C.c_int64, C.c_int, _i8p]
    L.ecq_oracle_unpack.restype = None
    L.ecq_oracle_bucket_step.argtypes = [_f32p, _f32p, C.c_int64, C.c_uint64, C.c_uint32, C.c_int,
                                         C.c_float, C.c_float, C.c_uint64, C.c_uint64, C.c_int,
                                         _i8p, C.POINTER(C.c_float), C.c_void_p, C.c_int]
    L.ecq_oracle_bucket_step.restype = None
    L.ecq_oracle_pack_rows.argtypes = [_i8p, C.c_int, C.c_int64, C.c_int, _u8p, C.c_int64]
    L.ecq_oracle_pack_rows.restype = None
    L.ecq_oracle_batch_step.argtypes = [_f32p, _f32p, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                        C.c_int, C.c_float, C.c_float, C.c_uint64, C.c_uint64,
                                        C.c_int, _i8p, _f32p, C.c_void_p, C.c_int, C.c_int]
    L.ecq_oracle_batch_step.restype = None
    L.ecq_oracle_max_threads.argtypes = []
    L.ecq_oracle_max_threads.restype = C.c_int
    L.ecq_oracle_error_update_row.argtypes = [_f32p, _u8p, _f32p, C.c_int64, C.c_int, C.c_int,
                                              C.c_float, _f32p]
    L.ecq_oracle_error_update_row.restype = None
    L.ecq_oracle_aggregate.argtypes = [_u8p, C.c_int64, _f32p, C.c_int64, C.c_int, C.c_int64,
                                       C.c_int, C.c_int, _f32p]
    L.ecq_oracle_aggregate.restype = None
    L.ecq_oracle_sgd_step.argtypes = [_f32p, _f32p, C.c_float, C.c_int64]
    L.ecq_oracle_sgd_step.restype = None
    L.ecq_oracle_level_histogram.argtypes = [_i8p, C.c_int64, C.c_int, _u64p]
    L.ecq_oracle_level_histogram.restype = None
    L.ecq_oracle_entropy_bound_bits.argtypes = [_u64p, C.c_int]
    L.ecq_oracle_entropy_bound_bits.restype = C.c_double
    L.ecq_oracle_huffman_lengths.argtypes = [_u64p, C.c_int, _u8p]
    L.ecq_oracle_huffman_lengths.restype = None
    L.ecq_oracle_huffman_codes.argtypes = [_u8p, C.c_int, _u64p]
    L.ecq_oracle_huffman_codes.restype = None
    L.ecq_oracle_huffman_encode.argtypes = [_i8p, C.c_int64, C.c_int, _u8p, _u64p, _u8p, C.c_int64, C.c_int64, _u64p]
    L.ecq_oracle_huffman_encode.restype = C.c_int64
    L.ecq_oracle_huffman_decode.argtypes = [_u8p, C.c_uint64, C.c_int64, C.c_int, _u8p, _u64p, _i8p]
    L.ecq_oracle_huffman_decode.restype = None
    L.ecq_oracle_zrun_max_run.argtypes = [C.c_int]
    L.ecq_oracle_zrun_max_run.restype = C.c_int
    L.ecq_oracle_zrun_symbols.argtypes = [C.c_int]
    L.ecq_oracle_zrun_symbols.restype = C.c_int
    L.ecq_oracle_zrun_tokens.argtypes = [_i8p, C.c_int64, C.c_int, _u8p]
    L.ecq_oracle_zrun_tokens.restype = C.c_int64
    L.ecq_oracle_zrun_histogram.argtypes = [_i8p, C.c_int64, C.c_int, C.c_int64, _u64p]
    L.ecq_oracle_zrun_histogram.restype = None
    L.ecq_oracle_zrun_max_bytes.argtypes = [C.c_int64, C.c_int, C.c_int64]
    L.ecq_oracle_zrun_max_bytes.restype = C.c_int64
    L.ecq_oracle_zrun_encode.argtypes = [_i8p, C.c_int64, C.c_int, _u8p, _u64p, _u8p, C.c_int64, C.c_int64,
                                         C.c_int64, _u32p, _u64p]
    L.ecq_oracle_zrun_encode.restype = C.c_int64
    L.ecq_oracle_zrun_decode.argtypes = [_u8p, C.c_uint64, C.c_int64, C.c_int, _u8p, _u64p, _i8p]
    L.ecq_oracle_zrun_decode.restype = None


# ------------------------------------------------------------------ scalar steps ------------

def philox4x32_10(ctr, key) -> np.ndarray:
    """Philox4x32-10 block (Salmon et al., SC'11) for a 4-word counter and 2-word key."""
    out = np.zeros(4, np.uint32)
    lib().ecq_oracle_philox4x32_10(np.asarray(ctr, np.uint32).copy(), np.asarray(key, np.uint32).copy(), out)
    return out


def word(seed: int, step: int, p: int, i: int) -> int:
    """Random word consumed by element i of worker p at iteration `step`."""
    return int(lib().ecq_oracle_word(seed, step, p, i))


def words(seed: int, step: int, p: int, i0: int, count: int) -> np.ndarray:
    out = np.zeros(count, np.uint32)
    lib().ecq_oracle_words(seed, step, p, i0, count, out)
    return out


def code_bits(s: int) -> int:
    """r = ceil(log2(2s+1)) (Section 4, cost paragraph)."""
    return int(lib().ecq_oracle_code_bits(s))


def row_bytes(n: int, s: int) -> int:
    return int(lib().ecq_oracle_row_bytes(n, s))


def compensate(g: float, alpha: float, h: float) -> np.float32:
    """Eq. (7)."""
    return np.float32(lib().ecq_oracle_compensate(g, alpha, h))


def bucket_scale(v: np.ndarray) -> np.float32:
    v = np.ascontiguousarray(v, np.float32)
    return np.float32(lib().ecq_oracle_bucket_scale(v, v.size))


def bucket_scale_l2(v: np.ndarray) -> np.float32:
    """l_2 norm of a bucket: tree sum of fl(v_i^2) by index, then sqrt."""
    v = np.ascontiguousarray(v, np.float32)
    return np.float32(lib().ecq_oracle_bucket_scale_l2(v, v.size))


def round_level(v: float, scale: float, s: int, w: int) -> int:
    """Eq. (8)-(9): signed level for one element."""
    return int(lib().ecq_oracle_round(v, scale, s, w))


def round_words(v: float, scale: float, s: int, ws: np.ndarray) -> np.ndarray:
    ws = np.ascontiguousarray(ws, np.uint32)
    q = np.zeros(ws.size, np.int8)
    lib().ecq_oracle_round_words(v, scale, s, ws, ws.size, q)
    return q


def dequant(q: int, scale: float, s: int) -> np.float32:
    """Eq. (8): scale * sgn * |q|/s."""
    return np.float32(lib().ecq_oracle_dequant(q, scale, s))


def error(beta: float, h: float, g: float, gt: float) -> np.float32:
    """Eq. (6)."""
    return np.float32(lib().ecq_oracle_error(beta, h, g, gt))


# ------------------------------------------------------------------ encoding ----------------

def pack(q: np.ndarray, s: int) -> np.ndarray:
    q = np.ascontiguousarray(q, np.int8)
    out = np.zeros(row_bytes(q.size, s), np.uint8)
    lib().ecq_oracle_pack(q, q.size, s, out)
    return out


def unpack(codes: np.ndarray, n: int, s: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    assert codes.size >= row_bytes(n, s)
    q = np.zeros(n, np.int8)
    lib().ecq_oracle_unpack(codes, n, s, q)
    return q


# ------------------------------------------------------------------ buckets and batches -----

def _norm_flag(norm) -> int:
    return {"linf": 0, "l2": 1, 0: 0, 1: 1}[norm]


def bucket_step(g, h, i0, p, s, alpha, beta, seed, step, update_h=True, want_gt=True, norm="linf"):
    """One bucket of one worker for one iteration.  Returns (q, scale, gt, h_next)."""
    g = np.ascontiguousarray(g, np.float32)
    h = np.array(h, np.float32, copy=True)
    n = g.size
    q = np.zeros(n, np.int8)
    gt = np.zeros(n, np.float32) if want_gt else None
    sc = C.c_float(0.0)
    lib().ecq_oracle_bucket_step(g, h, n, i0, p, s, alpha, beta, seed, step, int(update_h), q,
                                 C.byref(sc), gt.ctypes.data if want_gt else None, _norm_flag(norm))
    return q, np.float32(sc.value), gt, h


def batch_step(g, h, bucket, s, alpha, beta, seed, step, update_h=True, want_gt=False,
               threads=0, worker0=0, norm="linf"):
    """All workers for one iteration (Alg. 1, first loop).  g, h: [P, N] float32; h is updated
    IN PLACE when update_h.  Row j is worker worker0 + j.  Returns (q [P,N] int8, scales [P,nb]
    float32, gt or None)."""
    assert g.dtype == np.float32 and h.dtype == np.float32
    assert g.ndim == 2 and g.shape == h.shape
    assert g.flags.c_contiguous and h.flags.c_contiguous
    P, n = g.shape
    nb = (n + bucket - 1) // bucket
    q = np.zeros((P, n), np.int8)
    scales = np.zeros((P, nb), np.float32)
    gt = np.zeros((P, n), np.float32) if want_gt else None
    lib().ecq_oracle_batch_step(g, h, n, n, P, worker0, bucket, s, alpha, beta, seed, step,
                                int(update_h), q, scales,
                                gt.ctypes.data if want_gt else None, threads, _norm_flag(norm))
    return q, scales, gt


def pack_rows(q: np.ndarray, s: int) -> np.ndarray:
    """Encode every worker row; returns [P, row_bytes] uint8."""
    q = np.ascontiguousarray(q, np.int8)
    P, n = q.shape
    out = np.zeros((P, row_bytes(n, s)), np.uint8)
    lib().ecq_oracle_pack_rows(q, P, n, s, out, out.shape[1])
    return out


def error_update_row(g, codes, scales, bucket, s, beta, h):
    """Eq. (6) from an encoded message; h (1-D float32) is updated in place."""
    g = np.ascontiguousarray(g, np.float32)
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    assert h.dtype == np.float32 and h.flags.c_contiguous
    lib().ecq_oracle_error_update_row(g, codes, scales, g.size, bucket, s, beta, h)
    return h


def aggregate(codes: np.ndarray, scales: np.ndarray, n: int, bucket: int, s: int) -> np.ndarray:
    """Eq. (4): decode each worker's message and average.  codes [P, >=row_bytes] uint8,
    scales [P, >=nb] float32."""
    codes = np.ascontiguousarray(codes, np.uint8)
    scales = np.ascontiguousarray(scales, np.float32)
    P = codes.shape[0]
    out = np.zeros(n, np.float32)
    lib().ecq_oracle_aggregate(codes, codes.shape[1], scales, scales.shape[1], P, n, bucket, s, out)
    return out


def sgd_step(w: np.ndarray, gavg: np.ndarray, eta: float) -> np.ndarray:
    """Alg. 1, model update: w <- w - eta * g~ (w float32, updated in place)."""
    assert w.dtype == np.float32 and w.flags.c_contiguous
    lib().ecq_oracle_sgd_step(w, np.ascontiguousarray(gavg, np.float32), eta, w.size)
    return w


def level_histogram(q: np.ndarray, s: int) -> np.ndarray:
    """d_k of Section 4's cost paragraph for one worker row: counts over codes 0..2s."""
    q = np.ascontiguousarray(q, np.int8).reshape(-1)
    counts = np.zeros(2 * s + 1, np.uint64)
    lib().ecq_oracle_level_histogram(q, q.size, s, counts)
    return counts


def entropy_bound_bits(counts: np.ndarray) -> float:
    """sum_k d_k log2(d/d_k): the entropy-coded length bound of Section 4."""
    counts = np.ascontiguousarray(counts, np.uint64)
    return float(lib().ecq_oracle_entropy_bound_bits(counts, counts.size))


HUFFMAN_TILE = 1024     # elements per independently decodable tile


def huffman_lengths(counts: np.ndarray) -> np.ndarray:
    """Codeword length of every level from its count (Huffman, 1952; deterministic ties)."""
    counts = np.ascontiguousarray(counts, np.uint64)
    lengths = np.zeros(counts.size, np.uint8)
    lib().ecq_oracle_huffman_lengths(counts, counts.size, lengths)
    return lengths


def huffman_codes(lengths: np.ndarray) -> np.ndarray:
    """Canonical codewords (integers, most significant bit first) from the lengths."""
    lengths = np.ascontiguousarray(lengths, np.uint8)
    codes = np.zeros(lengths.size, np.uint64)
    lib().ecq_oracle_huffman_codes(lengths, lengths.size, codes)
    return codes


def huffman_encode(q: np.ndarray, s: int, lengths: np.ndarray, codes: np.ndarray, tile: int = HUFFMAN_TILE):
    """One worker row -> (stream bytes, tile bit offsets incl. the total, total bits)."""
    q = np.ascontiguousarray(q, np.int8).reshape(-1)
    cap = (row_bytes(q.size, s) + 3) // 4 * 4
    out = np.zeros(max(cap, 4), np.uint8)
    offs = np.zeros((q.size + tile - 1) // tile + 1, np.uint64)
    bits = lib().ecq_oracle_huffman_encode(q, q.size, s, np.ascontiguousarray(lengths, np.uint8),
                                           np.ascontiguousarray(codes, np.uint64), out, out.size, tile, offs)
    return out, offs, int(bits)


def huffman_decode(stream: np.ndarray, start: int, n: int, s: int, lengths: np.ndarray, codes: np.ndarray):
    q = np.zeros(n, np.int8)
    lib().ecq_oracle_huffman_decode(np.ascontiguousarray(stream, np.uint8), start, n, s,
                                    np.ascontiguousarray(lengths, np.uint8),
                                    np.ascontiguousarray(codes, np.uint64), q)
    return q


ZRUN_TILE = 4096        # elements per independently decodable tile of the zero-run code
ZRUN_GROUP = 64         # tiles per group (one 64-bit stream offset per group)


def zrun_max_run(s: int) -> int:
    """Z = floor(127/s): the longest zero run one token completes."""
    return int(lib().ecq_oracle_zrun_max_run(s))


def zrun_symbols(s: int) -> int:
    """Size of the token alphabet, 2sZ + 1."""
    return int(lib().ecq_oracle_zrun_symbols(s))


def zrun_tokens(q: np.ndarray, s: int) -> np.ndarray:
    """Tokens of ONE tile of levels (Section 4, cost paragraph; zero runs joined with the level
    that ends them)."""
    q = np.ascontiguousarray(q, np.int8).reshape(-1)
    out = np.zeros(q.size + 1, np.uint8)
    count = lib().ecq_oracle_zrun_tokens(q, q.size, s, out)
    return out[:count].copy()


def zrun_histogram(q: np.ndarray, s: int, tile: int = ZRUN_TILE) -> np.ndarray:
    """Token counts of one worker row."""
    q = np.ascontiguousarray(q, np.int8).reshape(-1)
    counts = np.zeros(zrun_symbols(s), np.uint64)
    lib().ecq_oracle_zrun_histogram(q, q.size, s, tile, counts)
    return counts


def zrun_max_bytes(n: int, s: int, tile: int = ZRUN_TILE) -> int:
    return int(lib().ecq_oracle_zrun_max_bytes(n, s, tile))


def zrun_encode(q: np.ndarray, s: int, lengths: np.ndarray, codes: np.ndarray, tile: int = ZRUN_TILE,
                group: int = ZRUN_GROUP):
    """One worker row -> (stream bytes, bits of every tile, group bit offsets incl. the total,
    total bits)."""
    q = np.ascontiguousarray(q, np.int8).reshape(-1)
    tiles = (q.size + tile - 1) // tile
    out = np.zeros(max(zrun_max_bytes(q.size, s, tile), 4), np.uint8)
    tile_bits = np.zeros(max(tiles, 1), np.uint32)
    group_offsets = np.zeros((tiles + group - 1) // group + 1, np.uint64)
    bits = lib().ecq_oracle_zrun_encode(q, q.size, s, np.ascontiguousarray(lengths, np.uint8),
                                        np.ascontiguousarray(codes, np.uint64), out, out.size, tile, group,
                                        tile_bits, group_offsets)
    return out, tile_bits[:tiles], group_offsets, int(bits)


def zrun_decode(stream: np.ndarray, start: int, n: int, s: int, lengths: np.ndarray, codes: np.ndarray):
    """One tile of n levels from the stream bit `start`."""
    q = np.full(n, -128, np.int8)
    lib().ecq_oracle_zrun_decode(np.ascontiguousarray(stream, np.uint8), start, n, s,
                                 np.ascontiguousarray(lengths, np.uint8),
                                 np.ascontiguousarray(codes, np.uint64), q)
    return q


def max_threads() -> int:
    return int(lib().ecq_oracle_max_threads())
