"""Exact-rational re-derivation of the quantiser, used only to pin the C oracle.

Everything here is pure Python: integers and ``fractions.Fraction``.  A binary32 operation is
modelled as the exact rational result followed by one round-to-nearest-even to the binary32
grid (denormals included), so an extra fused multiply-add, a double rounding or a flushed
denormal in the C oracle shows up as a mismatch.  Nothing here is imported by the oracle or by
the HIP path.

Citations are to Wu et al., "Error Compensated Quantized SGD ..." (ICML 2018), Section 4.
"""
from __future__ import annotations

import math
import struct
from fractions import Fraction

# ---------------------------------------------------------------- binary32 model ------------

_EMIN = -126          # smallest normal exponent
_P = 24               # significand bits


def f32_to_fraction(x) -> Fraction:
    """Exact value of a Python float that is already a binary32 value."""
    return Fraction(float(x))


def rn32(q: Fraction) -> Fraction:
    """Round an exact rational to the nearest binary32 value, ties to even."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, _EMIN)
    ulp = Fraction(2) ** (e - (_P - 1))
    n = a / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (lo & 1)):
        lo += 1
    r = lo * ulp
    assert r < Fraction(2) ** 128, "overflow not modelled"
    return sign * r


def bits_to_f32(u: int) -> float:
    return struct.unpack("<f", struct.pack("<I", u & 0xFFFFFFFF))[0]


def f32_bits(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0]


# ---------------------------------------------------------------- Philox4x32-10 -------------

_M0, _M1 = 0xD2511F53, 0xCD9E8D57
_W0, _W1 = 0x9E3779B9, 0xBB67AE85
_MASK = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    """Salmon et al. (SC'11), written with Python big integers."""
    c = list(ctr)
    k = list(key)
    for _ in range(10):
        p0 = _M0 * c[0]
        p1 = _M1 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & _MASK, (p0 >> 32) ^ c[3] ^ k[1], p0 & _MASK]
        k = [(k[0] + _W0) & _MASK, (k[1] + _W1) & _MASK]
    return c


def word(seed: int, step: int, p: int, i: int) -> int:
    ctr = [(i >> 2) & _MASK, p, step & _MASK, (step >> 32) & _MASK]
    key = [seed & _MASK, (seed >> 32) & _MASK]
    return philox4x32_10(ctr, key)[i & 3]


# ---------------------------------------------------------------- the quantiser -------------

def code_bits(s: int) -> int:
    """Smallest r with 2^r >= 2s+1, i.e. ceil(log2(2s+1))."""
    r = 0
    while (1 << r) < 2 * s + 1:
        r += 1
    return r


def rn32_sqrt(q: Fraction) -> Fraction:
    """Correctly rounded binary32 square root of an exact non-negative rational."""
    if q == 0:
        return Fraction(0)
    # scale by 4^k so that the integer square root carries well over 24 bits
    k = 0
    while q * Fraction(4) ** k < (1 << 60):
        k += 1
    while q * Fraction(4) ** k >= (1 << 64):
        k -= 1
    scaled = q * Fraction(4) ** k                  # sqrt(q) = sqrt(scaled) / 2^k
    n = scaled.numerator // scaled.denominator
    r = math.isqrt(n)                              # floor(sqrt(floor(scaled))) = floor(sqrt(scaled))
    # candidates on the binary32 grid around r / 2^k: round r to 24 significant bits both ways
    shift = r.bit_length() - _P
    lo = (r >> shift) << shift
    hi = lo + (1 << shift)
    mid = lo + (1 << (shift - 1))
    # compare sqrt(scaled) with mid exactly: scaled vs mid^2
    if scaled > mid * mid or (scaled == mid * mid and ((lo >> shift) & 1)):
        pick = hi
    else:
        pick = lo
    out = Fraction(pick) / Fraction(2) ** k
    assert rn32(out) == out, "result must be a binary32 value (no denormal results modelled)"
    return out


def tree_sum_squares(v, lo, width):
    """Balanced binary tree by index; one rounding per square and per addition."""
    if lo >= len(v):
        return Fraction(0)
    if width == 1:
        return rn32(v[lo] * v[lo])
    return rn32(tree_sum_squares(v, lo, width // 2) + tree_sum_squares(v, lo + width // 2, width // 2))


def norm_l2(v):
    width = 1
    while width < len(v):
        width *= 2
    return rn32_sqrt(tree_sum_squares(v, 0, width))


def bucket_step(g, h, i0, p, s, alpha, beta, seed, step, norm="linf"):
    """One bucket, exact rationals with one rounding per binary32 operation.

    g, h: lists of Python floats holding binary32 values; alpha, beta binary32 values.
    Returns (levels, scale, gt, h_next) with scale/gt/h_next as Fractions."""
    G = [f32_to_fraction(x) for x in g]
    H = [f32_to_fraction(x) for x in h]
    A, B = f32_to_fraction(alpha), f32_to_fraction(beta)
    # Eq. (7)
    v = [rn32(gi + rn32(A * hi)) for gi, hi in zip(G, H)]
    neg = []
    for gi, hi, vi in zip(g, h, v):
        neg.append(vi < 0)
    scale = max((abs(x) for x in v), default=Fraction(0)) if norm == "linf" else norm_l2(v)
    q, gt, hn = [], [], []
    for j, (gi, hi, vi) in enumerate(zip(G, H, v)):
        if scale == 0:
            m = 0
        else:
            a = rn32(abs(vi) / scale)                  # |v_i| / ||v||
            x = rn32(a * s)                            # s |v_i| / ||v||
            l = x.numerator // x.denominator           # floor
            frac = x - l                               # probability of rounding up, Eq. (9)
            u = Fraction(word(seed, step, p, i0 + j) >> 8, 1 << 24)
            m = min(s, l + (1 if u < frac else 0))
        qi = -m if neg[j] else m
        xi = rn32(Fraction(m, s))                      # Eq. (8): xi in {0, 1/s, ..., 1}
        gti = rn32(scale * xi)
        if qi < 0:
            gti = -gti
        q.append(qi)
        gt.append(gti)
        hn.append(rn32(rn32(B * hi) + rn32(gi - gti)))  # Eq. (6)
    return q, scale, gt, hn


def pack(levels, s: int) -> bytes:
    """LSB-first contiguous bit stream == one little-endian big integer."""
    r = code_bits(s)
    big = 0
    for i, q in enumerate(levels):
        big |= (q + s) << (i * r)
    nbytes = (len(levels) * r + 7) // 8
    return big.to_bytes(nbytes, "little")


def unpack(data: bytes, n: int, s: int):
    r = code_bits(s)
    big = int.from_bytes(data, "little")
    return [((big >> (i * r)) & ((1 << r) - 1)) - s for i in range(n)]


# ---------------------------------------------------------------- Huffman coding ------------

def huffman_lengths(counts):
    """Merge the two live nodes first in (weight, number) order; new nodes take the next
    number; a level's length is its depth (a lone occupied level gets length 1)."""
    bins = len(counts)
    live = {c: counts[c] for c in range(bins) if counts[c] > 0}
    lengths = [0] * bins
    if len(live) == 1:
        lengths[next(iter(live))] = 1
        return lengths
    members = {c: [c] for c in live}
    nxt = bins
    while len(live) > 1:
        a = min(live, key=lambda i: (live[i], i)); wa = live.pop(a)
        b = min(live, key=lambda i: (live[i], i)); wb = live.pop(b)
        for leaf in members[a] + members[b]:
            lengths[leaf] += 1
        live[nxt] = wa + wb
        members[nxt] = members.pop(a) + members.pop(b)
        nxt += 1
    return lengths


def huffman_codes(lengths):
    order = sorted((l, c) for c, l in enumerate(lengths) if l > 0)
    codes = [0] * len(lengths)
    code, prev = 0, None
    for l, c in order:
        if prev is not None:
            code = (code + 1) << (l - prev)
        codes[c] = code
        prev = l
    return codes


def huffman_encode(levels, s, lengths, codes):
    """Bit stream as one little-endian big integer; a codeword goes in first-bit-first."""
    big, pos = 0, 0
    for q in levels:
        c = q + s
        for b in range(lengths[c] - 1, -1, -1):
            big |= ((codes[c] >> b) & 1) << pos
            pos += 1
    return big, pos
