"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without the HIP path.

Citations: Wu et al., "Error Compensated Quantized SGD ..." (ICML 2018).  Each test names the
passage that fixes the property it checks.  A plausible slip in the oracle (a dropped term, a
wrong sign or index, g and v swapped, a fused operation) fails at least one of these.
"""
import math
import os
import random
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests.conftest import read_table
from tests import exact_ref as X

F32 = np.float32


def f32(x):
    return float(F32(x))


# ------------------------------------------------------------------ Philox -----------------

def test_philox_known_answers(golden_dir):
    """Published known answers of Philox4x32-10 (Salmon et al., SC'11)."""
    rows = read_table(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
    assert len(rows) == 3
    for row in rows:
        vals = [int(t, 16) for t in row if t != "->"]
        ctr, key, want = vals[:4], vals[4:6], vals[6:]
        assert list(oracle.philox4x32_10(ctr, key)) == want
        assert X.philox4x32_10(ctr, key) == want


def test_philox_two_implementations_agree():
    rng = random.Random(5)
    for _ in range(200):
        ctr = [rng.getrandbits(32) for _ in range(4)]
        key = [rng.getrandbits(32) for _ in range(2)]
        assert list(oracle.philox4x32_10(ctr, key)) == X.philox4x32_10(ctr, key)


def test_word_indexing():
    """Element i uses lane i&3 of the block whose counter is (i>>2, p, step_lo, step_hi)."""
    seed, step, p = 0x0123456789ABCDEF, (7 << 32) | 9, 5
    for i in (0, 1, 2, 3, 4, 7, 1023, (1 << 33) + 6):
        blk = oracle.philox4x32_10([(i >> 2) & 0xFFFFFFFF, p, 9, 7], [0x89ABCDEF, 0x01234567])
        assert oracle.word(seed, step, p, i) == int(blk[i & 3]) == X.word(seed, step, p, i)
    ws = oracle.words(seed, step, p, 40, 24)
    assert [int(w) for w in ws] == [X.word(seed, step, p, 40 + j) for j in range(24)]
    # distinct (p, step, i>>2) give distinct counters, hence (almost surely) distinct streams
    a = oracle.words(1, 0, 0, 0, 64)
    assert not np.array_equal(a, oracle.words(1, 1, 0, 0, 64))
    assert not np.array_equal(a, oracle.words(1, 0, 1, 0, 64))
    assert not np.array_equal(a, oracle.words(2, 0, 0, 0, 64))
    assert np.array_equal(a[8:], oracle.words(1, 0, 0, 8, 56))


def test_philox_uniformity():
    """Top-24-bit uniforms: mean 1/2 and variance 1/12 within a few standard errors."""
    w = oracle.words(3, 11, 2, 0, 1 << 18)
    u = (w >> 8).astype(np.float64) * 2.0 ** -24
    n = u.size
    assert abs(u.mean() - 0.5) < 5 * math.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 5 * math.sqrt(1 / 180 / n)
    # every bit of the word is balanced
    for b in range(32):
        frac = ((w >> b) & 1).mean()
        assert abs(frac - 0.5) < 5 * 0.5 / math.sqrt(n)


# ------------------------------------------------------------------ code width -------------

def test_code_bits_and_message_size(golden_dir):
    """r = ceil(log2(2s+1)); message = 32 + d*r bits (Section 4, cost paragraph)."""
    for s, r, d, bits in read_table(os.path.join(golden_dir, "code_bits.txt")):
        s, r, d, bits = int(s), int(r), int(d), int(bits)
        assert oracle.code_bits(s) == r == X.code_bits(s)
        assert oracle.row_bytes(d, s) * 8 - (-(d * r) % 8) + 32 == bits
    for s in range(1, 128):
        r = oracle.code_bits(s)
        assert (1 << r) >= 2 * s + 1 > (1 << (r - 1))
        assert r == math.ceil(math.log2(2 * s + 1))
    assert oracle.code_bits(0) < 0


# ------------------------------------------------------------------ rounding rule ----------

@pytest.mark.parametrize("s,num,den", [(1, 321, 1024), (2, 777, 1024), (4, 5, 8), (4, 1023, 1024),
                                       (3, 100, 1024), (7, 300, 1024), (1, 1, 1 << 20)])
def test_round_exhaustive_unbiased(s, num, den):
    """Eq. (9): the level rounds up with probability s|v|/||v|| - l.  Every one of the 2^24
    outcomes of the uniform is enumerated; with scale 1 and v a dyadic rational the
    probability is a multiple of 2^-24, so the count is exact and E[g~] = v (Lemma 1,
    unbiasedness) holds exactly whenever |q|/s is exact in binary32."""
    v = -num / den                      # negative: also pins the sign handling
    scale = 1.0
    k = np.arange(1 << 24, dtype=np.uint32)
    low = np.random.default_rng(s).integers(0, 256, k.size, dtype=np.uint32)
    q = oracle.round_words(v, scale, s, (k << 8) | low).astype(np.int64)
    x = Fraction(num, den) * s
    l = x.numerator // x.denominator
    frac = x - l
    ups = int((q == -(l + 1)).sum())
    downs = int((q == -l).sum())
    assert ups + downs == 1 << 24
    assert Fraction(ups, 1 << 24) == frac
    # the "up" outcomes are exactly the uniforms below frac
    assert np.array_equal(q == -(l + 1), k < ups)
    mean = Fraction(0)
    for lev, cnt in ((l, downs), (l + 1, ups)):
        mean += Fraction(cnt, 1 << 24) * Fraction(float(oracle.dequant(-lev, scale, s)))
    if s in (1, 2, 4):
        assert mean == Fraction(-num, den)
    else:
        assert abs(mean - Fraction(-num, den)) <= Fraction(num, den) * Fraction(1, 1 << 23)


def test_round_up_count_is_ceil_when_inexact():
    """When frac * 2^24 is not an integer the count of 'up' outcomes is its ceiling, so the
    bias is below 2^-24 * scale / s."""
    rng = np.random.default_rng(0)
    k = np.arange(1 << 24, dtype=np.uint32) << 8
    for s in (1, 3, 7):
        scale = f32(rng.uniform(0.5, 3.0))
        v = f32(rng.uniform(1e-4, 0.01) * scale)      # small: frac has bits below 2^-24
        a = X.rn32(Fraction(v) / Fraction(scale))
        x = X.rn32(a * s)
        l = x.numerator // x.denominator
        frac = x - l
        q = oracle.round_words(v, scale, s, k).astype(np.int64)
        ups = int((q == l + 1).sum())
        assert ups == math.ceil(frac * (1 << 24))
        assert (frac * (1 << 24)).denominator != 1


def test_round_boundaries_and_signs():
    """|v| = ||v|| sits outside every half-open interval of Eq. (9): it maps to level s for
    every random word.  Level 0 carries no sign; -0.0 is level 0."""
    for s in (1, 3, 4, 7, 127):
        for w in (0, 0xFFFFFFFF, 0x80000000, 0x000000FF):
            assert oracle.round_level(2.5, 2.5, s, w) == s
            assert oracle.round_level(-2.5, 2.5, s, w) == -s
            assert oracle.round_level(0.0, 2.5, s, w) == 0
            assert oracle.round_level(-0.0, 2.5, s, w) == 0
            assert oracle.round_level(1.0, 0.0, s, w) == 0
    # exact grid points never move, whatever the word
    for s in (2, 4):
        for j in range(s + 1):
            for w in (0, 0xFFFFFFFF):
                assert oracle.round_level(j / s, 1.0, s, w) == j
    # word 0 -> u = 0: rounds up whenever frac > 0; word 2^32-1 -> u = 1 - 2^-24: up only if
    # frac > u, impossible for frac on the 2^-24 grid below 1
    assert oracle.round_level(0.3, 1.0, 1, 0) == 1
    assert oracle.round_level(0.3, 1.0, 1, 0xFFFFFFFF) == 0
    # only the top 24 bits of the word matter
    assert oracle.round_level(0.3, 1.0, 1, 0x4CCCCC00) == oracle.round_level(0.3, 1.0, 1, 0x4CCCCCFF)
    # u < frac is strict: frac = 0.5 exactly, u = 0.5 exactly -> stays down
    assert oracle.round_level(0.5, 1.0, 1, 0x80000000) == 0
    assert oracle.round_level(0.5, 1.0, 1, 0x7FFFFF00) == 1


def test_ratio_never_exceeds_one():
    """Correctly rounded |v|/scale <= 1 and (|v|/scale)*s <= s whenever |v| <= scale."""
    rng = np.random.default_rng(1)
    bits = rng.integers(0x00000001, 0x7F000000, 4000, dtype=np.uint32)
    vals = bits.view(np.float32)
    for s in (1, 3, 7, 127):
        for a, b in zip(vals[::2], vals[1::2]):
            lo, hi = (a, b) if a <= b else (b, a)
            for w in (0, 0xFFFFFFFF):
                assert 0 <= oracle.round_level(float(lo), float(hi), s, w) <= s


# ------------------------------------------------------------------ exact re-derivation ----

def _random_bucket(rng, n, kind):
    if kind == "normal":
        g = rng.standard_normal(n)
        h = 0.3 * rng.standard_normal(n)
    elif kind == "tiny":            # denormal range: flush-to-zero would change the result
        g = rng.standard_normal(n) * 1e-41
        h = rng.standard_normal(n) * 1e-41
    elif kind == "mixed":
        g = rng.standard_normal(n) * 10.0 ** rng.integers(-30, 20, n)
        h = rng.standard_normal(n) * 10.0 ** rng.integers(-30, 20, n)
    else:                           # zeros, negative zeros, repeated maxima
        g = rng.choice([0.0, -0.0, 1.5, -1.5, 0.75], n)
        h = rng.choice([0.0, -0.0, 0.25], n)
    return g.astype(np.float32), h.astype(np.float32)


@pytest.mark.parametrize("kind", ["normal", "tiny", "mixed", "lattice"])
@pytest.mark.parametrize("s", [1, 3, 4, 7, 100])
def test_bucket_matches_exact_rational_model(kind, s):
    """Operation order and one-rounding-per-operation of Eq. (7), (8)-(9), (6), against exact
    rationals rounded once per binary32 operation."""
    rng = np.random.default_rng([len(kind), ord(kind[0]), s])
    alpha, beta = f32(0.7), f32(0.9)
    for trial in range(6):
        n = int(rng.integers(1, 40))
        g, h = _random_bucket(rng, n, kind)
        i0, p, seed, step = 8 * int(rng.integers(0, 1 << 20)), int(rng.integers(0, 64)), 0xABCDEF12345, trial
        q, scale, gt, hn = oracle.bucket_step(g, h, i0, p, s, alpha, beta, seed, step)
        eq, escale, egt, ehn = X.bucket_step([float(x) for x in g], [float(x) for x in h], i0, p, s,
                                             alpha, beta, seed, step)
        assert [int(x) for x in q] == eq
        assert Fraction(float(scale)) == escale
        assert [Fraction(float(x)) for x in gt] == egt
        assert [Fraction(float(x)) for x in hn] == ehn


def test_scalar_steps_are_the_equations():
    """Eq. (7), (8), (6) one at a time against the rational model (catches g/v swaps, a
    missing alpha or beta, a flipped subtraction)."""
    rng = np.random.default_rng(2)
    for _ in range(300):
        g, h, a, b, sc = (f32(t) for t in rng.standard_normal(5))
        sc = abs(sc)
        assert Fraction(float(oracle.compensate(g, a, h))) == X.rn32(Fraction(g) + X.rn32(Fraction(a) * Fraction(h)))
        gt = f32(rng.standard_normal())
        assert Fraction(float(oracle.error(b, h, g, gt))) == X.rn32(
            X.rn32(Fraction(b) * Fraction(h)) + X.rn32(Fraction(g) - Fraction(gt)))
        s = int(rng.integers(1, 128))
        q = int(rng.integers(-s, s + 1))
        want = X.rn32(Fraction(sc) * X.rn32(Fraction(abs(q), s)))
        assert Fraction(float(oracle.dequant(q, sc, s))) == (-want if q < 0 else want)


# ------------------------------------------------------------------ invariants -------------

def _run(P, n, bucket, s, alpha, beta, iters, seed=1, gscale=1.0, rng_seed=0, keep=False):
    rng = np.random.default_rng(rng_seed)
    h = np.zeros((P, n), np.float32)
    log = []
    for t in range(iters):
        g = (gscale * rng.standard_normal((P, n))).astype(np.float32)
        h_before = h.copy()
        q, scales, gt = oracle.batch_step(g, h, bucket, s, alpha, beta, seed, t, want_gt=True)
        log.append((g, h_before, q, scales, gt, h.copy()))
    return log


@pytest.mark.parametrize("s,bucket,n", [(1, 512, 4096), (3, 64, 1000), (7, 8, 250), (4, 4096, 5000)])
def test_code_range_error_bound_and_max_element(s, bucket, n):
    """Levels lie in [-s, s] (codebook of Eq. (8)); |v_i - g~_i| <= ||v||/s because the value
    moves to an end of its interval of width ||v||/s (Eq. (9)); the element attaining the norm
    is reproduced exactly (its rounding-up probability is 0)."""
    alpha, beta = f32(1.0), f32(0.9)
    for g, h0, q, scales, gt, h1 in _run(3, n, bucket, s, alpha, beta, 4):
        assert q.min() >= -s and q.max() <= s
        v = g + F32(alpha) * h0
        nb = scales.shape[1]
        for p in range(g.shape[0]):
            for k in range(nb):
                sl = slice(k * bucket, min(n, (k + 1) * bucket))
                vv = v[p, sl]
                assert scales[p, k] == np.abs(vv).max()
                err = np.abs(vv.astype(np.float64) - gt[p, sl])
                assert err.max() <= float(scales[p, k]) / s * (1 + 4 * 2.0 ** -24)
                imax = int(np.abs(vv).argmax())
                assert abs(int(q[p, sl][imax])) == s
                assert gt[p, sl][imax] == vv[imax]
                assert np.all(np.sign(gt[p, sl]) * np.sign(vv) >= 0)


def test_last_bucket_is_short_and_buckets_are_independent():
    """A bucket is a run of consecutive elements; the last may be short and takes its scale
    from the elements that exist.  Changing one bucket leaves the others' levels alone."""
    rng = np.random.default_rng(3)
    P, n, bucket, s = 2, 1000, 64, 3
    g = rng.standard_normal((P, n)).astype(np.float32)
    h = np.zeros_like(g)
    q, scales, _ = oracle.batch_step(g, h.copy(), bucket, s, 1.0, 1.0, 9, 0)
    assert scales.shape == (P, 16)
    assert scales[0, 15] == np.abs(g[0, 960:]).max()
    g2 = g.copy()
    g2[0, 70] = 100.0
    q2, scales2, _ = oracle.batch_step(g2, h.copy(), bucket, s, 1.0, 1.0, 9, 0)
    same = np.ones(n, bool)
    same[64:128] = False
    assert np.array_equal(q[0, same], q2[0, same]) and np.array_equal(q[1], q2[1])
    assert scales2[0, 1] == 100.0
    # a bucket computed on its own, with its offset, equals its slice of the batch
    qb, sb, _, _ = oracle.bucket_step(g[1, 128:192], h[1, 128:192], 128, 1, s, 1.0, 1.0, 9, 0)
    assert np.array_equal(qb, q[1, 128:192]) and sb == scales[1, 2]


def test_deterministic_cases():
    """Inputs on the quantisation grid are reproduced whatever the random words; with h = 0 and
    alpha = beta = 1 the error stays 0.  An all-zero bucket gives scale 0, levels 0,
    h' = beta*h + g.  A one-element bucket is its own norm."""
    for s in (1, 2, 4):
        M = 3.0
        levels = np.arange(-s, s + 1)
        g = np.tile((M * levels / s).astype(np.float32), 5)[None, :]
        for seed in (1, 2, 3):
            h = np.zeros_like(g)
            q, scales, gt = oracle.batch_step(g, h, 8 * len(levels), s, 1.0, 1.0, seed, 0, want_gt=True)
            assert np.array_equal(gt, g) and np.all(h == 0) and scales[0, 0] == M
            assert np.array_equal(q[0], np.tile(levels, 5))
    g = np.zeros((1, 16), np.float32)
    h = np.full((1, 16), 0.0, np.float32)
    q, scales, gt = oracle.batch_step(g, h, 8, 3, 1.0, 0.5, 1, 0, want_gt=True)
    assert not q.any() and not scales.any() and not gt.any() and not h.any()
    g = np.array([[0.25, -4.0, 7.5]], np.float32)
    h = np.zeros_like(g)
    q, scales, gt = oracle.batch_step(g, h, 1, 7, 1.0, 1.0, 5, 3, want_gt=True)
    assert list(q[0]) == [7, -7, 7] and np.array_equal(gt, g) and np.array_equal(scales[0], np.abs(g[0]))


@pytest.mark.parametrize("alpha,beta", [(1.0, 0.9), (0.2, 0.9), (0.01, 1.0), (1.0, 1.0)])
def test_error_recursion_closed_forms(alpha, beta):
    """Eq. (5): h(t) = sum_{t'<t} beta^(t-1-t') (g(t') - g~(t')), and the supplement's
    re-organisation (proof of Lemma 2): h(t) = -sum_{t'<t} (beta-alpha)^(t-t'-1) eps(t') with
    eps = g~ - (g + alpha h) (Eq. (10)); both recomputed in float64 from the logged g, g~."""
    alpha, beta = f32(alpha), f32(beta)
    log = _run(2, 600, 64, 3, alpha, beta, 8, gscale=0.5)
    T = len(log)
    a64, b64 = float(alpha), float(beta)
    for t in range(1, T + 1):
        h_t = log[t - 1][5].astype(np.float64)
        closed = np.zeros_like(h_t)
        eps_form = np.zeros_like(h_t)
        for tp in range(t):
            g, h0, q, scales, gt, h1 = log[tp]
            closed += b64 ** (t - 1 - tp) * (g.astype(np.float64) - gt)
            eps = gt.astype(np.float64) - (g.astype(np.float64) + a64 * h0.astype(np.float64))
            eps_form -= (b64 - a64) ** (t - tp - 1) * eps
        tol = 1e-6 * max(1.0, np.abs(h_t).max())
        assert np.abs(h_t - closed).max() <= tol
        assert np.abs(h_t - eps_form).max() <= tol
    assert np.abs(log[-1][5]).max() > 1e-3      # the recursion is not vacuous


def test_special_cases_qsgd_ternary_last_step():
    """alpha = 0: the levels do not depend on h (QSGD, Section 5.2).  s = 1: ternary
    {-||v||, 0, +||v||}.  beta = 0: h' = g - g~ (feedback from the last step only)."""
    rng = np.random.default_rng(4)
    P, n, bucket = 2, 512, 128
    g = rng.standard_normal((P, n)).astype(np.float32)
    h_rand = rng.standard_normal((P, n)).astype(np.float32)
    q0, sc0, _ = oracle.batch_step(g, np.zeros_like(g), bucket, 4, 0.0, 1.0, 7, 2)
    q1, sc1, _ = oracle.batch_step(g, h_rand.copy(), bucket, 4, 0.0, 1.0, 7, 2)
    assert np.array_equal(q0, q1) and np.array_equal(sc0, sc1)
    qa, _, _ = oracle.batch_step(g, h_rand.copy(), bucket, 4, 1.0, 1.0, 7, 2)
    assert not np.array_equal(q0, qa)
    q, sc, gt = oracle.batch_step(g, np.zeros_like(g), bucket, 1, 1.0, 1.0, 7, 2, want_gt=True)
    big = np.repeat(sc, bucket, axis=1)
    assert np.all((gt == 0) | (gt == big) | (gt == -big))
    h = h_rand.copy()
    q, sc, gt = oracle.batch_step(g, h, bucket, 4, 1.0, 0.0, 7, 2, want_gt=True)
    assert np.array_equal(h, g - gt)
    # update_h = 0 leaves h alone
    h = h_rand.copy()
    oracle.batch_step(g, h, bucket, 4, 1.0, 0.5, 7, 2, update_h=False)
    assert np.array_equal(h, h_rand)


def test_ternary_probability_statistical():
    """s = 1 with the l_inf norm: P(|level| = 1) = |v|/||v|| (the ternary quantiser the paper
    cites); checked over many iterations' independent words.  Also the per-element variance
    (||v||/s)^2 f(1-f) summed over the bucket."""
    n, iters = 256, 400
    rng = np.random.default_rng(6)
    g = rng.uniform(-1, 1, n).astype(np.float32)
    g[0] = 1.0
    hits = np.zeros(n)
    sq = 0.0
    for t in range(iters):
        q, sc, gt, _ = oracle.bucket_step(g, np.zeros(n, np.float32), 0, 0, 1, 1.0, 1.0, 77, t)
        hits += np.abs(q)
        sq += ((gt.astype(np.float64) - g) ** 2).sum()
    prob = np.abs(g.astype(np.float64))
    se = np.sqrt(prob * (1 - prob) / iters) + 1e-9
    assert np.all(np.abs(hits / iters - prob) < 5 * se + 1e-12)
    var = (prob * (1 - prob)).sum()
    assert abs(sq / iters - var) < 0.1 * var


def test_resume_is_bit_identical():
    """The random stream is a pure function of (seed, step, worker, element): running T steps
    equals running k steps, saving h, and running the remaining T-k."""
    rng = np.random.default_rng(8)
    gs = [rng.standard_normal((2, 300)).astype(np.float32) for _ in range(6)]
    h = np.zeros((2, 300), np.float32)
    qs = [oracle.batch_step(g, h, 64, 3, 1.0, 0.9, 5, t)[0] for t, g in enumerate(gs)]
    h2 = np.zeros((2, 300), np.float32)
    for t in range(3):
        oracle.batch_step(gs[t], h2, 64, 3, 1.0, 0.9, 5, t)
    saved = h2.copy()
    qs2 = [oracle.batch_step(gs[t], saved, 64, 3, 1.0, 0.9, 5, t)[0] for t in range(3, 6)]
    assert all(np.array_equal(a, b) for a, b in zip(qs[3:], qs2))
    assert np.array_equal(saved, h)


# ------------------------------------------------------------------ encoding ---------------

@pytest.mark.parametrize("s", [1, 2, 3, 4, 7, 8, 20, 40, 100, 127])
def test_pack_is_lsb_first_bitstream(s):
    """r bits per element in one contiguous LSB-first stream: the packed row read as a
    little-endian integer is sum_i (q_i + s) << (i r); pad bits are zero; unpack inverts."""
    rng = np.random.default_rng(s)
    r = oracle.code_bits(s)
    for n in (1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 63, 64, 65, 200):
        q = rng.integers(-s, s + 1, n).astype(np.int8)
        packed = oracle.pack(q, s)
        assert packed.size == (n * r + 7) // 8 == oracle.row_bytes(n, s)
        assert bytes(packed) == X.pack([int(x) for x in q], s)
        assert int.from_bytes(bytes(packed), "little") >> (n * r) == 0
        assert np.array_equal(oracle.unpack(packed, n, s), q)
        assert X.unpack(bytes(packed), n, s) == [int(x) for x in q]
    # explicit small case, r = 2: codes 0,1,2,1 -> bits 00 01 10 01 LSB-first = 0b01100100
    assert list(oracle.pack(np.array([-1, 0, 1, 0], np.int8), 1)) == [0b01100100]
    # r = 3, s = 3: codes 6,0,3 -> 110 | 000<<3 | 011<<6 = 0b0_1100_0110 -> bytes C6 00
    assert list(oracle.pack(np.array([3, -3, 0], np.int8), 3)) == [0xC6, 0x00]


# ------------------------------------------------------------------ aggregation ------------

@pytest.mark.parametrize("P", [1, 3, 4, 8])
def test_aggregate_is_the_mean(P):
    """Eq. (4): g~ = (1/P) sum_p g~_p, against a float64 mean of the per-worker dequantised
    vectors; P = 1 returns the single worker's g~ bit for bit."""
    rng = np.random.default_rng(P)
    n, bucket, s = 777, 64, 3
    g = rng.standard_normal((P, n)).astype(np.float32)
    h = np.zeros_like(g)
    q, scales, gt = oracle.batch_step(g, h, bucket, s, 1.0, 1.0, 3, 0, want_gt=True)
    codes = oracle.pack_rows(q, s)
    out = oracle.aggregate(codes, scales, n, bucket, s)
    mean = gt.astype(np.float64).mean(axis=0)
    assert np.abs(out - mean).max() <= 1e-6 * np.abs(mean).max()
    if P == 1:
        assert np.array_equal(out, gt[0])
    # exact model of the summation order: p = 0..P-1, then one division
    acc = np.zeros(n, np.float32)
    for p in range(P):
        acc = acc + gt[p]
    assert np.array_equal(out, acc / F32(P))
    # strided rows
    codes2 = np.zeros((P, codes.shape[1] + 5), np.uint8)
    codes2[:, : codes.shape[1]] = codes
    scales2 = np.zeros((P, scales.shape[1] + 3), np.float32)
    scales2[:, : scales.shape[1]] = scales
    assert np.array_equal(oracle.aggregate(codes2, scales2, n, bucket, s), out)


def test_error_update_from_message_equals_fused_step():
    """Eq. (6) applied to the decoded message reproduces the fused step's h."""
    rng = np.random.default_rng(11)
    n, bucket, s = 500, 40, 7
    g = rng.standard_normal((1, n)).astype(np.float32)
    h0 = rng.standard_normal((1, n)).astype(np.float32)
    h = h0.copy()
    q, scales, _ = oracle.batch_step(g, h, bucket, s, 0.5, 0.8, 3, 1)
    h2 = h0[0].copy()
    oracle.error_update_row(g[0], oracle.pack(q[0], s), scales[0], bucket, s, 0.8, h2)
    assert np.array_equal(h2, h[0])


# ------------------------------------------------------------------ l_2 scaling ------------

@pytest.mark.parametrize("kind", ["normal", "mixed", "lattice"])
@pytest.mark.parametrize("s", [1, 4, 7])
def test_l2_bucket_matches_exact_rational_model(kind, s):
    """The l_2 route against exact rationals: squares, the balanced tree by index, one
    correctly rounded square root, then Eq. (7)-(9), (6) as before."""
    rng = np.random.default_rng([7, len(kind), s])
    alpha, beta = f32(0.2), f32(0.9)
    for trial in range(6):
        n = int(rng.integers(1, 40))
        g, h = _random_bucket(rng, n, kind)
        if kind == "mixed":                       # keep squares inside the binary32 range
            g = (rng.standard_normal(n) * 10.0 ** rng.integers(-12, 12, n)).astype(np.float32)
            h = (rng.standard_normal(n) * 10.0 ** rng.integers(-12, 12, n)).astype(np.float32)
        q, scale, gt, hn = oracle.bucket_step(g, h, 64, 3, s, alpha, beta, 99, trial, norm="l2")
        eq, escale, egt, ehn = X.bucket_step([float(x) for x in g], [float(x) for x in h], 64, 3, s,
                                             alpha, beta, 99, trial, norm="l2")
        assert Fraction(float(scale)) == escale
        assert [int(x) for x in q] == eq
        assert [Fraction(float(x)) for x in gt] == egt
        assert [Fraction(float(x)) for x in hn] == ehn


def test_l2_norm_value_and_order():
    """Close to the float64 norm; independent of zero padding; the summation order is the
    balanced tree (a left-to-right sum gives a different binary32 value on this input)."""
    rng = np.random.default_rng(12)
    for n in (1, 2, 3, 5, 8, 100, 512, 1000, 4096):
        v = rng.standard_normal(n).astype(np.float32)
        got = float(oracle.bucket_scale_l2(v))
        ref = float(np.linalg.norm(v.astype(np.float64)))
        assert abs(got - ref) <= ref * (math.log2(max(n, 2)) + 2) * 2.0 ** -24
        padded = np.concatenate([v, np.zeros(3, np.float32)])
        assert float(oracle.bucket_scale_l2(padded)) == got
    differ = 0
    for trial in range(200):
        v = rng.standard_normal(16).astype(np.float32)
        sq = v * v
        level = sq.copy()
        while level.size > 1:
            level = level[0::2] + level[1::2]
        tree = np.sqrt(level[0])
        seq = np.float32(0)
        for x in sq:
            seq = np.float32(seq + x)
        seq = np.sqrt(seq)
        got = oracle.bucket_scale_l2(v)
        assert float(got) == float(tree)
        assert Fraction(float(got)) == X.norm_l2([Fraction(float(x)) for x in v])
        differ += float(tree) != float(seq)
    assert differ > 10          # the order is observable, and it is the tree's


def test_l2_norm_dominates_every_element():
    """fl(sqrt(fl(x^2))) = |x| in binary32 while x^2 is a normal number, and sums of
    non-negative terms are monotone under rounding, so the computed l_2 norm is then never below
    max|v_i|: the ratio stays <= 1 and the element of a one-element bucket is reproduced
    exactly, as with l_inf."""
    rng = np.random.default_rng(13)
    for x in rng.uniform(1.0, 2.0, 2000).astype(np.float32):
        assert float(oracle.bucket_scale_l2(np.array([x], np.float32))) == float(x)
    for n in (2, 3, 17, 64):
        for _ in range(200):
            v = (rng.standard_normal(n) * 10.0 ** rng.integers(-6, 6)).astype(np.float32)
            assert float(oracle.bucket_scale_l2(v)) >= float(np.abs(v).max())
    q, sc, gt, _ = oracle.bucket_step(np.array([-1.7], np.float32), np.zeros(1, np.float32), 0, 0, 3, 1.0, 1.0,
                                      1, 0, norm="l2")
    assert int(q[0]) == -3 and float(gt[0]) == float(np.float32(-1.7))


@pytest.mark.parametrize("s", [1, 4, 127])
def test_l2_squares_that_underflow(s):
    """Where fl(v_i^2) is a denormal number the computed l_2 norm can fall below |v_i| (the
    quotient of Eq. (9) then exceeds 1 and the level is s, the end of the grid of Eq. (8)), and
    where every square rounds to 0 the norm is 0 and every level is 0 with h' = beta*h + g
    (Eq. (6) with g~ = 0).  Against the exact-rational model, plus the two facts themselves."""
    rng = np.random.default_rng([21, s])
    alpha, beta = f32(0.2), f32(0.9)
    above = 0
    for trial in range(40):
        n = int(rng.integers(1, 24))
        g = np.zeros(n, np.float32)
        h = np.zeros(n, np.float32)
        at = int(rng.integers(n))
        g[at] = F32(rng.choice([-1.0, 1.0]) * 10.0 ** rng.uniform(-23.0, -19.0))
        if trial % 3 == 0:                           # a few more tiny neighbours
            g[rng.integers(n, size=3)] = F32(10.0 ** rng.uniform(-24.0, -20.0))
        q, scale, gt, hn = oracle.bucket_step(g, h, 8 * trial, 2, s, alpha, beta, 5, trial, norm="l2")
        eq, escale, egt, ehn = X.bucket_step([float(x) for x in g], [float(x) for x in h], 8 * trial, 2, s,
                                             alpha, beta, 5, trial, norm="l2")
        assert Fraction(float(scale)) == escale
        assert [int(x) for x in q] == eq
        assert [Fraction(float(x)) for x in gt] == egt
        assert [Fraction(float(x)) for x in hn] == ehn
        assert all(-s <= int(x) <= s for x in q)
        big = int(np.abs(g).argmax())
        if float(scale) == 0.0:                      # every square rounded to 0
            assert not q.any()
        elif float(scale) < abs(float(g[big])):      # the norm fell below its largest element
            above += 1
            assert abs(int(q[big])) == s
    assert above > 0
    # every square underflows to 0
    g = (rng.standard_normal(16) * 1e-30).astype(np.float32)
    h = (rng.standard_normal(16) * 1e-30).astype(np.float32)
    q, scale, gt, hn = oracle.bucket_step(g, h, 0, 0, s, alpha, beta, 5, 0, norm="l2")
    assert float(scale) == 0.0 and not q.any() and not gt.any()
    want = [X.rn32(X.rn32(Fraction(float(beta)) * Fraction(float(b))) + Fraction(float(a))) for a, b in zip(g, h)]
    assert [Fraction(float(x)) for x in hn] == want


def test_linf_scale_is_the_largest_magnitude():
    """The l_inf norm of a bucket (text after Eq. (8)) against numpy's norm(., inf): order-free,
    sign-free, exact (one of the |v_i| themselves), denormals kept, 0 for an all-zero bucket."""
    rng = np.random.default_rng(31)
    for n in (1, 2, 7, 64, 1000):
        for scale in (1.0, 1e-41, 1e30):
            v = (rng.standard_normal(n) * scale).astype(np.float32)
            got = float(oracle.bucket_scale(v))
            assert got == float(np.linalg.norm(v.astype(np.float64), np.inf))
            assert got == float(oracle.bucket_scale(-v[::-1].copy()))
            assert got in set(np.abs(v).tolist())
    assert float(oracle.bucket_scale(np.array([0.0, -0.0, 0.0], np.float32))) == 0.0
    assert float(oracle.bucket_scale(np.array([-3.5, 2.0, 3.25], np.float32))) == 3.5
    # the bucket step takes its scale from this function
    g = rng.standard_normal(24).astype(np.float32)
    h = rng.standard_normal(24).astype(np.float32)
    _, sc, _, _ = oracle.bucket_step(g, h, 0, 0, 3, f32(0.5), f32(0.9), 1, 0)
    v = np.array([oracle.compensate(float(a), f32(0.5), float(b)) for a, b in zip(g, h)], np.float32)
    assert float(sc) == float(oracle.bucket_scale(v))


def test_l2_lemma1_unbiased_and_variance_bound():
    """Lemma 1 (borrowed from QSGD for l_2 scaling): E[eps] = 0 and
    E||eps||^2 <= min(d/s^2, sqrt(d)/s) ||v||^2, over many independent iterations' words."""
    d, iters = 64, 3000
    rng = np.random.default_rng(14)
    v = rng.standard_normal(d).astype(np.float32)
    for s in (1, 4):
        acc = np.zeros(d)
        sq = 0.0
        for t in range(iters):
            q, sc, gt, _ = oracle.bucket_step(v, np.zeros(d, np.float32), 0, 0, s, 1.0, 1.0, 5, t, norm="l2")
            eps = gt.astype(np.float64) - v
            acc += eps
            sq += float((eps ** 2).sum())
        norm2 = float((v.astype(np.float64) ** 2).sum())
        bound = min(d / s ** 2, math.sqrt(d) / s) * norm2
        assert sq / iters <= bound
        assert sq / iters > 0.05 * bound            # the bound is not vacuous here
        per_elem_sd = float(sc) / s * 0.5 / math.sqrt(iters)
        assert np.abs(acc / iters).max() < 6 * per_elem_sd
    # sparse output: with l_2 scaling most levels are 0 (expected non-zeros <= s(s + sqrt(d)))
    q, _, _, _ = oracle.bucket_step(v, np.zeros(d, np.float32), 0, 0, 1, 1.0, 1.0, 5, 0, norm="l2")
    assert (q != 0).sum() < d / 2


def test_l2_batch_uses_tree_per_bucket_and_recursion_holds():
    """Batch route with l_2: per-bucket norms equal the single-bucket routine; Eq. (5) closed
    form still holds (it does not depend on the norm)."""
    rng = np.random.default_rng(15)
    P, n, bucket, s = 2, 300, 64, 4
    alpha, beta = f32(0.2), f32(0.9)
    h = np.zeros((P, n), np.float32)
    closed = np.zeros((P, n))
    for t in range(5):
        g = rng.standard_normal((P, n)).astype(np.float32)
        v = g + F32(alpha) * h
        q, scales, gt = oracle.batch_step(g, h, bucket, s, alpha, beta, 3, t, want_gt=True, norm="l2")
        for p in range(P):
            for k in range(scales.shape[1]):
                assert scales[p, k] == oracle.bucket_scale_l2(v[p, k * bucket:(k + 1) * bucket])
        closed = float(beta) * closed + (g.astype(np.float64) - gt)
        assert np.abs(h - closed).max() <= 1e-6 * max(1.0, np.abs(closed).max())


# ------------------------------------------------------------------ model update -----------

def test_sgd_step_is_the_update_rule():
    """Eq. (4) / Alg. 1 last line: w <- w - eta * g~; the product is rounded, then the
    difference."""
    rng = np.random.default_rng(21)
    w = rng.standard_normal(500).astype(np.float32)
    g = rng.standard_normal(500).astype(np.float32)
    eta = f32(0.02)
    got = oracle.sgd_step(w.copy(), g, eta)
    ref = w.astype(np.float64) - float(eta) * g.astype(np.float64)
    assert np.abs(got - ref).max() <= 1e-6 * np.abs(ref).max()
    for i in range(50):
        want = X.rn32(Fraction(float(w[i])) - X.rn32(Fraction(eta) * Fraction(float(g[i]))))
        assert Fraction(float(got[i])) == want
    assert np.array_equal(oracle.sgd_step(w.copy(), g, 0.0), w)


def _least_squares_run(d, alpha, beta, quantise, iters=600, P=4, mb=16, s=4, eta=0.02, seed=0):
    """Distributed least squares as in Section 6.1 (synthetic y = w*^T x + noise, eta = 0.02,
    l_2 scaling, s = 4), whole vector as one bucket; returns the mean distance to the optimum
    over the last 100 iterations."""
    rng = np.random.default_rng(seed)
    n = 4000
    Xd = rng.standard_normal((n, d)).astype(np.float32)
    wstar = rng.standard_normal(d).astype(np.float32)
    y = (Xd @ wstar + 0.1 * rng.standard_normal(n)).astype(np.float32)
    wopt = np.linalg.lstsq(Xd.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    w = np.zeros(d, np.float32)
    h = np.zeros((P, d), np.float32)
    shards = np.array_split(np.arange(n), P)
    dist = []
    for t in range(iters):
        g = np.zeros((P, d), np.float32)
        for p in range(P):
            idx = rng.choice(shards[p], mb, replace=False)
            g[p] = (Xd[idx].T @ (Xd[idx] @ w - y[idx]) / mb).astype(np.float32)
        if quantise:
            q, sc, _ = oracle.batch_step(g, h, d, s, alpha, beta, 1, t, norm="l2")
            gavg = oracle.aggregate(oracle.pack_rows(q, s), sc, d, d, s)
        else:
            gavg = g.mean(axis=0).astype(np.float32)
        oracle.sgd_step(w, gavg, eta)
        dist.append(float(np.linalg.norm(w - wopt)))
    return float(np.mean(dist[-100:]))


def test_closed_loop_error_feedback_shrinks_the_gap():
    """Section 6.1 / Fig. 2, qualitatively: with the paper's settings (alpha = 0.2, beta = 0.9)
    the error-compensated run ends closer to the optimum than QSGD (alpha = 0, no feedback),
    and both stay above the unquantised run."""
    fp = _least_squares_run(256, 0.0, 0.0, quantise=False)
    qsgd = _least_squares_run(256, 0.0, 0.0, quantise=True)
    ecq = _least_squares_run(256, f32(0.2), f32(0.9), quantise=True)
    assert fp < ecq < qsgd
    assert (ecq - fp) < 0.5 * (qsgd - fp)


# ------------------------------------------------------------------ entropy-coded length ---

def test_level_histogram_and_entropy_bound():
    """Section 4, cost paragraph: d_k = dimensions on level k; length <= sum_k d_k log2(d/d_k).
    Closed forms: a single occupied level costs 0 bits, m equally occupied levels cost
    d log2(m); the bound never exceeds the fixed-length d*r bits."""
    rng = np.random.default_rng(31)
    for s in (1, 3, 7, 127):
        q = rng.integers(-s, s + 1, 5000).astype(np.int8)
        counts = oracle.level_histogram(q, s)
        assert np.array_equal(counts, np.bincount(q.astype(np.int64) + s, minlength=2 * s + 1).astype(np.uint64))
        assert counts.sum() == q.size
        bits = oracle.entropy_bound_bits(counts)
        p = counts[counts > 0] / q.size
        assert abs(bits - q.size * float(-(p * np.log2(p)).sum())) < 1e-6 * bits
        assert bits <= q.size * oracle.code_bits(s)
    assert oracle.entropy_bound_bits(np.array([0, 4096, 0], np.uint64)) == 0.0
    assert oracle.entropy_bound_bits(np.array([100, 100, 100, 100], np.uint64)) == 400 * 2.0
    assert abs(oracle.entropy_bound_bits(np.array([50, 50, 50], np.uint64)) - 150 * math.log2(3)) < 1e-9
    # heavy-tailed gradients put most elements on level 0: far below r bits per element
    g = (1e-3 * rng.standard_t(3, 8192)).astype(np.float32)
    q, _, _, _ = oracle.bucket_step(g, np.zeros_like(g), 0, 0, 7, 1.0, 1.0, 1, 0)
    assert oracle.entropy_bound_bits(oracle.level_histogram(q, 7)) < 0.5 * g.size * oracle.code_bits(7)


# ------------------------------------------------------------------ Huffman coding ---------

def _kraft(lengths):
    return sum(Fraction(1, 1 << int(l)) for l in lengths if l > 0)


def test_huffman_textbook_example_and_kraft():
    """Huffman (1952).  The classic six-symbol example with frequencies 45, 13, 12, 16, 9, 5
    costs 224 bits with lengths 1,3,3,3,4,4; a full code satisfies Kraft with equality."""
    counts = np.array([45, 13, 12, 16, 9, 5], np.uint64)
    lengths = oracle.huffman_lengths(counts)
    assert list(lengths) == [1, 3, 3, 3, 4, 4]
    assert int((counts * lengths).sum()) == 224
    assert _kraft(lengths) == 1
    assert [int(c) for c in oracle.huffman_codes(lengths)] == [0b0, 0b100, 0b101, 0b110, 0b1110, 0b1111]
    # degenerate rows
    assert list(oracle.huffman_lengths(np.array([0, 7, 0], np.uint64))) == [0, 1, 0]
    assert list(oracle.huffman_lengths(np.array([0, 0, 0], np.uint64))) == [0, 0, 0]
    assert list(oracle.huffman_lengths(np.array([3, 0, 3], np.uint64))) == [1, 0, 1]


def test_huffman_is_optimal_and_between_entropy_bounds():
    """Optimal among prefix codes (brute force over every length assignment with Kraft <= 1 on
    small alphabets) and entropy <= length < entropy + d, the window the paper's bound
    sum_k d_k log2(d/d_k) sits at the bottom of."""
    import itertools
    rng = np.random.default_rng(41)
    for trial in range(60):
        m = int(rng.integers(2, 6))
        counts = rng.integers(1, 50, m).astype(np.uint64)
        if trial % 5 == 0:
            counts[:] = counts[0]                       # all ties
        lengths = oracle.huffman_lengths(counts)
        cost = int((counts * lengths).sum())
        best = min(int(sum(int(c) * l for c, l in zip(counts, ls)))
                   for ls in itertools.product(range(1, m + 1), repeat=m) if _kraft(ls) <= 1)
        assert cost == best
        assert _kraft(lengths) == 1
        assert list(lengths) == X.huffman_lengths([int(c) for c in counts])
    for s in (1, 3, 7, 60, 127):
        p = rng.dirichlet(np.full(2 * s + 1, 0.3))
        counts = rng.multinomial(200_000, p).astype(np.uint64)
        lengths = oracle.huffman_lengths(counts)
        assert list(lengths) == X.huffman_lengths([int(c) for c in counts])
        assert [int(c) for c in oracle.huffman_codes(lengths)] == X.huffman_codes([int(l) for l in lengths])
        bits = int((counts * lengths).sum())
        h = oracle.entropy_bound_bits(counts)
        assert h <= bits < h + counts.sum()
        assert bits <= int(counts.sum()) * oracle.code_bits(s)      # never worse than fixed length
        assert _kraft(lengths) == 1 and lengths.max() < 64


def test_huffman_codes_are_prefix_free_and_canonical():
    rng = np.random.default_rng(42)
    counts = rng.integers(0, 1000, 31).astype(np.uint64)
    counts[5] = 0
    lengths = oracle.huffman_lengths(counts)
    codes = oracle.huffman_codes(lengths)
    words = {c: format(int(codes[c]), "b").zfill(int(lengths[c])) for c in range(31) if lengths[c]}
    assert 5 not in words and len(set(words.values())) == len(words)
    for a in words:
        for b in words:
            assert a == b or not words[b].startswith(words[a])
    order = sorted(words, key=lambda c: (lengths[c], c))
    assert [words[c] for c in order] == sorted(words.values(), key=lambda w: (len(w), w))


@pytest.mark.parametrize("s", [1, 3, 7, 100])
def test_huffman_stream_round_trip_and_tiles(s):
    """Encode / decode round trip, the stream read as a little-endian integer against the
    big-integer model, zero pad bits, and independent decoding from every tile offset."""
    rng = np.random.default_rng(s)
    n = 3 * oracle.HUFFMAN_TILE + 77
    g = (rng.standard_t(3, n) * 1e-3).astype(np.float32)
    q, _, _, _ = oracle.bucket_step(g, np.zeros_like(g), 0, 0, s, 1.0, 1.0, 1, 0)
    counts = oracle.level_histogram(q, s)
    lengths = oracle.huffman_lengths(counts)
    codes = oracle.huffman_codes(lengths)
    stream, offs, bits = oracle.huffman_encode(q, s, lengths, codes)
    assert bits == int((counts * lengths).sum()) == int(offs[-1])
    big, pos = X.huffman_encode([int(x) for x in q], s, [int(l) for l in lengths], [int(c) for c in codes])
    assert pos == bits and int.from_bytes(bytes(stream), "little") == big
    assert np.array_equal(oracle.huffman_decode(stream, 0, n, s, lengths, codes), q)
    T = oracle.HUFFMAN_TILE
    assert offs.size == 5 and offs[0] == 0 and np.all(np.diff(offs.astype(np.int64)) > 0)
    for t in range(4):
        cnt = min(T, n - t * T)
        assert np.array_equal(oracle.huffman_decode(stream, int(offs[t]), cnt, s, lengths, codes), q[t * T:t * T + cnt])
    assert bits < n * oracle.code_bits(s)


# ------------------------------------------------------------------ zero-run Huffman coding --

def _zrun_tokens_by_runs(levels, s):
    """Second implementation of the tokeniser, from the runs of the tile instead of a scan:
    every maximal run of zeros gives floor(run / Z) "Z zeros" tokens, the rest joins the level
    that follows it; a rest at the end of the tile gives one closing token."""
    import itertools
    Z = 127 // s
    tokens, pending = [], 0
    for is_zero, grp in itertools.groupby(levels, key=lambda v: v == 0):
        grp = list(grp)
        if is_zero:
            tokens += [2 * s * Z] * (len(grp) // Z)
            pending = len(grp) % Z
        else:
            for v in grp:
                rank = sorted(set(range(-s, s + 1)) - {0}).index(v)
                tokens.append(pending * 2 * s + rank)
                pending = 0
    if pending:
        tokens.append(2 * s * Z)
    return tokens


def _zrun_expand(tokens, s, n):
    Z = 127 // s
    ranks = [v for v in range(-s, s + 1) if v != 0]
    out = []
    for t in tokens:
        if t == 2 * s * Z:
            out += [0] * Z
        else:
            out += [0] * (t // (2 * s)) + [ranks[t % (2 * s)]]
    assert len(out) >= n and not any(out[n:])                  # only zeros are dropped at the tile's end
    return out[:n]


def _random_levels(rng, n, s, p_nonzero):
    q = rng.integers(1, s + 1, n) * rng.choice([-1, 1], n)
    return np.where(rng.random(n) < p_nonzero, q, 0).astype(np.int8)


def test_zrun_alphabet():
    """Z = floor(127/s) and 2sZ + 1 <= 255 tokens for every s the codec takes."""
    for s in range(1, 128):
        Z, A = oracle.zrun_max_run(s), oracle.zrun_symbols(s)
        assert Z == 127 // s and Z >= 1
        assert A == 2 * s * Z + 1 and A <= 255 and A % 2 == 1
        assert 2 * s * (Z + 1) + 1 > 255                      # Z is the largest run that fits a byte of tokens
    assert [oracle.zrun_max_run(s) for s in (1, 3, 4, 7, 127)] == [127, 42, 31, 18, 1]


def test_zrun_tokens_hand_worked():
    """Tokens of small tiles written out by hand (run * 2s + rank; 2sZ for "Z zeros")."""
    tok = lambda q, s: oracle.zrun_tokens(np.array(q, np.int8), s).tolist()
    # s = 1: ranks -1 -> 0, +1 -> 1; Z = 127, "Z zeros" = 254
    assert tok([0, 0, 1, 0, -1, 0, 0], 1) == [2 * 2 + 1, 1 * 2 + 0, 254]
    assert tok([1, 1, -1], 1) == [1, 1, 0]
    assert tok([0] * 127, 1) == [254]                          # exactly Z zeros: one token, nothing pending
    assert tok([0] * 128, 1) == [254, 254]                     # ... one more: a closing token
    assert tok([0] * 127 + [1], 1) == [254, 1]
    assert tok([0] * 126 + [-1], 1) == [126 * 2 + 0]
    assert tok([], 1) == []
    # s = 3: ranks -3,-2,-1,1,2,3 -> 0..5; Z = 42, "Z zeros" = 252
    assert tok([-3, 0, 2, 0, 0, 0, 1], 3) == [0, 1 * 6 + 4, 3 * 6 + 3]
    # s = 63: Z = 2, 126 ranks, "Z zeros" = 252
    assert tok([0, 0, 5], 63) == [252, 5 + 63 - 1]
    assert tok([0, 0, 0, 5], 63) == [252, 126 + 67]
    assert tok([0] * 5, 63) == [252, 252, 252]
    # s = 127: Z = 1, every zero is a token of its own
    assert tok([0, -127, 0, 0, 127], 127) == [254, 0, 254, 254, 253]


@pytest.mark.parametrize("s", [1, 3, 4, 7, 20, 63, 127])
def test_zrun_tokens_against_run_based_implementation(s):
    """The scan in the oracle against a tokeniser written from the tile's runs; tokens expand
    back to the levels; the histogram is the count of the tiles' tokens."""
    rng = np.random.default_rng([41, s])
    Z = 127 // s
    for p_nz in (0.0, 0.01, 0.2, 0.9, 1.0):
        for n in (1, Z, Z + 1, 3 * Z + 2, 257, 1000):
            q = _random_levels(rng, n, s, p_nz)
            got = oracle.zrun_tokens(q, s).tolist()
            assert got == _zrun_tokens_by_runs(q.tolist(), s)
            assert _zrun_expand(got, s, n) == q.tolist()
    q = _random_levels(rng, 5000, s, 0.1)
    tile = 512
    want = np.zeros(oracle.zrun_symbols(s), np.uint64)
    for e0 in range(0, q.size, tile):
        for t in _zrun_tokens_by_runs(q[e0:e0 + tile].tolist(), s):
            want[t] += 1
    assert np.array_equal(oracle.zrun_histogram(q, s, tile=tile), want)


@pytest.mark.parametrize("s,n,tile,group", [(1, 10000, 4096, 64), (1, 8192, 4096, 1), (3, 5000, 512, 4), (7, 3000, 256, 3),
                                            (127, 900, 128, 2), (4, 100, 4096, 64)])
def test_zrun_stream_is_the_big_integer_model_and_decodes_by_tile(s, n, tile, group):
    """The stream against a big-integer model (token codewords first bit first, LSB-first
    stream, tiles back to back); per-tile bit counts and per-group offsets; every tile decodes
    on its own from its offset."""
    rng = np.random.default_rng([43, s, n])
    q = _random_levels(rng, n, s, 0.15)
    counts = oracle.zrun_histogram(q, s, tile=tile)
    lengths = oracle.huffman_lengths(counts)
    codes = oracle.huffman_codes(lengths)
    assert lengths.tolist() == X.huffman_lengths([int(c) for c in counts])
    stream, tile_bits, group_offsets, bits = oracle.zrun_encode(q, s, lengths, codes, tile=tile, group=group)
    big, pos, want_bits = 0, 0, []
    for e0 in range(0, n, tile):
        begin = pos
        for t in _zrun_tokens_by_runs(q[e0:e0 + tile].tolist(), s):
            for b in range(int(lengths[t]) - 1, -1, -1):
                big |= ((int(codes[t]) >> b) & 1) << pos
                pos += 1
        want_bits.append(pos - begin)
    assert bits == pos and tile_bits.tolist() == want_bits
    nbytes = (bits + 7) // 8
    assert bytes(stream[:nbytes]) == big.to_bytes(nbytes, "little") and not stream[nbytes:].any()
    starts = np.concatenate([[0], np.cumsum(tile_bits.astype(np.int64))])
    assert group_offsets.tolist() == [int(starts[j]) for j in range(0, len(tile_bits), group)] + [bits]
    assert bits <= 8 * oracle.zrun_max_bytes(n, s, tile)
    for t, e0 in enumerate(range(0, n, tile)):
        length = min(tile, n - e0)
        assert np.array_equal(oracle.zrun_decode(stream, int(starts[t]), length, s, lengths, codes), q[e0:e0 + length])


def test_zrun_length_against_the_entropy_bound():
    """Section 4's bound sum_k d_k log2(d/d_k) for memoryless levels: the token code stays within
    2 % of it while at most a third of the levels are non-zero (a per-level code cannot go below
    one bit per element) and within 6 % for dense messages, never exceeds the Huffman guarantee
    (token entropy + one bit per token), and never the capacity the library reserves."""
    rng = np.random.default_rng(47)
    n = 1 << 18
    for s, p_nz in [(1, 0.005), (1, 0.04), (1, 0.3), (1, 0.66), (4, 0.05), (7, 0.3), (127, 0.5)]:
        q = _random_levels(rng, n, s, p_nz)
        bound = oracle.entropy_bound_bits(oracle.level_histogram(q, s))
        counts = oracle.zrun_histogram(q, s)
        lengths = oracle.huffman_lengths(counts)
        _, tile_bits, _, bits = oracle.zrun_encode(q, s, lengths, oracle.huffman_codes(lengths))
        assert bits == int(tile_bits.astype(np.int64).sum())
        tokens = int(counts.sum())
        token_entropy = oracle.entropy_bound_bits(counts)
        assert token_entropy - 1e-6 <= bits < token_entropy + tokens
        assert bits <= 8 * oracle.zrun_max_bytes(n, s)
        if s < 127:
            assert bits <= (1.02 if p_nz <= 0.34 else 1.06) * bound, (s, p_nz, bits / n, bound / n)
        else:                                                  # Z = 1: a per-level Huffman code in effect
            assert bits < bound + n
    # the adversary of the capacity bound: alternating long runs and rare levels
    q = np.zeros(n, np.int8)
    q[::4097] = 1
    counts = oracle.zrun_histogram(q, 1)
    lengths = oracle.huffman_lengths(counts)
    _, _, _, bits = oracle.zrun_encode(q, 1, lengths, oracle.huffman_codes(lengths))
    assert bits <= 8 * oracle.zrun_max_bytes(n, 1)
