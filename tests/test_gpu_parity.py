"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bars: packed codes, scales and Philox words bit-exact; fp32 h and averaged update within 1e-6
relative per bucket (and the number of non-bit-identical values is reported -- expected 0).
"""
import os

import numpy as np
import pytest

import oracle
import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SEED = 0x5EED0123456789AB
# The seeded random tests below run a fixed default set; a wider sweep is a matter of two
# environment variables (e.g. ECQ_RANDOM_SCALE=100 ECQ_RANDOM_SEED=32 pytest -m gpu -k random).
RANDOM_SCALE = int(os.environ.get("ECQ_RANDOM_SCALE", "1"))
RANDOM_SEED = int(os.environ.get("ECQ_RANDOM_SEED", "0"))


@pytest.fixture(scope="module")
def E():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1806_08054_amd as E
    return E


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


class GpuState:
    """Device buffers of one workload, laid out as the C ABI documents."""

    def __init__(self, E, P, N, bucket, s, pad=0, norm="linf", aligned=False):
        self.E, self.P, self.N, self.bucket, self.s, self.norm = E, P, N, bucket, s, norm
        make = E.Shape.aligned if aligned else E.Shape.packed     # 128-byte rows (as benchmarked) or tight
        sh = make(N, P, bucket, s, norm={"linf": 0, "l2": 1}[norm])
        sh.gh_stride += 4 * pad
        sh.code_stride += 4 * pad
        sh.scale_stride += pad
        self.sh = sh
        self.rb = E.row_bytes(N, s)
        self.nb = E.num_buckets(N, bucket)
        self.g = torch.zeros(P, sh.gh_stride, dtype=torch.float32, device="cuda")
        self.h = torch.zeros(P, sh.gh_stride, dtype=torch.float32, device="cuda")
        self.codes = torch.full((P, sh.code_stride), 0xEE, dtype=torch.uint8, device="cuda")
        self.scales = torch.full((P, sh.scale_stride), -7.0, dtype=torch.float32, device="cuda")
        self.out = torch.full((N,), -7.0, dtype=torch.float32, device="cuda")

    def poison(self):
        self.codes.fill_(0xEE)
        self.scales.fill_(-7.0)


def _rel_ok(got, ref, bucket, tol=1e-6):
    """max|d| <= tol * max|ref| per bucket (rows = workers or a single row)."""
    got = np.atleast_2d(got).astype(np.float64)
    ref = np.atleast_2d(ref).astype(np.float64)
    n = ref.shape[1]
    nb = (n + bucket - 1) // bucket
    padn = nb * bucket - n
    d = np.pad(np.abs(got - ref), ((0, 0), (0, padn))).reshape(ref.shape[0], nb, bucket).max(axis=2)
    m = np.pad(np.abs(ref), ((0, 0), (0, padn))).reshape(ref.shape[0], nb, bucket).max(axis=2)
    return bool(np.all(d <= tol * m))


def _compare_step(st, g_np, h_ref, alpha, beta, step, tuning=None, fused=True):
    """Runs one iteration on both sides from the same (g, h); returns oracle outputs.
    h_ref is advanced in place by the oracle; st.h by the library."""
    E = st.E
    P, N = st.P, st.N
    q, scales, _ = oracle.batch_step(g_np, h_ref, st.bucket, st.s, alpha, beta, SEED, step, norm=st.norm)
    codes_ref = oracle.pack_rows(q, st.s)
    st.poison()
    if fused:
        E.ecq_quantize_update_ex(st.sh, st.g, st.h, alpha, beta, SEED, step, st.codes, st.scales, tuning)
    else:
        E.ecq_quantize(st.sh, st.g, st.h, alpha, SEED, step, st.codes, st.scales)
        E.ecq_error_update(st.sh, st.g, st.codes, st.scales, beta, st.h)
    torch.cuda.synchronize()
    codes = st.codes.cpu().numpy()
    sc = st.scales.cpu().numpy()
    hh = st.h.cpu().numpy()
    assert np.array_equal(sc[:, : st.nb].view(np.uint32), scales.view(np.uint32)), "scales differ"
    bad = np.nonzero(codes[:, : st.rb] != codes_ref)
    assert bad[0].size == 0, f"{bad[0].size} code bytes differ, first at worker {bad[0][0]} byte {bad[1][0]}"
    # bytes and floats outside the documented extents are never touched
    assert np.all(codes[:, st.rb:] == 0xEE)
    assert np.all(sc[:, st.nb:] == -7.0)
    assert np.all(hh[:, N:] == 0)
    assert _rel_ok(hh[:, :N], h_ref, st.bucket), "h outside 1e-6"
    nbits = int((hh[:, :N].view(np.uint32) != h_ref.view(np.uint32)).sum())
    assert nbits == 0, f"{nbits} h values not bit-identical"
    return codes_ref, scales


def _aggregate_check(st, codes_ref, scales_ref):
    E = st.E
    ref = oracle.aggregate(codes_ref, scales_ref, st.N, st.bucket, st.s)
    st.out.fill_(-7.0)
    E.ecq_dequant_aggregate(st.sh, st.codes, st.scales, st.out)
    torch.cuda.synchronize()
    out = st.out.cpu().numpy()
    assert _rel_ok(out, ref, st.bucket), "aggregate outside 1e-6"
    nbits = int((out.view(np.uint32) != ref.view(np.uint32)).sum())
    assert nbits == 0, f"{nbits} aggregate values not bit-identical"


def _free_run(E, wl, iters, tuning=None, pad=0, fused=True, gens=None):
    st = GpuState(E, wl.P, wl.N, wl.bucket, wl.s, pad=pad, norm=wl.norm)
    h_ref = np.zeros((wl.P, wl.N), np.float32)
    for t in range(iters):
        g_np = gens(t) if gens else synth.gradients(wl, t).numpy()
        st.g[:, : wl.N] = _dev(g_np)
        codes_ref, scales_ref = _compare_step(st, g_np, h_ref, wl.alpha, wl.beta, t, tuning, fused)
        _aggregate_check(st, codes_ref, scales_ref)
        st.oracle_message = (codes_ref, scales_ref)         # the oracle's own, last iteration
    return st


# ------------------------------------------------------------------ RNG stream -------------

def test_philox_words_bit_exact(E):
    for seed, step, p, i0, count in [(SEED, 0, 0, 0, 4096), (1, (5 << 32) | 3, 31, 1 << 33, 1000),
                                     (2**64 - 1, 2**64 - 1, 65534, 12345, 777)]:
        w = torch.zeros(count, dtype=torch.int32, device="cuda")
        E.ecq_philox_words(seed, step, p, i0, count, w)
        torch.cuda.synchronize()
        got = w.cpu().numpy().view(np.uint32)
        assert np.array_equal(got, oracle.words(seed, step, p, i0, count))


def test_division_routine_matches_ieee_division(E):
    """The per-bucket-reciprocal quotient equals the correctly rounded division for every
    divisor significand: 2^23 divisors x 256 numerators x 2 exponent ranges x 2 forms."""
    bad = torch.full((1,), 77, dtype=torch.int64, device="cuda")
    E.ecq_check_division(256, 0xC0FFEE, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 0


# ------------------------------------------------------------------ the five workloads -----

def test_tiny_free_running(E):
    """Workload 1 in full: 10 free-running iterations, every element compared."""
    wl = synth.WORKLOADS["tiny"]
    _free_run(E, wl, wl.iters)


@pytest.mark.parametrize("name,N,iters", [("linear", 40_000, 6), ("resnet50", 161 * 700 + 40, 6),
                                          ("alexnet", 100_000 + 808, 4), ("vgg16", 8192 * 5 + 2856, 4)])
def test_workload_shapes_reduced(E, name, N, iters):
    """Workloads 2-5 with their bucket, s, alpha, beta and value distribution at a length the
    oracle covers in full (several buckets plus the same ragged tail), free-running."""
    wl = synth.scaled(synth.WORKLOADS[name], N=N, P=min(synth.WORKLOADS[name].P, 4))
    _free_run(E, wl, iters)


# ------------------------------------------------------------------ shapes and edges -------

@pytest.mark.parametrize("s", [1, 2, 3, 4, 7, 8, 15, 16, 31, 33, 64, 127])
@pytest.mark.parametrize("bucket", [8, 64, 512, 1000])
def test_levels_and_buckets(E, s, bucket):
    """Every code width r = 2..8 against every kernel route (lane groups, wave teams, two-pass),
    N not a multiple of 4, 8 or the bucket, padded strides."""
    wl = synth.Workload("edge", P=3, N=2 * 1024 + 8 * 37 + 3, bucket=bucket, s=s, alpha=0.5, beta=0.75,
                        iters=2, kind="normal", data_seed=s * 131 + bucket)
    _free_run(E, wl, 2, pad=3)
    _free_run(E, wl, 2, pad=3, fused=False)                    # ecq_quantize, then ecq_error_update


@pytest.mark.parametrize("bucket", [16, 24, 32, 40, 96, 128, 248, 256, 264, 2048, 4096, 8192, 16384, 32768, 40000,
                                    65536, 100_000, 1 << 20, 56, 136, 200])
def test_bucket_routes(E, bucket):
    """Every mapping of buckets to lanes: lane groups (powers of two up to 128), teams of waves
    (256 ... 32768), and the two-pass route with its two first passes (other buckets below 256;
    buckets beyond 32768, cut into several pieces)."""
    wl = synth.Workload("edge", P=2, N=3 * bucket + bucket // 2 + 5, bucket=bucket, s=3, alpha=1.0, beta=0.9,
                        iters=2, kind="normal", data_seed=bucket)
    _free_run(E, wl, 2)


@pytest.mark.parametrize("N,s", [(700_001, 1), (2_500_000, 4)])
def test_one_norm_per_row(E, N, s):
    """Eq. (8) as first stated, without buckets: the bucket is the whole row (one norm per
    worker), here as the smallest multiple of 8 that holds the row."""
    bucket = (N + 7) // 8 * 8
    wl = synth.Workload("edge", P=3, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=2, kind="student_t",
                        data_seed=N)
    _free_run(E, wl, 2)
    _free_run(E, wl, 2, fused=False)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 7, 8, 9, 255, 256, 257, 511, 513])
@pytest.mark.parametrize("s", [1, 3, 7])
def test_tiny_lengths(E, N, s):
    wl = synth.Workload("edge", P=2, N=N, bucket=512, s=s, alpha=1.0, beta=1.0, iters=2, kind="normal",
                        data_seed=N)
    _free_run(E, wl, 2)
    _free_run(E, wl, 2, fused=False)
    wl = synth.scaled(wl, bucket=8)
    _free_run(E, wl, 2)


def _random_workloads(count, seed):
    rng = np.random.default_rng(seed)
    levels = [1, 1, 1, 2, 3, 4, 4, 7, 8, 15, 16, 31, 40, 127]
    out = []
    for i in range(count):
        N = int(rng.choice([rng.integers(1, 300), rng.integers(300, 9000), rng.integers(9000, 90_000)]))
        kind = rng.integers(4)
        if kind == 0:
            bucket = 8 * int(rng.integers(1, 32))                       # lane groups
        elif kind == 1:
            bucket = 8 * int(rng.integers(32, 4097))                    # teams of waves
        elif kind == 2:
            bucket = 8 * int(rng.integers(4097, 12_000))                # two passes
        else:
            bucket = (N + 7) // 8 * 8 + 8 * int(rng.integers(0, 3))     # one norm per row
        out.append(synth.Workload(f"random{i}", P=int(rng.integers(1, 10)), N=N, bucket=bucket,
                                  s=int(rng.choice(levels)), alpha=float(np.float32(rng.uniform(0, 1.2))),
                                  beta=float(np.float32(rng.uniform(0, 1))), iters=2,
                                  kind=str(rng.choice(["normal", "student_t"])), data_seed=1000 + i,
                                  norm=str(rng.choice(["linf", "l2"]))))
    return out


@pytest.mark.parametrize("wl", _random_workloads(48 * RANDOM_SCALE, seed=2024 + RANDOM_SEED), ids=lambda w: f"{w.name}-P{w.P}-N{w.N}-b{w.bucket}-s{w.s}-{w.norm}")
def test_random_shapes(E, wl):
    """Seeded random corners of the configuration space: worker counts, lengths, every class of
    bucket size, levels, both norms, alpha and beta; fused and unfused entry points."""
    _free_run(E, wl, 2, pad=int(wl.N % 3))
    _free_run(E, wl, 2, fused=False)


# ------------------------------------------------------------------ l_2 scaling ------------

@pytest.mark.parametrize("s", [1, 4, 7])
@pytest.mark.parametrize("bucket", [8, 24, 32, 40, 96, 128, 136, 248, 256, 512, 1000, 1024, 4096, 8192, 16384, 32768])
def test_l2_norm_buckets(E, s, bucket):
    """l_2 scaling (tree sum of squares by index, one square root) on every single-pass route,
    ragged tails included; the paper's own setting is l_2 with s = 4 (Section 6)."""
    wl = synth.Workload("edge", P=2, N=2 * bucket + bucket // 2 + 3 + 1024, bucket=bucket, s=s, alpha=0.2,
                        beta=0.9, iters=3, kind="normal", data_seed=bucket + s, norm="l2")
    _free_run(E, wl, 3)


@pytest.mark.parametrize("bucket,N,s", [(40_000, 140_003, 4), (65_536, 200_000, 1), (100_000, 350_001, 7),
                                        (1 << 20, (1 << 20) + 8192 * 3 + 5, 4)])
def test_l2_norm_long_buckets(E, bucket, N, s):
    """l_2 scaling of buckets beyond 32768 elements: sums of squares of 8192-element pieces, then
    the tree over the pieces (two passes); several buckets with a short last one."""
    wl = synth.Workload("edge", P=2, N=N, bucket=bucket, s=s, alpha=0.2, beta=0.9, iters=2, kind="normal",
                        data_seed=bucket + s, norm="l2")
    _free_run(E, wl, 2)
    _free_run(E, wl, 2, fused=False)


@pytest.mark.parametrize("N", [5, 100, 200, 5000, 40_000, 700_001])
@pytest.mark.parametrize("norm", ["linf", "l2"])
def test_one_norm_per_row_any_length(E, N, norm):
    """The bucket holds the whole row, for rows of every size class (the library then takes the
    tightest bucket one of its mappings accepts); both norms; a bucket far beyond the row."""
    for bucket in ((N + 7) // 8 * 8, 1 << 24):
        wl = synth.Workload("edge", P=2, N=N, bucket=bucket, s=4, alpha=0.2, beta=0.9, iters=2, kind="normal",
                            data_seed=N, norm=norm)
        _free_run(E, wl, 2)


def test_l2_geometry_invariance_and_unfused(E):
    wl = synth.Workload("edge", P=2, N=5 * 2048 + 1000, bucket=2048, s=4, alpha=0.2, beta=0.9, iters=2,
                        kind="normal", data_seed=77, norm="l2")
    for path, waves, threads in [(1, 1, 64), (1, 1, 256), (1, 2, 256), (1, 4, 256), (1, 8, 512), (1, 16, 1024)]:
        _free_run(E, wl, 2, tuning=E.Tuning(path, waves, threads, 0))
    _free_run(E, wl, 2, fused=False)


def test_l2_degenerate(E):
    """Zero buckets, sparse buckets (one non-zero), equal magnitudes."""
    P, N, bucket = 3, 4096, 512
    rng = np.random.default_rng(2)

    def gens(t):
        g = rng.standard_normal((P, N)).astype(np.float32)
        g[0] = 0.0
        g[1, :] = 0.0
        g[1, ::512] = 2.5
        g[2, :1024] = np.float32(0.125) * np.sign(g[2, :1024])
        return g

    for s in (1, 4):
        wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=3,
                            kind="normal", norm="l2")
        _free_run(E, wl, 3, gens=gens)


@pytest.mark.parametrize("bucket", [16, 96, 512, 2048, 16384, 65536])
def test_l2_squares_that_underflow(E, bucket):
    """l_2 scaling where fl(v_i^2) is denormal or 0: buckets whose only non-zero element lies in
    1e-23..1e-19 (the computed norm can fall below the element: level s, the end of the grid),
    a few tiny neighbours, and buckets whose squares all round to 0 (norm 0: every level 0).
    Every bucket route, s = 1, 4, 127."""
    P = 3
    N = max(4 * bucket + 40, 4096)
    rng = np.random.default_rng(bucket)

    def gens(t):
        g = np.zeros((P, N), np.float32)
        for k in range(0, N, bucket):
            width = min(bucket, N - k)
            g[0, k + int(rng.integers(width))] = np.float32(rng.choice([-1.0, 1.0]) * 10.0 ** rng.uniform(-23, -19))
            at = k + rng.integers(width, size=4)
            g[1, at] = (10.0 ** rng.uniform(-24, -19, 4)).astype(np.float32)
        g[2] = (rng.standard_normal(N) * 1e-30).astype(np.float32)      # every square rounds to 0
        g[2, : N // 2] = rng.standard_normal(N // 2).astype(np.float32) * np.float32(1e-21)
        return g

    for s in (1, 4, 127):
        wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=2,
                            kind="normal", norm="l2")
        _free_run(E, wl, 2, gens=gens)
        _free_run(E, wl, 1, gens=gens, fused=False)


@pytest.mark.parametrize("s", [1, 2, 5, 6, 100])
def test_codes_beyond_the_grid_decode_as_level_zero(E, s):
    """A message that holds codes above 2s (none written by the library does): the error update
    and the aggregation both read them as level 0, i.e. as the same message with those codes
    replaced by s, which the oracle decodes."""
    P, N, bucket = 3, 3 * 1024 + 72, 256
    r = E.code_bits(s)
    if (1 << r) == 2 * s + 1:
        pytest.skip("every r-bit code is on the grid")
    rng = np.random.default_rng(s)
    st = GpuState(E, P, N, bucket, s)
    c = rng.integers(0, 1 << r, (P, N))
    clean = np.where(c > 2 * s, s, c)
    g_np = rng.standard_normal((P, N)).astype(np.float32)
    h_np = rng.standard_normal((P, N)).astype(np.float32)
    scales = np.abs(rng.standard_normal((P, st.nb))).astype(np.float32)
    # (codes beyond the grid are not levels the oracle's packer takes: lay the fields out as the
    # little-endian big integer they are)
    from tests import exact_ref as X
    dirty_bytes = np.stack([np.frombuffer(X.pack([int(v) - s for v in row], s), np.uint8) for row in c])
    clean_bytes = oracle.pack_rows((clean - s).astype(np.int8), s)
    st.g[:, :N] = _dev(g_np)
    st.h[:, :N] = _dev(h_np)
    st.codes[:, : st.rb] = _dev(dirty_bytes)
    st.scales[:, : st.nb] = _dev(scales)
    E.ecq_error_update(st.sh, st.g, st.codes, st.scales, 0.9, st.h)
    E.ecq_dequant_aggregate(st.sh, st.codes, st.scales, st.out)
    torch.cuda.synchronize()
    h_ref = h_np.copy()
    for p in range(P):
        oracle.error_update_row(g_np[p], clean_bytes[p], scales[p], bucket, s, 0.9, h_ref[p])
    assert np.array_equal(st.h.cpu().numpy()[:, :N].view(np.uint32), h_ref.view(np.uint32))
    ref = oracle.aggregate(clean_bytes, scales, N, bucket, s)
    assert np.array_equal(st.out.cpu().numpy().view(np.uint32), ref.view(np.uint32))


def test_launch_geometry_invariance(E):
    """Same bits for every mapping of buckets to lanes."""
    wl = synth.Workload("edge", P=2, N=5 * 2048 + 1000, bucket=2048, s=3, alpha=1.0, beta=0.9, iters=2,
                        kind="normal", data_seed=99)
    for path, waves, threads in [(1, 1, 64), (1, 1, 256), (1, 2, 256), (1, 4, 256), (1, 8, 512),
                                 (1, 8, 1024), (1, 16, 1024), (2, 0, 0)]:
        _free_run(E, wl, 2, tuning=E.Tuning(path, waves, threads, 0))
    # The two-pass route on request for buckets below 256 elements (segmented wave maximum).
    for bucket in (8, 40, 96, 248):
        small = synth.scaled(wl, bucket=bucket)
        _free_run(E, small, 2, tuning=E.Tuning(2, 0, 0, 0))


def test_unfused_equals_fused(E):
    wl = synth.Workload("edge", P=3, N=7000, bucket=512, s=7, alpha=0.3, beta=0.9, iters=3, kind="normal",
                        data_seed=5)
    _free_run(E, wl, 3, fused=False)


@pytest.mark.parametrize("bucket,s", [(512, 1), (512, 7), (1024, 3), (2048, 1), (8192, 4), (32768, 1)])
def test_unfused_whole_blocks(E, bucket, s):
    """ecq_quantize on rows long enough that most blocks hold only complete buckets (the route
    without bounds checks) followed by a ragged rest, then ecq_error_update."""
    wl = synth.Workload("edge", P=2, N=5 * max(4096, bucket) + bucket // 2 + 12, bucket=bucket, s=s, alpha=1.0,
                        beta=0.9, iters=2, kind="normal", data_seed=bucket + s)
    _free_run(E, wl, 2, fused=False)
    _free_run(E, wl, 2, fused=True)


def test_degenerate_values(E):
    """All-zero buckets, a zero row, negative zeros, denormals, repeated maxima, huge range."""
    P, N, bucket = 4, 4096, 512
    rng = np.random.default_rng(0)

    def gens(t):
        g = rng.standard_normal((P, N)).astype(np.float32)
        g[0] = 0.0
        g[1, 512:1024] = 0.0
        g[1, 1024:1536] = -0.0
        g[2] *= 1e-41                                   # denormal inputs and denormal norms
        g[3, :100] = np.float32(3.0) * np.sign(g[3, :100])   # many elements attain the norm
        g[3, 2048:2560] *= (10.0 ** rng.integers(-30, 30, 512)).astype(np.float32)
        return g

    for s in (1, 3, 127):
        wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=3,
                            kind="normal")
        _free_run(E, wl, 3, gens=gens)


def test_teacher_forced_and_alpha_zero(E):
    """The oracle's h is fed to the library every iteration; alpha = 0 (QSGD) ignores h."""
    wl = synth.Workload("edge", P=2, N=6000, bucket=1024, s=4, alpha=0.0, beta=1.0, iters=3, kind="normal",
                        data_seed=3)
    st = GpuState(E, wl.P, wl.N, wl.bucket, wl.s)
    h_ref = np.random.default_rng(1).standard_normal((wl.P, wl.N)).astype(np.float32)
    for t in range(3):
        g_np = synth.gradients(wl, t).numpy()
        st.g[:, : wl.N] = _dev(g_np)
        st.h[:, : wl.N] = _dev(h_ref)
        _compare_step(st, g_np, h_ref, wl.alpha, wl.beta, t)


@pytest.mark.parametrize("P,s,bucket", [(1, 1, 512), (9, 1, 512), (33, 1, 1024), (7, 3, 2048), (12, 7, 512),
                                        (33, 127, 1024), (6, 1, 16), (10, 5, 48)])
def test_aggregate_worker_counts(E, P, s, bucket):
    """Eq. (4) with worker counts around the kernel's unrolling (also not powers of two, so the
    final division is a true division), per-lane and per-wave norms, several full runs of 1024
    outputs plus a ragged tail."""
    wl = synth.Workload("edge", P=P, N=5 * 1024 + 8 * 13 + 5, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=2,
                        kind="student_t", data_seed=P * 1000 + s)
    _free_run(E, wl, 2)


@pytest.mark.parametrize("P,s,bucket", [(13, 1, 512), (16, 1, 8192), (13, 7, 2048), (12, 5, 496), (34, 3, 1000),
                                        (18, 31, 4096)])
def test_aggregate_many_workers_long_rows(E, P, s, bucket):
    """Twelve or more workers on rows of more than 2^23 elements (2-, 3-, 4- and 6-bit codes):
    per-lane and per-wave norms, worker counts that are not a multiple of the batch of four,
    a ragged last run, and the model update fused into the aggregation.  The last two cases
    hold more than 96 MB of codes in all, the size from which the codes are streamed past the
    cache, at code widths the benchmark's workloads do not have."""
    N = (1 << 23) + 3 * 1024 + 500
    wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=1, kind="student_t",
                        data_seed=P + s)
    st = _free_run(E, wl, 1)
    codes_ref, scales_ref = st.oracle_message
    gavg = oracle.aggregate(codes_ref, scales_ref, N, bucket, s)
    w0 = np.random.default_rng(P).standard_normal(N).astype(np.float32)
    eta = float(np.float32(0.05))
    w_ref = oracle.sgd_step(w0.copy(), gavg, eta)
    w = _dev(w0)
    E.ecq_dequant_aggregate_sgd(st.sh, st.codes, st.scales, eta, w, None)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


def test_calibration_gather(E):
    """The aggregation-pattern calibration kernel reads the rows it is given and nothing else:
    every whole run of 1024 outputs holds the sum of the P rows' code words of its lane."""
    P, N, s = 5, 3 * 1024 + 100, 7
    sh = E.Shape.packed(N, P, 512, s)
    rng = np.random.default_rng(1)
    codes_np = rng.integers(0, 256, size=(P, sh.code_stride), dtype=np.uint8)
    out = torch.full((N,), -3.0, device="cuda")
    E.ecq_calib_gather(sh, _dev(codes_np), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    words = codes_np[:, : 3 * 1024 // 2].copy().view(np.uint32).reshape(P, 3, 64, 2)   # r = 4: 8 bytes per lane
    want = words.astype(np.uint64).sum(axis=(0, 3)) & 0xFFFFFFFF                       # [run][lane]
    for run in range(3):
        block = got[run * 1024:(run + 1) * 1024].reshape(4, 64, 4)
        assert np.array_equal(block, np.broadcast_to(want[run].astype(np.float32)[None, :, None], (4, 64, 4)))
    assert np.all(got[3 * 1024:] == -3.0)


# ------------------------------------------------------------------ model update -----------

@pytest.mark.parametrize("s,bucket,N,P", [(1, 512, 5000, 4), (4, 1024, 3 * 1024 + 77, 3), (3, 24, 1000, 5),
                                          (7, 8192, 4_200_000, 2)])
def test_aggregate_sgd_step(E, s, bucket, N, P):
    """ecq_dequant_aggregate_sgd: the averaged gradient and w <- w - eta * g~ in one kernel,
    with and without storing the average."""
    rng = np.random.default_rng(N)
    wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=1, kind="normal",
                        data_seed=N)
    st = GpuState(E, P, N, bucket, s)
    g_np = synth.gradients(wl, 0).numpy()
    st.g[:, :N] = _dev(g_np)
    h_ref = np.zeros((P, N), np.float32)
    codes_ref, scales_ref = _compare_step(st, g_np, h_ref, wl.alpha, wl.beta, 0)
    gavg = oracle.aggregate(codes_ref, scales_ref, N, bucket, s)
    w0 = rng.standard_normal(N).astype(np.float32)
    eta = float(np.float32(0.02))
    w_ref = oracle.sgd_step(w0.copy(), gavg, eta)
    for keep_avg in (True, False):
        w = _dev(w0)
        st.out.fill_(-7.0)
        E.ecq_dequant_aggregate_sgd(st.sh, st.codes, st.scales, eta, w, st.out if keep_avg else None)
        torch.cuda.synchronize()
        assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))
        out = st.out.cpu().numpy()
        if keep_avg:
            assert np.array_equal(out.view(np.uint32), gavg.view(np.uint32))
        else:
            assert np.all(out == -7.0)


def test_closed_loop_least_squares(E):
    """Algorithm 1 end to end on synthetic least squares (the setting of Section 6.1: l_2
    scaling, s = 4, alpha = 0.2, beta = 0.9, eta = 0.02): gradients from the current model,
    quantise + error update, aggregate + model update, for 150 iterations.  The library's model
    replica must follow the oracle's bit for bit, and the loss must fall."""
    d, P, mb, s, iters = 2048, 4, 32, 4, 150
    alpha, beta, eta = float(np.float32(0.2)), float(np.float32(0.9)), float(np.float32(0.02))
    gen = torch.Generator(device="cuda").manual_seed(5)
    X = torch.randn(P, 2000, d, generator=gen, device="cuda")
    wstar = torch.randn(d, generator=gen, device="cuda")
    y = X @ wstar + 0.1 * torch.randn(P, 2000, generator=gen, device="cuda")
    st = GpuState(E, P, d, 512, s, norm="l2")
    w = torch.zeros(d, device="cuda")
    w_ref = np.zeros(d, np.float32)
    h_ref = np.zeros((P, d), np.float32)
    losses = []
    for t in range(iters):
        idx = torch.randint(0, 2000, (P, mb), generator=gen, device="cuda")
        Xb = torch.gather(X, 1, idx[:, :, None].expand(P, mb, d))
        yb = torch.gather(y, 1, idx)
        w_in = _dev(w_ref)                                     # gradients come from the oracle's model
        resid = torch.einsum("pmd,d->pm", Xb, w_in) - yb
        st.g[:, :d] = torch.einsum("pmd,pm->pd", Xb, resid) / mb
        losses.append(float((resid ** 2).mean()))
        g_np = st.g[:, :d].cpu().numpy()
        E.ecq_quantize_update(st.sh, st.g, st.h, alpha, beta, SEED, t, st.codes, st.scales)
        E.ecq_dequant_aggregate_sgd(st.sh, st.codes, st.scales, eta, w, None)
        q, sc, _ = oracle.batch_step(g_np, h_ref, 512, s, alpha, beta, SEED, t, norm="l2")
        oracle.sgd_step(w_ref, oracle.aggregate(oracle.pack_rows(q, s), sc, d, 512, s), eta)
        torch.cuda.synchronize()
        assert np.array_equal(w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32)), f"model differs at step {t}"
    assert np.array_equal(st.h[:, :d].cpu().numpy().view(np.uint32), h_ref.view(np.uint32))
    assert np.mean(losses[-10:]) < 0.05 * np.mean(losses[:3])


# ------------------------------------------------------------------ entropy-coded length ---

@pytest.mark.parametrize("s,bucket,N,P", [(1, 512, 70_001, 3), (3, 64, 5000, 2), (7, 2048, 300_000, 4),
                                          (127, 8, 9, 2), (1, 512, 1_200_003, 2)])
def test_level_histogram(E, s, bucket, N, P):
    """Integer counts per level, bit-exact; ragged tails (pad bits are not counted); the
    library's entropy bound equals the oracle's."""
    wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=1, kind="student_t",
                        data_seed=N)
    st = GpuState(E, P, N, bucket, s)
    g_np = synth.gradients(wl, 0).numpy()
    st.g[:, :N] = _dev(g_np)
    h_ref = np.zeros((P, N), np.float32)
    q, _, _ = oracle.batch_step(g_np, h_ref.copy(), bucket, s, wl.alpha, wl.beta, SEED, 0)
    _compare_step(st, g_np, h_ref, wl.alpha, wl.beta, 0)
    stride = 2 * s + 1 + 3
    counts = torch.full((P, stride), 12345, dtype=torch.int64, device="cuda")
    E.ecq_level_histogram(st.sh, st.codes, counts, stride)
    torch.cuda.synchronize()
    got = counts.cpu().numpy()
    assert np.all(got[:, 2 * s + 1:] == 12345)
    for p in range(P):
        ref = oracle.level_histogram(q[p], s)
        assert np.array_equal(got[p, : 2 * s + 1].astype(np.uint64), ref)
        bits = E.ecq_entropy_bound_bits(list(got[p, : 2 * s + 1]))
        assert abs(bits - oracle.entropy_bound_bits(ref)) <= 1e-9 * max(bits, 1.0)


# ------------------------------------------------------------------ Huffman coding ---------

def _huffman_roundtrip(E, sh, P, N, s, codes_dev, q_rows, poison_stream=0xEE):
    """Histogram -> code construction -> encode -> decode on the GPU, every product compared
    bit for bit with the oracle run on the same levels q_rows [P][N]."""
    bins = 2 * s + 1
    stride = bins + 2
    tiles = E.huffman_num_tiles(N)
    assert tiles == (N + oracle.HUFFMAN_TILE - 1) // oracle.HUFFMAN_TILE
    rb = E.row_bytes(N, s)
    counts = torch.full((P, stride), 4242, dtype=torch.int64, device="cuda")
    lengths = torch.full((P, stride), 0xEE, dtype=torch.uint8, device="cuda")
    codewords = torch.full((P, stride), -1, dtype=torch.int64, device="cuda")
    stream_stride = (rb + 3) // 4 * 4 + 8
    streams = torch.full((P, stream_stride), poison_stream, dtype=torch.uint8, device="cuda")
    offs = torch.full((P, tiles + 3), -1, dtype=torch.int64, device="cuda")
    E.ecq_level_histogram(sh, codes_dev, counts, stride)
    E.ecq_huffman_build(P, s, counts, stride, lengths, codewords)
    E.ecq_huffman_encode(sh, codes_dev, lengths, codewords, stride, streams, stream_stride, offs, tiles + 3)
    back = torch.full_like(codes_dev, 0x77)
    E.ecq_huffman_decode(sh, streams, stream_stride, offs, tiles + 3, lengths, codewords, stride, back)
    torch.cuda.synchronize()
    len_np, cw_np = lengths.cpu().numpy(), codewords.cpu().numpy().view(np.uint64)
    str_np, off_np = streams.cpu().numpy(), offs.cpu().numpy().view(np.uint64)
    cnt_np = counts.cpu().numpy()
    total_bits = 0
    for p in range(P):
        ref_counts = oracle.level_histogram(q_rows[p], s)
        assert np.array_equal(cnt_np[p, :bins].astype(np.uint64), ref_counts)
        ref_len = oracle.huffman_lengths(ref_counts)
        ref_cw = oracle.huffman_codes(ref_len)
        assert np.array_equal(len_np[p, :bins], ref_len), (p, len_np[p, :bins], ref_len)
        assert np.array_equal(cw_np[p, :bins], ref_cw)
        assert np.all(len_np[p, bins:] == 0xEE) and np.all(cw_np[p, bins:] == np.uint64(2**64 - 1))
        ref_stream, ref_offs, bits = oracle.huffman_encode(q_rows[p], s, ref_len, ref_cw)
        assert np.array_equal(off_np[p, : tiles + 1], ref_offs)
        assert np.all(off_np[p, tiles + 1:] == np.uint64(2**64 - 1))
        nbytes = (bits + 7) // 8
        written = (nbytes + 3) // 4 * 4
        assert np.array_equal(str_np[p, :nbytes], ref_stream[:nbytes]), p
        assert np.all(str_np[p, nbytes:written] == 0)
        assert np.all(str_np[p, written:] == poison_stream)
        assert bits <= N * E.code_bits(s)
        total_bits += bits
    back_np = back.cpu().numpy()
    orig = codes_dev.cpu().numpy()
    assert np.array_equal(back_np[:, :rb], orig[:, :rb])
    assert np.all(back_np[:, rb:] == 0x77)
    return total_bits


@pytest.mark.parametrize("s,bucket,N,P,kind", [(1, 512, 70_001, 3, "student_t"), (3, 64, 5000, 2, "normal"),
                                               (7, 2048, 300_000, 4, "student_t"), (127, 8, 9, 2, "normal"),
                                               (127, 512, 150_000, 2, "student_t"), (1, 512, 1_200_003, 2, "normal"),
                                               (3, 1024, 1025, 1, "normal"), (1, 8, 1024, 1, "normal"),
                                               (4, 512, 4_200_000, 2, "normal"),
                                               # whole runs of 16 tiles, whole steps, one element more
                                               (1, 512, 16_384, 2, "normal"), (1, 512, 16_385, 1, "student_t"),
                                               (1, 512, 4_096 + 16, 2, "normal"), (1, 512, 65_536 + 3, 3, "normal"),
                                               (7, 512, 32_768 + 1_023, 2, "normal"),
                                               # 5-, 6- and 7-bit codes: two tiles, then one tile per step
                                               (9, 512, 40_000, 2, "normal"), (20, 512, 33_000, 2, "student_t"),
                                               (40, 512, 20_000, 1, "normal")])
def test_huffman_matches_oracle(E, s, bucket, N, P, kind):
    """Section 4's Huffman encoding of a quantised message: counts, codeword lengths,
    canonical codewords, tile offsets and the stream itself bit-exact against the oracle;
    decoding gives back the fixed-length message."""
    wl = synth.Workload("edge", P=P, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=1, kind=kind,
                        data_seed=N + s)
    st = GpuState(E, P, N, bucket, s)
    g_np = synth.gradients(wl, 0).numpy()
    st.g[:, :N] = _dev(g_np)
    h_ref = np.zeros((P, N), np.float32)
    q, _, _ = oracle.batch_step(g_np, h_ref.copy(), bucket, s, wl.alpha, wl.beta, SEED, 0)
    _compare_step(st, g_np, h_ref, wl.alpha, wl.beta, 0)
    bits = _huffman_roundtrip(E, st.sh, P, N, s, st.codes, q)
    assert bits < P * N * E.code_bits(s)


@pytest.mark.parametrize("case", range(1000 * RANDOM_SEED, 1000 * RANDOM_SEED + 24 * RANDOM_SCALE))
def test_huffman_random_messages(E, case):
    """Seeded random messages: level distributions from nearly flat to one dominant level, any
    number of unused levels, lengths around tile, step and run boundaries."""
    rng = np.random.default_rng(7000 + case)
    s = int(rng.choice([1, 1, 2, 3, 4, 7, 8, 15, 16, 31, 63, 127]))
    P = int(rng.integers(1, 4))
    N = int(rng.choice([rng.integers(1, 2000), rng.integers(2000, 20_000), 16_384 * int(rng.integers(1, 4)) + int(rng.integers(-3, 4)),
                        rng.integers(20_000, 150_000)]))
    q = np.zeros((P, N), np.int8)
    for p in range(P):
        w = rng.random(2 * s + 1) ** float(rng.choice([1.0, 4.0, 16.0, 64.0]))
        w[rng.random(2 * s + 1) < 0.3] = 0.0                    # unused levels
        w[s] += float(rng.choice([0.0, 1.0, 20.0]))             # level 0 often dominates
        if w.sum() == 0.0:
            w[s] = 1.0
        q[p] = rng.choice(np.arange(-s, s + 1), size=N, p=w / w.sum()).astype(np.int8)
    sh = E.Shape.packed(N, P, 512, s)
    packed = oracle.pack_rows(q, s)
    codes = _dev(np.pad(packed, ((0, 0), (0, sh.code_stride - packed.shape[1]))))
    _huffman_roundtrip(E, sh, P, N, s, codes, q)


def test_huffman_degenerate_rows(E):
    """A message with a single occupied level (all-zero gradient: every level 0) costs one bit
    per element; a two-level message costs one bit per element too."""
    P, N, s = 2, 5000, 3
    sh = E.Shape.packed(N, P, 512, s)
    q = np.zeros((P, N), np.int8)
    q[1, ::3] = -2
    codes = _dev(np.pad(oracle.pack_rows(q, s), ((0, 0), (0, sh.code_stride - E.row_bytes(N, s)))))
    assert _huffman_roundtrip(E, sh, P, N, s, codes, q) == 2 * N


@pytest.mark.parametrize("s", [17, 7, 3])
def test_huffman_long_codewords(E, s):
    """Level counts that follow the Fibonacci numbers give the deepest possible tree: with 35
    levels (s = 17) the rarest codeword is 34 bits long, beyond one 32-bit stream word; with 15
    levels (s = 7, 4-bit codes) two codewords together can exceed the 24 bits a pair-table
    entry holds; with 7 levels every pair fits."""
    fib = [1, 1]
    while len(fib) < 2 * s + 1:
        fib.append(fib[-1] + fib[-2])
    rng = np.random.default_rng(17)
    levels = rng.permutation(2 * s + 1) - s
    q = np.repeat(levels.astype(np.int8), fib)
    q = np.tile(q, max(1, 40_000 // q.size))                  # the same proportions, several tiles
    rng.shuffle(q)
    N = q.size
    assert int(oracle.huffman_lengths(oracle.level_histogram(q, s)).max()) == 2 * s
    sh = E.Shape.packed(N, 1, 512, s)
    packed = oracle.pack_rows(q[None, :], s)
    codes = _dev(np.pad(packed, ((0, 0), (0, sh.code_stride - packed.shape[1]))))
    _huffman_roundtrip(E, sh, 1, N, s, codes, q[None, :])


def test_huffman_decodes_an_oracle_stream(E):
    """The decoder reads a stream it did not write: encoded by the oracle, decoded on the GPU."""
    P, N, s = 1, 40_000, 7
    rng = np.random.default_rng(3)
    q = np.clip(np.round(rng.standard_normal(N) * 1.5), -s, s).astype(np.int8)
    counts = oracle.level_histogram(q, s)
    lengths = oracle.huffman_lengths(counts)
    cw = oracle.huffman_codes(lengths)
    stream, offs, bits = oracle.huffman_encode(q, s, lengths, cw)
    sh = E.Shape.packed(N, P, 512, s)
    tiles = E.huffman_num_tiles(N)
    back = torch.zeros(P, sh.code_stride, dtype=torch.uint8, device="cuda")
    E.ecq_huffman_decode(sh, _dev(stream[None, :]), stream.size, _dev(offs.view(np.int64)[None, :]), tiles + 1,
                         _dev(lengths[None, :]), _dev(cw.view(np.int64)[None, :]), 2 * s + 1, back)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy()[0, : E.row_bytes(N, s)], oracle.pack_rows(q[None, :], s)[0])


# ------------------------------------------------------------------ HIP graph ---------------

def test_step_under_graph_capture(E):
    """The library only launches kernels on the caller's stream, so a whole step (fused
    quantise + update, then aggregate) can be captured into a HIP graph.  Every replay, with
    eager work and synchronisations in between, must reproduce the eager step bit for bit
    (the step number is a launch argument, so a replay repeats the captured iteration)."""
    wl = synth.Workload("edge", P=4, N=300_000 + 40, bucket=512, s=1, alpha=1.0, beta=0.9, iters=1,
                        kind="normal", data_seed=11)
    st = GpuState(E, wl.P, wl.N, wl.bucket, wl.s, aligned=True)
    g_np = synth.gradients(wl, 0).numpy()
    st.g[:, : wl.N] = _dev(g_np)
    h0 = torch.randn_like(st.h) * 0.01
    st.h.copy_(h0)
    E.ecq_quantize_update(st.sh, st.g, st.h, wl.alpha, wl.beta, SEED, 5, st.codes, st.scales)
    E.ecq_dequant_aggregate(st.sh, st.codes, st.scales, st.out)
    torch.cuda.synchronize()
    want = [x.clone() for x in (st.h, st.codes, st.scales, st.out)]

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    st.h.copy_(h0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            E.ecq_quantize_update(st.sh, st.g, st.h, wl.alpha, wl.beta, SEED, 5, st.codes, st.scales)
            E.ecq_dequant_aggregate(st.sh, st.codes, st.scales, st.out)
    for replay in range(4):
        st.h.copy_(h0)                                         # eager work between replays
        st.poison()
        st.out.fill_(-7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip((st.h, st.codes, st.scales, st.out), want):
            assert torch.equal(got, ref), f"replay {replay} differs from the eager step"


# ------------------------------------------------------------------ boundary errors --------

def test_argument_errors_leave_outputs_untouched(E):
    st = GpuState(E, 2, 1024, 512, 1)
    lib = E.lib()
    import ctypes as C

    def call(sh, g=st.g, h=st.h, codes=st.codes, scales=st.scales, alpha=1.0, beta=1.0):
        ptr = lambda t: None if t is None else C.c_void_p(t.data_ptr() if hasattr(t, "data_ptr") else t)
        return lib.ecq_quantize_update(C.byref(sh), ptr(g), ptr(h), alpha, beta, 1, 0, ptr(codes), ptr(scales), None)

    def shape(**kw):
        sh = E.Shape.packed(1024, 2, 512, 1)
        for k, v in kw.items():
            setattr(sh, k, v)
        return sh

    assert call(shape(), g=None) == -1
    assert call(shape(n=0)) == -2 and call(shape(workers=0)) == -2 and call(shape(workers=70000)) == -2
    assert call(shape(s=0)) == -3 and call(shape(s=128)) == -3
    assert call(shape(bucket=0)) == -4 and call(shape(bucket=12)) == -4
    assert call(shape(gh_stride=1000)) == -5 and call(shape(gh_stride=1026)) == -5
    assert call(shape(code_stride=100)) == -5 and call(shape(scale_stride=1)) == -5
    assert call(shape(), g=st.g.data_ptr() + 4) == -6
    assert call(shape(), alpha=-1.0) == -8 and call(shape(), beta=1.5) == -8
    assert call(shape(), alpha=float("nan")) == -8 and call(shape(norm=7)) == -8
    torch.cuda.synchronize()
    assert bool((st.codes == 0xEE).all()) and bool((st.scales == -7.0).all()) and not bool(st.h.any())
    assert call(shape()) == 0
    torch.cuda.synchronize()
