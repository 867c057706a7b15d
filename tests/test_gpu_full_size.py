"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(default plan of ecq_quantize_update, then ecq_dequant_aggregate), free-running for every
iteration of each workload.

The comparison is total for all five workloads: every code byte, every scale and every h value
of every worker at every iteration, and every value of the average, against the oracle
free-running from h = 0 on the seeded gradients alone (no oracle input ever comes from the
library).  Rows are streamed one at a time so that the 32 x 138 M element workload needs one
row of g on the host at a time.  Bars as in test_gpu_parity.py; the tests require bit
identity, which implies the 1e-6 bar, and report the 1e-6 verdict when bits differ.
"""
import numpy as np
import pytest

import oracle
import synth
from tests.test_gpu_parity import SEED, GpuState, _rel_ok

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1806_08054_amd as E
    return E


def _pack_row_chunked(q_row, s, chunk=1 << 20):
    """oracle.pack of one long row, taken in byte-aligned chunks that run in parallel."""
    n = q_row.size
    whole = n // chunk
    parts = []
    if whole:
        parts.append(oracle.pack_rows(q_row[: whole * chunk].reshape(whole, chunk), s).reshape(-1))
    if n > whole * chunk:
        parts.append(oracle.pack(q_row[whole * chunk:], s))
    return np.concatenate(parts)


def _bucket_extent(wl, k, r):
    """(first element, end element, first byte, end byte) of bucket k of a row."""
    e0 = k * wl.bucket
    e1 = min(wl.N, e0 + wl.bucket)
    return e0, e1, e0 * r // 8, (e1 * r + 7) // 8


class _Staging:
    """Pinned host buffers and device buffers of one worker row, reused for every row: the
    gradient row travels to the oracle through them, the oracle's results back to the GPU,
    where they are compared bit for bit with the library's (a 138 M element row takes well
    under a second that way)."""

    def __init__(self, N, rb):
        self.g = torch.empty(N, dtype=torch.float32, pin_memory=True)
        self.h = torch.empty(N, dtype=torch.float32, pin_memory=True)
        self.codes = torch.empty(rb, dtype=torch.uint8, pin_memory=True)
        self.dev_h = torch.empty(N, dtype=torch.float32, device="cuda")
        self.dev_codes = torch.empty(rb, dtype=torch.uint8, device="cuda")


def _same_bits(a, b):
    """Bitwise equality of two device tensors of the same dtype (NaN-safe, -0.0 != +0.0)."""
    if a.dtype == torch.float32:
        a, b = a.view(torch.int32), b.view(torch.int32)
    return bool(torch.equal(a, b))


def _check_row(st, stg, wl, t, p, h_row):
    """One whole worker row: the oracle runs on the seeded g row and ITS OWN h row (advanced in
    place); every code byte, every scale (as u32) and every h value of the library's row must
    equal the oracle's.  Returns the oracle's encoded row and scales."""
    N = wl.N
    stg.g.copy_(st.g[p, :N])
    g_np = stg.g.numpy()[None, :]
    q, scales, _ = oracle.batch_step(g_np, h_row[None, :], wl.bucket, wl.s, wl.alpha, wl.beta, SEED, t,
                                     worker0=p, norm=wl.norm)
    codes_ref = _pack_row_chunked(q[0], wl.s)
    sc = st.scales[p, : st.nb].cpu().numpy()
    assert np.array_equal(sc.view(np.uint32), scales[0].view(np.uint32)), f"scales differ, worker {p}, iteration {t}"
    stg.codes.numpy()[:] = codes_ref
    stg.dev_codes.copy_(stg.codes)
    if not _same_bits(stg.dev_codes, st.codes[p, : st.rb]):
        nbad = int((st.codes[p, : st.rb].cpu().numpy() != codes_ref).sum())
        raise AssertionError(f"{nbad} code bytes differ, worker {p}, iteration {t}")
    stg.h.numpy()[:] = h_row
    stg.dev_h.copy_(stg.h)
    if not _same_bits(stg.dev_h, st.h[p, :N]):
        hh = st.h[p, :N].cpu().numpy()
        nbits = int((hh.view(np.uint32) != h_row.view(np.uint32)).sum())
        within = _rel_ok(hh, h_row, wl.bucket)
        raise AssertionError(f"{nbits} h values not bit-identical (within 1e-6 per bucket: {within}), "
                             f"worker {p}, iteration {t}")
    return codes_ref, scales[0]


def _run(E, wl, aligned=True):
    """Free-running iterations of a whole workload, compared in full: every code byte, scale
    and h value of every worker at every iteration, and every value of the average.  The
    comparison is streamed one worker row at a time (the oracle keeps its own h rows on the
    host; one row of g is copied over at a time), and the average is taken by the oracle from
    its own messages.  aligned: worker rows start on 128-byte lines, the layout bench.py times;
    otherwise the tightest legal strides."""
    st = GpuState(E, wl.P, wl.N, wl.bucket, wl.s, aligned=aligned, norm=wl.norm)
    stg = _Staging(wl.N, st.rb)
    h_rows = [np.zeros(wl.N, np.float32) for _ in range(wl.P)]
    dev_out = torch.empty(wl.N, dtype=torch.float32, device="cuda")
    for t in range(wl.iters):
        synth.gradients(wl, t, device="cuda", out=st.g)
        st.poison()
        E.ecq_quantize_update(st.sh, st.g, st.h, wl.alpha, wl.beta, SEED, t, st.codes, st.scales)
        st.out.fill_(-7.0)
        E.ecq_dequant_aggregate(st.sh, st.codes, st.scales, st.out)
        torch.cuda.synchronize()
        assert bool((st.codes[:, st.rb:] == 0xEE).all())
        assert bool((st.scales[:, st.nb:] == -7.0).all())
        codes_ref = np.empty((wl.P, st.rb), np.uint8)
        scales_ref = np.empty((wl.P, st.nb), np.float32)
        for p in range(wl.P):
            codes_ref[p], scales_ref[p] = _check_row(st, stg, wl, t, p, h_rows[p])
        ref = oracle.aggregate(codes_ref, scales_ref, wl.N, wl.bucket, wl.s)
        dev_out.copy_(torch.from_numpy(ref))
        if not _same_bits(dev_out, st.out):
            got = st.out.cpu().numpy()
            nbits = int((got.view(np.uint32) != ref.view(np.uint32)).sum())
            raise AssertionError(f"{nbits} values of the average not bit-identical "
                                 f"(within 1e-6 per bucket: {_rel_ok(got, ref, wl.bucket)}), iteration {t}")
        print(f"{wl.name}: iteration {t}: {wl.P} rows and the average equal the oracle's", flush=True)


def test_linear_full(E):
    """Workload 2: 100 free-running iterations, every element of every iteration."""
    _run(E, synth.WORKLOADS["linear"])


def test_resnet50_full(E):
    """Workload 3 (the metric workload): 20 free-running iterations, every element of every
    iteration."""
    _run(E, synth.WORKLOADS["resnet50"])


def test_resnet50_tight_rows(E):
    """Workload 3 with the tightest legal strides (worker rows start 32 bytes into a cache
    line): 2 iterations, every element."""
    wl = synth.scaled(synth.WORKLOADS["resnet50"], iters=2)
    _run(E, wl, aligned=False)


def test_resnet50_l2(E):
    """Workload 3's shape with l_2 scaling, the setting of the paper's CNN experiments
    (Section 6.2): 3 iterations, every element."""
    wl = synth.scaled(synth.WORKLOADS["resnet50"], iters=3, norm="l2")
    _run(E, wl)


@pytest.mark.parametrize("norm", ["linf", "l2"])
def test_resnet50_one_norm_per_row(E, norm):
    """Workload 3's rows quantised as Eq. (8) states it, without buckets: one norm per worker
    (two passes over g and h; for l_2 the tree over 8192-element pieces): 2 iterations, every
    element."""
    wl = synth.WORKLOADS["resnet50"]
    wl = synth.scaled(wl, iters=2, norm=norm, bucket=(wl.N + 7) // 8 * 8)
    _run(E, wl)


@pytest.mark.parametrize("name", ["paper_cnn", "paper_linear"])
def test_paper_settings_full(E, name):
    """The paper's own quantiser settings on the metric workload's gradient (P = 8,
    N = 25,557,032): Section 6.2's (bucket 4096, l_2 scaling, s = 4, alpha = 0.01, beta = 1.0) and
    Section 6.1's (l_2, s = 4, alpha = 0.2, beta = 0.9, 1024-element vectors): 3 free-running
    iterations, every element."""
    _run(E, synth.WORKLOADS[name])


def test_alexnet_full(E):
    """Workload 4: 10 free-running iterations, all 16 workers and the average in full at every
    iteration."""
    _run(E, synth.WORKLOADS["alexnet"])


def test_vgg16_full(E):
    """Workload 5: 5 free-running iterations incl. the average over all 32 workers (35 GB of g
    and h resident, 64-bit element offsets); all 32 workers and the average in full at every
    iteration, streamed one worker row at a time."""
    _run(E, synth.WORKLOADS["vgg16"])


@pytest.mark.parametrize("name,rows", [("resnet50", [0, 7]), ("alexnet", [5]), ("vgg16", [31])])
def test_huffman_full_size(E, name, rows):
    """Huffman coding (Section 4) of one iteration's messages at the benchmark's sizes: every
    row decodes back to its fixed-length message; every row's length lies between the
    entropy bound sum_k d_k log2(d/d_k) and that bound plus one bit per element; the rows in
    `rows` are compared in full (counts, code, tile offsets, stream) with the oracle."""
    wl = synth.WORKLOADS[name]
    st = GpuState(E, wl.P, wl.N, wl.bucket, wl.s, aligned=True)
    synth.gradients(wl, 0, device="cuda", out=st.g)
    E.ecq_quantize_update(st.sh, st.g, st.h, wl.alpha, wl.beta, SEED, 0, st.codes, st.scales)
    P, N, s = wl.P, wl.N, wl.s
    # The levels of the rows compared in full come from the oracle, run on the seeded gradients.
    q_rows = {}
    for p in rows:
        g_row = st.g[p, :N].cpu().numpy()[None, :]
        q_rows[p] = oracle.batch_step(g_row, np.zeros_like(g_row), wl.bucket, s, wl.alpha, wl.beta, SEED, 0,
                                      worker0=p)[0][0]
    del st.g, st.h
    bins, tiles = 2 * s + 1, E.huffman_num_tiles(N)
    counts = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    lengths = torch.zeros(P, bins, dtype=torch.uint8, device="cuda")
    codewords = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    stream_stride = st.sh.code_stride
    streams = torch.full((P, stream_stride), 0xEE, dtype=torch.uint8, device="cuda")
    offs = torch.zeros(P, tiles + 1, dtype=torch.int64, device="cuda")
    back = torch.zeros_like(st.codes)
    E.ecq_level_histogram(st.sh, st.codes, counts, bins)
    E.ecq_huffman_build(P, s, counts, bins, lengths, codewords)
    E.ecq_huffman_encode(st.sh, st.codes, lengths, codewords, bins, streams, stream_stride, offs, tiles + 1)
    E.ecq_huffman_decode(st.sh, streams, stream_stride, offs, tiles + 1, lengths, codewords, bins, back)
    torch.cuda.synchronize()
    assert torch.equal(back[:, : st.rb], st.codes[:, : st.rb]), "decode(encode(message)) differs from the message"
    cnt = counts.cpu().numpy().astype(np.uint64)
    total = offs[:, tiles].cpu().numpy()
    for p in range(P):
        assert int(cnt[p].sum()) == N
        bound = oracle.entropy_bound_bits(cnt[p])
        assert bound - 1e-6 * N <= int(total[p]) < bound + N, (p, bound, int(total[p]))
        assert int(total[p]) <= N * E.code_bits(s)
    for p in rows:
        q = q_rows[p]
        assert np.array_equal(st.codes[p, : st.rb].cpu().numpy(), _pack_row_chunked(q, s))
        ref_counts = oracle.level_histogram(q, s)
        assert np.array_equal(cnt[p], ref_counts)
        ref_len = oracle.huffman_lengths(ref_counts)
        ref_cw = oracle.huffman_codes(ref_len)
        assert np.array_equal(lengths[p].cpu().numpy(), ref_len)
        assert np.array_equal(codewords[p].cpu().numpy().view(np.uint64), ref_cw)
        ref_stream, ref_offs, bits = oracle.huffman_encode(q, s, ref_len, ref_cw)
        assert np.array_equal(offs[p].cpu().numpy().view(np.uint64), ref_offs)
        nbytes = (bits + 7) // 8
        assert np.array_equal(streams[p, :nbytes].cpu().numpy(), ref_stream[:nbytes]), f"stream differs, worker {p}"
        print(f"{name}: worker {p}: {bits / N:.4f} bits per element (fixed length: {E.code_bits(s)})", flush=True)


def test_row_longer_than_2_pow_32(E):
    """One worker row of 2^32 + 5,000 elements (17 GB each of g and h): element indices, byte
    offsets and the Philox counter beyond 32 bits.  Buckets around the 2^32 boundary, the first
    and the ragged last one are recomputed by the oracle; the aggregate (P = 1) is checked on
    the same buckets."""
    N, bucket, s = (1 << 32) + 5000, 512, 1
    wl = synth.Workload("long", P=1, N=N, bucket=bucket, s=s, alpha=1.0, beta=0.9, iters=1, kind="normal",
                        data_seed=3)
    st = GpuState(E, 1, N, bucket, s, aligned=True)
    gen = torch.Generator(device="cuda").manual_seed(1234)
    step = 1 << 28
    for e0 in range(0, N, step):                               # seeded input, drawn in slabs
        e1 = min(N, e0 + step)
        st.g[0, e0:e1] = torch.randn(e1 - e0, generator=gen, device="cuda") * 0.01
    r = E.code_bits(s)
    edge = (1 << 32) // bucket
    ks = [0, 1, edge - 2, edge - 1, edge, edge + 1, wl.nb - 2, wl.nb - 1, 12345, edge // 2 + 7]
    before = {k: st.g[0, k * bucket:min(N, (k + 1) * bucket)].cpu().numpy() for k in ks}
    E.ecq_quantize_update(st.sh, st.g, st.h, wl.alpha, wl.beta, SEED, 3, st.codes, st.scales)
    E.ecq_dequant_aggregate(st.sh, st.codes, st.scales, st.out)
    torch.cuda.synchronize()
    for k in ks:
        e0, e1, b0, b1 = _bucket_extent(wl, k, r)
        g_np = before[k]
        q, scale, gt, h_next = oracle.bucket_step(g_np, np.zeros_like(g_np), e0, 0, s, wl.alpha, wl.beta, SEED, 3)
        assert st.scales[0, k].item() == float(scale), f"scale differs in bucket {k}"
        assert np.array_equal(st.codes[0, b0:b1].cpu().numpy(), oracle.pack(q, s)), f"codes differ in bucket {k}"
        assert np.array_equal(st.h[0, e0:e1].cpu().numpy().view(np.uint32), h_next.view(np.uint32))
        ref = oracle.aggregate(oracle.pack(q, s)[None, :], np.array([[scale]], np.float32), e1 - e0, bucket, s)
        assert np.array_equal(st.out[e0:e1].cpu().numpy().view(np.uint32), ref.view(np.uint32))
    assert bool((st.codes[0, st.rb:] == 0xEE).all())
    w = torch.zeros(8, dtype=torch.int32, device="cuda")
    E.ecq_philox_words(SEED, 3, 0, (1 << 32) + 4, 8, w)
    torch.cuda.synchronize()
    assert np.array_equal(w.cpu().numpy().view(np.uint32), oracle.words(SEED, 3, 0, (1 << 32) + 4, 8))
