"""GPU parity of the zero-run Huffman coder (Section 4, cost paragraph: entropy coding of the
quantised levels) against the CPU oracle: token counts, code, per-tile bit counts, group
offsets and stream bit-exact; decode(encode(message)) = message; the library decodes a stream
the oracle wrote.  Every oracle input is a seeded level array or the oracle's own output.
"""
import numpy as np
import pytest

import oracle
import synth
from tests.test_gpu_parity import SEED, GpuState, _dev

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def E():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1806_08054_amd as E
    return E


def _levels(rng, P, n, s, p_nonzero):
    q = rng.integers(1, s + 1, (P, n)) * rng.choice([-1, 1], (P, n))
    return np.where(rng.random((P, n)) < p_nonzero, q, 0).astype(np.int8)


class ZrunBuffers:
    def __init__(self, E, P, N, s, pad=0):
        self.Z, self.symbols = E.zrun_symbols(s)
        self.tiles, self.groups = E.zrun_num_tiles(N)
        self.table_stride = self.symbols + pad
        self.stream_stride = E.zrun_stream_bytes(N, s) + 4 * pad
        self.tile_stride = self.tiles + pad
        self.group_stride = self.groups + 1 + pad
        dev = "cuda"
        self.counts = torch.full((P, self.table_stride), -1, dtype=torch.int64, device=dev)
        self.lengths = torch.full((P, self.table_stride), 0xEE, dtype=torch.uint8, device=dev)
        self.codewords = torch.full((P, self.table_stride), -1, dtype=torch.int64, device=dev)
        self.streams = torch.full((P, self.stream_stride), 0xEE, dtype=torch.uint8, device=dev)
        self.tile_bits = torch.full((P, self.tile_stride), -1, dtype=torch.int32, device=dev)
        self.group_offsets = torch.full((P, self.group_stride), -1, dtype=torch.int64, device=dev)


def _roundtrip(E, q, s, bucket=512, pad=0):
    """q: [P, N] int8 levels.  Encodes their fixed-length message on the GPU and compares every
    product with the oracle's."""
    P, N = q.shape
    st = GpuState(E, P, N, bucket, s, pad=pad)
    codes_ref = oracle.pack_rows(q, s)
    st.codes[:, : st.rb] = _dev(codes_ref)
    zb = ZrunBuffers(E, P, N, s, pad=pad)
    E.ecq_zrun_histogram(st.sh, st.codes, zb.counts, zb.table_stride)
    E.ecq_zrun_build(P, s, zb.counts, zb.table_stride, zb.lengths, zb.codewords)
    E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, zb.table_stride, zb.streams, zb.stream_stride,
                      zb.tile_bits, zb.tile_stride, zb.group_offsets, zb.group_stride)
    back = torch.full_like(st.codes, 0xEE)
    E.ecq_zrun_decode(st.sh, zb.streams, zb.stream_stride, zb.tile_bits, zb.tile_stride, zb.group_offsets,
                      zb.group_stride, zb.lengths, zb.codewords, zb.table_stride, back)
    torch.cuda.synchronize()
    A = zb.symbols
    counts = zb.counts.cpu().numpy()
    lengths = zb.lengths.cpu().numpy()
    codewords = zb.codewords.cpu().numpy().view(np.uint64)
    streams = zb.streams.cpu().numpy()
    tile_bits = zb.tile_bits.cpu().numpy().view(np.uint32)
    group_offsets = zb.group_offsets.cpu().numpy().view(np.uint64)
    total_bits = 0
    for p in range(P):
        ref_counts = oracle.zrun_histogram(q[p], s)
        assert np.array_equal(counts[p, :A].astype(np.uint64), ref_counts), f"token counts differ, row {p}"
        ref_len = oracle.huffman_lengths(ref_counts)
        ref_cw = oracle.huffman_codes(ref_len)
        assert np.array_equal(lengths[p, :A], ref_len), f"codeword lengths differ, row {p}"
        assert np.array_equal(codewords[p, :A], ref_cw), f"codewords differ, row {p}"
        ref_stream, ref_bits, ref_groups, bits = oracle.zrun_encode(q[p], s, ref_len, ref_cw)
        assert np.array_equal(tile_bits[p, : zb.tiles], ref_bits), f"tile sizes differ, row {p}"
        assert np.array_equal(group_offsets[p, : zb.groups + 1], ref_groups), f"group offsets differ, row {p}"
        nbytes = (bits + 31) // 32 * 4
        assert np.array_equal(streams[p, :nbytes], ref_stream[:nbytes]), f"stream differs, row {p}"
        assert np.all(streams[p, nbytes:] == 0xEE), "bytes beyond the stream were written"
        total_bits += bits
    # nothing outside the documented extents is touched
    assert np.all(counts[:, A:] == -1) and np.all(lengths[:, A:] == 0xEE)
    assert np.all(zb.tile_bits.cpu().numpy()[:, zb.tiles:] == -1)
    assert np.all(zb.group_offsets.cpu().numpy()[:, zb.groups + 1:] == -1)
    assert torch.equal(back[:, : st.rb].cpu(), torch.from_numpy(codes_ref)), "decode(encode(message)) differs"
    assert bool((back[:, st.rb:] == 0xEE).all())
    return total_bits


@pytest.mark.parametrize("s,p_nz", [(1, 0.04), (1, 0.33), (1, 0.0), (1, 1.0), (3, 0.1), (4, 0.06), (7, 0.3),
                                    (20, 0.2), (63, 0.5), (127, 0.5), (2, 0.002)])
def test_zrun_matches_oracle(E, s, p_nz):
    """Several groups of 64 tiles, whole tiles and a ragged tail, from all zeros to all
    non-zero, every code width."""
    rng = np.random.default_rng([s, int(p_nz * 1000)])
    N = 2 * 64 * 4096 + 5 * 4096 + 777
    _roundtrip(E, _levels(rng, 2, N, s, p_nz), s)


@pytest.mark.parametrize("N", [1, 7, 16, 127, 128, 1023, 1024, 1025, 4095, 4096, 4097, 8192, 64 * 4096, 64 * 4096 + 1])
def test_zrun_lengths_around_tile_and_group_boundaries(E, N):
    rng = np.random.default_rng(N)
    for s, p_nz in ((1, 0.1), (5, 0.3)):
        _roundtrip(E, _levels(rng, 3, N, s, p_nz), s, bucket=8, pad=3)


def test_zrun_runs_around_the_longest_run(E):
    """Runs of exactly Z - 1, Z, Z + 1 and multiples of Z zeros, at the start, in the middle and
    at the end of tiles, and across step (1024) and tile (4096) boundaries."""
    for s in (1, 4, 31, 127):
        Z = 127 // s
        rng = np.random.default_rng(s)
        q = np.zeros((2, 5 * 4096 + 300), np.int8)
        at = 0
        for run in [Z - 1, Z, Z + 1, 2 * Z, 2 * Z + 1, 0, 0, 1, 1023, 1024, 4095, 4096, 3 * Z - 1, 5]:
            at += max(run, 0)
            if at >= q.shape[1]:
                break
            q[0, at] = rng.integers(1, s + 1) * rng.choice([-1, 1])
            at += 1
        q[1, 4095] = 1                                       # a tile that ends with its only level
        q[1, 4096] = -1                                      # ... and one that starts with it
        q[1, 2 * 4096 + 1023: 2 * 4096 + 1025] = 1           # both sides of a step boundary
        _roundtrip(E, q, s)


def test_zrun_long_codewords(E):
    """Token counts that fall off like Fibonacci numbers give codewords beyond 24 and beyond 32
    bits: the encoder's long path and the decoder's canonical walk."""
    s = 1
    fib = [1, 1]
    while len(fib) < 40:
        fib.append(fib[-1] + fib[-2])
    # token (z, +1) for z = 0..39 occurs fib[z] times: a message made of such tokens in random order
    rng = np.random.default_rng(5)
    reps = np.repeat(np.arange(28), [fib[z] for z in range(28)])      # about 830 k tokens
    rng.shuffle(reps)
    total = int((reps + 1).sum())
    q = np.zeros((1, total), np.int8)
    ends = np.cumsum(reps + 1) - 1
    q[0, ends] = 1
    _roundtrip(E, q, s)


def test_zrun_long_codewords_in_sparse_tiles(E):
    """Codewords of up to 47 bits, from a prefix code given to the coder instead of its own
    Huffman code (lengths 1, 2, ..., 39 by falling token count, 47 for the rest: Kraft's sum stays
    below 1), on a message whose first part is dense and whose second part has runs of 111 to 126
    zeros: the encoder writes sparse tiles a whole tile at a time and dense ones in steps, and
    in both appends codewords longer than 32 bits in two parts; the decoder walks the canonical
    code beyond its table and beyond 32 bits.  Sizes, offsets and stream against the oracle's
    encoder with the same code, then decode(encode(message)) = message."""
    s = 1
    fib = [1, 1]
    while len(fib) < 30:
        fib.append(fib[-1] + fib[-2])
    rng = np.random.default_rng(11)
    runs_of = [126 - k if k < 16 else 29 - k for k in range(30)]      # zeros before the level of token k
    dense = np.repeat([runs_of[k] for k in range(16, 30)], [fib[k] for k in range(16, 30)])
    sparse = np.repeat([runs_of[k] for k in range(16)], [40 * fib[k] for k in range(16)])
    rng.shuffle(dense)
    rng.shuffle(sparse)
    reps = np.concatenate([dense, sparse]).astype(np.int64)
    N = int((reps + 1).sum())
    q = np.zeros((1, N), np.int8)
    q[0, np.cumsum(reps + 1) - 1] = 1
    counts = oracle.zrun_histogram(q[0], s)
    order = np.argsort(-counts.astype(np.int64), kind="stable")
    lengths = np.zeros(len(counts), np.uint8)
    lengths[order] = [min(rank + 1, 39) if rank < 39 else 47 for rank in range(len(counts))]
    codewords = oracle.huffman_codes(lengths)
    assert sum(2.0 ** -int(l) for l in lengths) <= 1.0
    ref_stream, ref_bits, ref_groups, bits = oracle.zrun_encode(q[0], s, lengths, codewords)
    assert int(ref_bits.min()) <= 2048 < int(ref_bits.max())          # sparse tiles and dense ones
    st = GpuState(E, 1, N, 512, s)
    codes_ref = oracle.pack_rows(q, s)
    st.codes[:, : st.rb] = _dev(codes_ref)
    zb = ZrunBuffers(E, 1, N, s)
    zb.lengths[0, : zb.symbols] = _dev(lengths)
    zb.codewords[0, : zb.symbols] = _dev(codewords.view(np.int64))
    E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, zb.table_stride, zb.streams, zb.stream_stride,
                      zb.tile_bits, zb.tile_stride, zb.group_offsets, zb.group_stride)
    back = torch.full_like(st.codes, 0xEE)
    E.ecq_zrun_decode(st.sh, zb.streams, zb.stream_stride, zb.tile_bits, zb.tile_stride, zb.group_offsets,
                      zb.group_stride, zb.lengths, zb.codewords, zb.table_stride, back)
    torch.cuda.synchronize()
    assert (bits + 7) // 8 <= zb.stream_stride
    assert np.array_equal(zb.tile_bits[0, : zb.tiles].cpu().numpy().view(np.uint32), ref_bits)
    assert np.array_equal(zb.group_offsets[0, : zb.groups + 1].cpu().numpy().view(np.uint64), ref_groups)
    nbytes = (bits + 7) // 8
    assert np.array_equal(zb.streams[0, :nbytes].cpu().numpy(), ref_stream[:nbytes]), "stream differs"
    assert torch.equal(back[:, : st.rb].cpu(), torch.from_numpy(codes_ref)), "decode(encode(message)) differs"


def test_zrun_decodes_an_oracle_stream(E):
    """The library's decoder on a stream, index and tables written by the oracle."""
    s, P, N = 3, 2, 64 * 4096 + 3000
    rng = np.random.default_rng(77)
    q = _levels(rng, P, N, s, 0.08)
    st = GpuState(E, P, N, 512, s)
    zb = ZrunBuffers(E, P, N, s)
    zb.streams.zero_()
    for p in range(P):
        counts = oracle.zrun_histogram(q[p], s)
        lengths = oracle.huffman_lengths(counts)
        cw = oracle.huffman_codes(lengths)
        stream, tile_bits, groups, bits = oracle.zrun_encode(q[p], s, lengths, cw)
        zb.lengths[p, : zb.symbols] = _dev(lengths)
        zb.codewords[p, : zb.symbols] = _dev(cw.view(np.int64))
        zb.streams[p, : stream.size] = _dev(stream)
        zb.tile_bits[p, : zb.tiles] = _dev(tile_bits.view(np.int32))
        zb.group_offsets[p, : zb.groups + 1] = _dev(groups.view(np.int64))
    E.ecq_zrun_decode(st.sh, zb.streams, zb.stream_stride, zb.tile_bits, zb.tile_stride, zb.group_offsets,
                      zb.group_stride, zb.lengths, zb.codewords, zb.table_stride, st.codes)
    torch.cuda.synchronize()
    assert np.array_equal(st.codes.cpu().numpy()[:, : st.rb], oracle.pack_rows(q, s))


def test_zrun_foreign_tables_stay_in_bounds(E):
    """Tables that do not belong to the message (all lengths 63, or all 0) give a meaningless
    stream, never an access outside the documented extents."""
    s, P, N = 1, 2, 3 * 4096 + 100
    rng = np.random.default_rng(9)
    q = _levels(rng, P, N, s, 0.5)
    st = GpuState(E, P, N, 512, s)
    st.codes[:, : st.rb] = _dev(oracle.pack_rows(q, s))
    for fill in (63, 0, 200):
        zb = ZrunBuffers(E, P, N, s, pad=2)
        zb.lengths.fill_(fill)
        zb.codewords.fill_(-1)
        E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, zb.table_stride, zb.streams, zb.stream_stride,
                          zb.tile_bits, zb.tile_stride, zb.group_offsets, zb.group_stride)
        back = torch.full_like(st.codes, 0xEE)
        E.ecq_zrun_decode(st.sh, zb.streams, zb.stream_stride, zb.tile_bits, zb.tile_stride, zb.group_offsets,
                          zb.group_stride, zb.lengths, zb.codewords, zb.table_stride, back)
        torch.cuda.synchronize()
        assert bool((back[:, st.rb:] == 0xEE).all())
        assert bool((zb.tile_bits[:, zb.tiles:] == -1).all()) and bool((zb.group_offsets[:, zb.groups + 1:] == -1).all())


def test_zrun_argument_errors(E):
    s, P, N = 1, 2, 10000
    st = GpuState(E, P, N, 512, s)
    zb = ZrunBuffers(E, P, N, s)
    enc = lambda **kw: E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, kw.get("ts", zb.table_stride),
                                         zb.streams, kw.get("ss", zb.stream_stride), zb.tile_bits,
                                         kw.get("tl", zb.tile_stride), zb.group_offsets, kw.get("gs", zb.group_stride))
    for kw in ({"ts": zb.symbols - 1}, {"ss": zb.stream_stride - 4}, {"ss": zb.stream_stride + 2},
               {"tl": zb.tiles - 1}, {"gs": zb.groups}):
        with pytest.raises(E.EcqError) as err:
            enc(**kw)
        assert err.value.status == -5
    with pytest.raises(E.EcqError) as err:
        E.ecq_zrun_histogram(st.sh, st.codes, zb.counts, zb.symbols - 1)
    assert err.value.status == -5
    with pytest.raises(E.EcqError) as err:
        E.ecq_zrun_build(P, 0, zb.counts, zb.table_stride, zb.lengths, zb.codewords)
    assert err.value.status == -3
    torch.cuda.synchronize()
    assert bool((zb.streams == 0xEE).all()) and bool((zb.tile_bits == -1).all())


@pytest.mark.parametrize("name,rows", [("resnet50", [0, 7]), ("alexnet", [5]), ("vgg16", [31]), ("paper_cnn", [3])])
def test_zrun_full_size(E, name, rows):
    """The zero-run coder on one iteration's messages at the benchmark's sizes: every row
    decodes back to its fixed-length message; the rows in `rows` are compared in full (token
    counts, code, tile sizes, group offsets, stream) with the oracle, whose levels come from its
    own quantiser run on the seeded gradients; every row's length stays below the paper's bound
    sum_k d_k log2(d/d_k) plus 3 % (index excluded)."""
    wl = synth.WORKLOADS[name]
    st = GpuState(E, wl.P, wl.N, wl.bucket, wl.s, aligned=True, norm=wl.norm)
    synth.gradients(wl, 0, device="cuda", out=st.g)
    E.ecq_quantize_update(st.sh, st.g, st.h, wl.alpha, wl.beta, SEED, 0, st.codes, st.scales)
    P, N, s = wl.P, wl.N, wl.s
    q_rows = {}
    for p in rows:
        g_row = st.g[p, :N].cpu().numpy()[None, :]
        q_rows[p] = oracle.batch_step(g_row, np.zeros_like(g_row), wl.bucket, s, wl.alpha, wl.beta, SEED, 0,
                                      worker0=p, norm=wl.norm)[0][0]
    del st.g, st.h
    zb = ZrunBuffers(E, P, N, s)
    bins = 2 * s + 1
    level_counts = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    E.ecq_level_histogram(st.sh, st.codes, level_counts, bins)
    E.ecq_zrun_histogram(st.sh, st.codes, zb.counts, zb.table_stride)
    E.ecq_zrun_build(P, s, zb.counts, zb.table_stride, zb.lengths, zb.codewords)
    E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, zb.table_stride, zb.streams, zb.stream_stride,
                      zb.tile_bits, zb.tile_stride, zb.group_offsets, zb.group_stride)
    back = torch.zeros_like(st.codes)
    E.ecq_zrun_decode(st.sh, zb.streams, zb.stream_stride, zb.tile_bits, zb.tile_stride, zb.group_offsets,
                      zb.group_stride, zb.lengths, zb.codewords, zb.table_stride, back)
    torch.cuda.synchronize()
    assert torch.equal(back[:, : st.rb], st.codes[:, : st.rb]), "decode(encode(message)) differs from the message"
    total = zb.group_offsets[:, zb.groups].cpu().numpy()
    lc = level_counts.cpu().numpy().astype(np.uint64)
    for p in range(P):
        bound = oracle.entropy_bound_bits(lc[p])
        assert int(total[p]) <= 1.03 * bound + 64, (p, int(total[p]) / N, bound / N)
        assert int(total[p]) == int(zb.tile_bits[p, : zb.tiles].to(torch.int64).sum().item())
    for p in rows:
        q = q_rows[p]
        ref_counts = oracle.zrun_histogram(q, s)
        assert np.array_equal(zb.counts[p, : zb.symbols].cpu().numpy().astype(np.uint64), ref_counts)
        ref_len = oracle.huffman_lengths(ref_counts)
        ref_cw = oracle.huffman_codes(ref_len)
        assert np.array_equal(zb.lengths[p, : zb.symbols].cpu().numpy(), ref_len)
        assert np.array_equal(zb.codewords[p, : zb.symbols].cpu().numpy().view(np.uint64), ref_cw)
        ref_stream, ref_bits, ref_groups, bits = oracle.zrun_encode(q, s, ref_len, ref_cw)
        assert np.array_equal(zb.tile_bits[p, : zb.tiles].cpu().numpy().view(np.uint32), ref_bits)
        assert np.array_equal(zb.group_offsets[p, : zb.groups + 1].cpu().numpy().view(np.uint64), ref_groups)
        nbytes = (bits + 7) // 8
        assert np.array_equal(zb.streams[p, :nbytes].cpu().numpy(), ref_stream[:nbytes]), f"stream differs, worker {p}"
        bound = oracle.entropy_bound_bits(oracle.level_histogram(q, s))
        print(f"{name}: worker {p}: {bits / N:.4f} bits per element, bound {bound / N:.4f}, "
              f"fixed length {E.code_bits(s)}", flush=True)


@pytest.mark.parametrize("P,tiles,s", [(1, 300, 1), (2, 10_000, 4), (2, 20_000, 1), (3, 50_000, 2), (2, 100_000, 1)])
def test_zrun_decoder_tiles_per_wave(E, P, tiles, s):
    """The decoder gives a wave 8, 16, 32 or 64 tiles depending on how many tiles the whole
    message has (the first four cases, in that order; the last one is a message of the size at
    which it takes output windows of 16 words instead of 32), the per-level decoder between 8 and 64: every
    setting decodes the message it was given, through groups of 64 tiles that several waves
    share and a ragged last tile.  Levels come straight from the seeded generator; the encoder
    that feeds the decoder is compared with the oracle elsewhere, here on row 0."""
    N = tiles * 4096 - 1234
    rng = np.random.default_rng([P, tiles, s])
    q = _levels(rng, P, N, s, 0.08)
    q[:, N // 3: N // 3 + 3 * 64 * 4096] = 0                    # three whole groups of zeros
    st = GpuState(E, P, N, 512, s)
    codes_ref = oracle.pack_rows(q, s)
    st.codes[:, : st.rb] = _dev(codes_ref)
    zb = ZrunBuffers(E, P, N, s)
    E.ecq_zrun_histogram(st.sh, st.codes, zb.counts, zb.table_stride)
    E.ecq_zrun_build(P, s, zb.counts, zb.table_stride, zb.lengths, zb.codewords)
    E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, zb.table_stride, zb.streams, zb.stream_stride,
                      zb.tile_bits, zb.tile_stride, zb.group_offsets, zb.group_stride)
    back = torch.full_like(st.codes, 0xEE)
    E.ecq_zrun_decode(st.sh, zb.streams, zb.stream_stride, zb.tile_bits, zb.tile_stride, zb.group_offsets,
                      zb.group_stride, zb.lengths, zb.codewords, zb.table_stride, back)
    torch.cuda.synchronize()
    ref_counts = oracle.zrun_histogram(q[0], s)
    ref_len = oracle.huffman_lengths(ref_counts)
    ref_cw = oracle.huffman_codes(ref_len)
    ref_stream, ref_bits, ref_groups, bits = oracle.zrun_encode(q[0], s, ref_len, ref_cw)
    assert np.array_equal(zb.tile_bits[0, : zb.tiles].cpu().numpy().view(np.uint32), ref_bits)
    assert np.array_equal(zb.streams[0, : (bits + 7) // 8].cpu().numpy(), ref_stream[: (bits + 7) // 8])
    assert torch.equal(back[:, : st.rb].cpu(), torch.from_numpy(codes_ref)), "decode(encode(message)) differs"
    assert bool((back[:, st.rb:] == 0xEE).all())
    # the per-level coder on the same message
    bins = 2 * s + 1
    hcounts = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    hlen = torch.zeros(P, bins, dtype=torch.uint8, device="cuda")
    hwords = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    htiles = E.huffman_num_tiles(N)
    offs = torch.zeros(P, htiles + 1, dtype=torch.int64, device="cuda")
    hstreams = torch.zeros(P, st.sh.code_stride, dtype=torch.uint8, device="cuda")
    E.ecq_level_histogram(st.sh, st.codes, hcounts, bins)
    E.ecq_huffman_build(P, s, hcounts, bins, hlen, hwords)
    E.ecq_huffman_encode(st.sh, st.codes, hlen, hwords, bins, hstreams, st.sh.code_stride, offs, htiles + 1)
    back.fill_(0xEE)
    E.ecq_huffman_decode(st.sh, hstreams, st.sh.code_stride, offs, htiles + 1, hlen, hwords, bins, back)
    torch.cuda.synchronize()
    assert torch.equal(back[:, : st.rb].cpu(), torch.from_numpy(codes_ref)), "per-level decode(encode(message)) differs"


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5, 7, 20])
def test_zrun_codes_beyond_the_grid_count_as_level_zero(E, s):
    """r-bit patterns above 2s (no message of this library holds one) are tokenised as level 0:
    a message with such codes planted in it gives the token counts, tile sizes and stream of
    the same message with the code of level 0 in their place.  (The oracle works on levels and
    cannot hold such a code; the reference here is the library on the cleaned message, whose
    products are compared with the oracle's by the other tests.)"""
    r = E.code_bits(s)
    if 2 * s + 1 == (1 << r):
        pytest.skip("every r-bit pattern is a level")
    rng = np.random.default_rng(s)
    P, N = 2, 3 * 64 * 4096 + 1000
    q = _levels(rng, P, N, s, 0.2)
    clean = oracle.pack_rows(q, s)
    # plant codes beyond the grid in one element out of 50
    codes = np.zeros((P, N), np.int64) + (q.astype(np.int64) + s)
    planted = rng.random((P, N)) < 0.02
    codes_bad = np.where(planted, rng.integers(2 * s + 1, 1 << r, (P, N)), codes)
    codes_clean = np.where(planted, s, codes)
    def pack(c):
        out = np.zeros((P, clean.shape[1]), np.uint8)
        for p in range(P):
            bits = ((c[p][:, None] >> np.arange(r)) & 1).astype(np.uint8).reshape(-1)
            packed = np.packbits(bits, bitorder="little")
            out[p, : len(packed)] = packed
        return out
    assert np.array_equal(pack(codes), clean)                   # the packer above is the oracle's layout
    results = []
    for message in (pack(codes_bad), pack(codes_clean)):
        st = GpuState(E, P, N, 512, s)
        st.codes[:, : st.rb] = _dev(message)
        zb = ZrunBuffers(E, P, N, s)
        E.ecq_zrun_histogram(st.sh, st.codes, zb.counts, zb.table_stride)
        E.ecq_zrun_build(P, s, zb.counts, zb.table_stride, zb.lengths, zb.codewords)
        E.ecq_zrun_encode(st.sh, st.codes, zb.lengths, zb.codewords, zb.table_stride, zb.streams, zb.stream_stride,
                          zb.tile_bits, zb.tile_stride, zb.group_offsets, zb.group_stride)
        torch.cuda.synchronize()
        total = int(zb.group_offsets[0, zb.groups].item())
        results.append((zb.counts[:, : zb.symbols].cpu().numpy(), zb.tile_bits[:, : zb.tiles].cpu().numpy(),
                        zb.streams[0, : (total + 7) // 8].cpu().numpy()))
    for got, ref in zip(results[0], results[1]):
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("s", [1, 2, 4, 9])
def test_zrun_tiles_around_the_encoder_route_limits(E, s):
    """The encoder takes a tile by a list of its non-zero levels while it has at most 1024 of
    them, and a wave writes whole tiles while each of its four tiles has at most 4096 stream
    bits: tiles with exactly 0, 1, 1023, 1024, 1025 and 4096 non-zero levels, side by side in
    one wave and on their own, with the levels spread evenly, bunched at the tile's start and at
    its end, and a ragged last tile."""
    rng = np.random.default_rng(100 + s)
    counts = [1024, 1025, 1023, 0, 4096, 1, 1024, 1024, 1024, 1024, 0, 0, 0, 0, 1023, 1025, 2048, 600, 1024, 300]
    N = len(counts) * 4096 - 777
    q = np.zeros((2, N), np.int8)
    for p in range(2):
        for t, c in enumerate(counts):
            lo, hi = t * 4096, min((t + 1) * 4096, N)
            c = min(c, hi - lo)
            if p == 0:
                where = rng.choice(hi - lo, c, replace=False)               # spread
            elif t % 2 == 0:
                where = np.arange(c)                                        # bunched at the start
            else:
                where = (hi - lo) - 1 - np.arange(c)                        # bunched at the end
            q[p, lo + where] = rng.integers(1, s + 1, c) * rng.choice([-1, 1], c)
    _roundtrip(E, q, s)
