#!/usr/bin/env python3
"""Benchmark of the ECQ-SGD hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic gradients that already
sit in HBM: the fused compensate / norm / stochastic-round / encode / error-update kernel
over all P workers (Section 4, Eq. (6)-(9) of Wu et al., ICML 2018), then the
dequantise-and-average kernel over the P encoded messages (Eq. (4)).

Prints ONE JSON line.  `value` is the algorithmic bytes of a whole step divided by the step
time; the `roofline` object is the fused kernel alone (the kernel the headline metric is
about), timed with HIP events inside the timed region; `cpu_baseline` is the CPU oracle
timed on a bounded sample of the same workload on this machine's host cores.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth


def algorithmic_bytes(P, N, bucket, s, E):
    """(fused, dequant) bytes one step must move: read g, read h, write h, write codes and
    scales; then read codes and scales of all workers, write the fp32 average."""
    rb, nb = E.row_bytes(N, s), E.num_buckets(N, bucket)
    fused = P * (12 * N + rb + 4 * nb)
    dequant = P * (rb + 4 * nb) + 4 * N
    return fused, dequant


def kernel_sources_sha():
    """Hash of the sources of the fused and aggregation kernels: the counter summaries under
    profiles/ are stamped with it, and a figure taken from one is only reported while it
    matches."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1806_08054_amd", "csrc")
    for name in ("ecq_device.hpp", "ecq_kernels.hip"):
        h.update(name.encode())
        h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(workload):
    """(bytes per launch of the fused kernel, source) from the committed FETCH_SIZE / WRITE_SIZE
    summary of this workload, or (None, reason) when there is none for the current sources."""
    path = os.path.join(ROOT, "profiles", f"fused_{workload}_pmc_traffic.txt")
    if not os.path.exists(path):
        return None, "no profiles/ summary for this workload"
    stamp, value = None, None
    for line in open(path):
        if line.startswith("kernel_sources_sha:"):
            stamp = line.split(":")[1].strip()
        if line.startswith("hbm_bytes_per_launch:"):
            value = int(line.split(":")[1])
    rel = os.path.relpath(path, ROOT)
    if stamp != kernel_sources_sha():
        return None, f"{rel} was taken on other kernel sources ({stamp}); not reported"
    return value, f"{rel} (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by the copy kernel; kernel sources {stamp})"


def cpu_baseline(wl, sample_n, g_sample, steps=3):
    """The oracle as it stands on a prefix of every worker's gradient (whole buckets), `steps`
    free-running steps: about 10-30 s of CPU work at the default sizes."""
    import numpy as np
    import oracle
    P = wl.P
    g = np.ascontiguousarray(g_sample, np.float32)
    h = np.zeros_like(g)
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    for t in range(steps):
        q, scales, _ = oracle.batch_step(g, h, wl.bucket, wl.s, wl.alpha, wl.beta, 1, t, threads=threads,
                                         norm=wl.norm)
        codes = oracle.pack_rows(q, wl.s)
        oracle.aggregate(codes, scales, sample_n, wl.bucket, wl.s)
    dt = (time.perf_counter() - t0) / steps

    def step_bytes(n):
        rb = oracle.row_bytes(n, wl.s)
        nb = (n + wl.bucket - 1) // wl.bucket
        return P * (12 * n + rb + 4 * nb) + P * (rb + 4 * nb) + 4 * n

    # The same on one thread, one step, on a sixteenth of the sample (whole buckets).
    n1 = max(wl.bucket, sample_n // 16 // wl.bucket * wl.bucket)
    n1 = min(n1, sample_n)
    g1 = np.ascontiguousarray(g[:, :n1])
    h1 = np.zeros_like(g1)
    t0 = time.perf_counter()
    q, scales, _ = oracle.batch_step(g1, h1, wl.bucket, wl.s, wl.alpha, wl.beta, 1, 0, threads=1, norm=wl.norm)
    oracle.aggregate(oracle.pack_rows(q, wl.s), scales, n1, wl.bucket, wl.s)
    dt1 = time.perf_counter() - t0
    return {"value": round(step_bytes(sample_n) / dt / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"first {sample_n} elements of each of the {P} workers, {steps} steps "
                      f"(quantise+update, pack, aggregate), {dt:.2f} s wall per step on {threads} threads",
            "gelem_per_s": round(P * sample_n / dt / 1e9, 5),
            "one_thread": {"value": round(step_bytes(n1) / dt1 / 1e9, 4), "unit": "GB/s",
                           "sample": f"first {n1} elements of each worker, one step, {dt1:.2f} s"}}


def entropy_coding(E, torch, sh, wl, codes, timed):
    """Outside the timed region: the entropy coding of the last step's messages that the paper's
    communication-cost figures assume (Section 4, cost paragraph), leg by leg, for the per-level
    Huffman code and for the zero-run Huffman code.  bits_per_element counts everything that has
    to travel besides the bucket scales: stream, per-tile sizes, group offsets, code lengths;
    compression_vs_fp32 also counts the 32-bit scale of every bucket."""
    P, N, s = wl.P, wl.N, wl.s
    bins, tiles = 2 * s + 1, E.huffman_num_tiles(N)
    counts = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    lengths = torch.zeros(P, bins, dtype=torch.uint8, device="cuda")
    words = torch.zeros(P, bins, dtype=torch.int64, device="cuda")
    streams = torch.zeros(P, sh.code_stride, dtype=torch.uint8, device="cuda")
    offs = torch.zeros(P, tiles + 1, dtype=torch.int64, device="cuda")
    back = torch.zeros_like(codes)
    hist_ms = timed(lambda: E.ecq_level_histogram(sh, codes, counts, bins))
    build_ms = timed(lambda: E.ecq_huffman_build(P, s, counts, bins, lengths, words))
    enc_ms = timed(lambda: E.ecq_huffman_encode(sh, codes, lengths, words, bins, streams, sh.code_stride, offs,
                                                tiles + 1))
    dec_ms = timed(lambda: E.ecq_huffman_decode(sh, streams, sh.code_stride, offs, tiles + 1, lengths, words, bins,
                                                back))
    rb = E.row_bytes(N, s)
    ok = bool(torch.equal(back[:, :rb], codes[:, :rb]))
    bits = int(offs[:, tiles].sum().item())
    bound = sum(E.ecq_entropy_bound_bits(row) for row in counts.cpu().tolist())
    per_level = {"bits_per_element": round(bits / (P * N), 4), "histogram_ms": round(hist_ms, 4),
                 "build_ms": round(build_ms, 4), "encode_ms": round(enc_ms, 4), "decode_ms": round(dec_ms, 4),
                 "encode_gelem_per_s": round(P * N / (enc_ms * 1e-3) / 1e9, 1),
                 "decode_gelem_per_s": round(P * N / (dec_ms * 1e-3) / 1e9, 1), "round_trip_ok": ok}
    del streams, offs
    # The zero-run code (tokens = a run of zeros with the level that ends it): the one that can
    # reach the paper's bound when it lies below one bit per element.
    _, symbols = E.zrun_symbols(s)
    ztiles, zgroups = E.zrun_num_tiles(N)
    zstride = E.zrun_stream_bytes(N, s)
    zcounts = torch.zeros(P, symbols, dtype=torch.int64, device="cuda")
    zlengths = torch.zeros(P, symbols, dtype=torch.uint8, device="cuda")
    zwords = torch.zeros(P, symbols, dtype=torch.int64, device="cuda")
    zstreams = torch.zeros(P, zstride, dtype=torch.uint8, device="cuda")
    tile_bits = torch.zeros(P, ztiles, dtype=torch.int32, device="cuda")
    group_offs = torch.zeros(P, zgroups + 1, dtype=torch.int64, device="cuda")
    back.zero_()
    zhist_ms = timed(lambda: E.ecq_zrun_histogram(sh, codes, zcounts, symbols))
    zbuild_ms = timed(lambda: E.ecq_zrun_build(P, s, zcounts, symbols, zlengths, zwords))
    zenc_ms = timed(lambda: E.ecq_zrun_encode(sh, codes, zlengths, zwords, symbols, zstreams, zstride, tile_bits, ztiles,
                                              group_offs, zgroups + 1))
    zdec_ms = timed(lambda: E.ecq_zrun_decode(sh, zstreams, zstride, tile_bits, ztiles, group_offs, zgroups + 1,
                                              zlengths, zwords, symbols, back))
    zok = bool(torch.equal(back[:, :rb], codes[:, :rb]))
    zbits = int(group_offs[:, zgroups].sum().item())
    index_bits = P * (32 * ztiles + 64 * (zgroups + 1) + 8 * symbols)      # tile sizes, group offsets, code lengths
    zero_run = {"stream_bits_per_element": round(zbits / (P * N), 4),
                "index_bits_per_element": round(index_bits / (P * N), 4),
                "bits_per_element": round((zbits + index_bits) / (P * N), 4),
                "over_entropy_bound_pct": round(100 * ((zbits + index_bits) / bound - 1), 2) if bound > 0 else None,
                "histogram_ms": round(zhist_ms, 4), "build_ms": round(zbuild_ms, 4), "encode_ms": round(zenc_ms, 4),
                "decode_ms": round(zdec_ms, 4), "encode_gelem_per_s": round(P * N / (zenc_ms * 1e-3) / 1e9, 1),
                "decode_gelem_per_s": round(P * N / (zdec_ms * 1e-3) / 1e9, 1), "round_trip_ok": zok}
    return {"entropy_bound_bits_per_element": round(bound / (P * N), 4),
            "fixed_length_bits_per_element": E.code_bits(s),
            "bits_per_element": zero_run["bits_per_element"],
            "compression_vs_fp32": round(32 * P * N / (zbits + index_bits + 32 * P * wl.nb), 2),
            "zero_run_huffman": zero_run, "per_level_huffman": per_level}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50",
                    choices=["tiny", "linear", "resnet50", "alexnet", "vgg16", "paper_cnn", "paper_linear"],
                    help="resnet50 is the metric workload; paper_cnn / paper_linear are the paper's own "
                         "quantiser settings (Sections 6.2 / 6.1) on the same gradient")
    ap.add_argument("--pool", type=int, default=2, help="distinct gradient batches cycled through")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-entropy-coding", action="store_true",
                    help="skip the Huffman legs (level histogram, code construction, encode, decode)")
    ap.add_argument("--cpu-sample", type=int, default=32 * 1024 * 1024)
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; the P workers are a resident batch on it "
                 "(--gpus must be 1)")

    import torch
    import paper_1806_08054_amd as E
    import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    wl = synth.WORKLOADS[args.workload]
    P, N = wl.P, wl.N
    sh = E.Shape.aligned(N, P, wl.bucket, wl.s, norm={"linf": 0, "l2": 1}[wl.norm])   # rows start on 128-byte lines
    pool = [synth.gradients(wl, t, device="cuda",
                            out=torch.zeros(P, sh.gh_stride, dtype=torch.float32, device="cuda"))
            for t in range(max(1, args.pool))]
    h = torch.zeros(P, sh.gh_stride, dtype=torch.float32, device="cuda")
    codes = torch.zeros(P, sh.code_stride, dtype=torch.uint8, device="cuda")
    scales = torch.zeros(P, sh.scale_stride, dtype=torch.float32, device="cuda")
    out = torch.zeros(N, dtype=torch.float32, device="cuda")
    fused_b, deq_b = algorithmic_bytes(P, N, wl.bucket, wl.s, E)
    seed = 1

    def step(t, ev=None):
        g = pool[t % len(pool)]
        if ev:
            ev[0].record()
        E.ecq_quantize_update(sh, g, h, wl.alpha, wl.beta, seed, t, codes, scales)
        if ev:
            ev[1].record()
        E.ecq_dequant_aggregate(sh, codes, scales, out)

    # Achievable-bandwidth calibration, outside the timed region: the fused pass's access
    # pattern (read two fp32 streams, write one; one float4 per lane) without its arithmetic,
    # and a plain copy of known size (also the reference for scaling profiler byte counters).
    n_cal = P * sh.gh_stride
    cal_a, cal_b = pool[0].view(-1), h.view(-1)
    cal_o = torch.empty_like(cal_a)

    def timed(fn, reps=10):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    add_ms = timed(lambda: E.ecq_calib_add(cal_a, cal_b, cal_o, n_cal))
    copy_ms = timed(lambda: E.ecq_calib_copy(cal_a, cal_o, n_cal))
    del cal_o
    # The aggregation's access pattern (P rows of codes read side by side, one float written per
    # element) without its arithmetic.
    gather_ms = timed(lambda: E.ecq_calib_gather(sh, codes, out))

    for t in range(args.warmup):
        step(t)
    torch.cuda.synchronize()
    K = args.steps
    # Two events per step bracket the fused kernel; the aggregation of step i ends where the
    # fused kernel of step i+1 starts (one more event closes the last step).
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(args.warmup + i, evs[i])
    evs[K][0].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / K
    fused_ms = sum(evs[i][0].elapsed_time(evs[i][1]) for i in range(K)) / K
    deq_ms = sum(evs[i][1].elapsed_time(evs[i + 1][0]) for i in range(K)) / K

    value = (fused_b + deq_b) / (ms_per_step * 1e-3) / 1e9
    fused_gbps = fused_b / (fused_ms * 1e-3) / 1e9
    traffic, traffic_source = profiled_traffic(wl.name)
    result = {
        "metric": "ECQ quantize+error-update GB/s (% HBM peak), 25M-elem grad, P=8",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: P={P} workers x N={N} fp32, bucket {wl.bucket}, s={wl.s} "
                               f"({E.code_bits(wl.s)}-bit codes), {wl.norm} norm, alpha={wl.alpha}, beta={wl.beta}; "
                               "step = fused quantise+error-update over all workers, then dequantise+average",
                   "workers": P, "n": N, "bucket": wl.bucket, "s": wl.s, "norm": wl.norm},
        # `value` is the whole step; the kernel the metric's name refers to is reported beside it.
        "value_is": "whole step: algorithmic bytes of fused quantise+error-update plus dequantise+average / step time",
        "whole_step_GBps": round(value, 1),
        "fused_quantize_update_GBps": round(fused_gbps, 1),
        "fused_quantize_update_pct_hbm_peak": round(100 * fused_gbps / HBM_PEAK_GBPS, 2),
        "step_bytes": fused_b + deq_b,
        "gelem_per_s": round(P * N / (ms_per_step * 1e-3) / 1e9, 2),
        "fused": {"ms": round(fused_ms, 4), "GBps": round(fused_gbps, 1),
                  "pct_hbm_peak": round(100 * fused_gbps / HBM_PEAK_GBPS, 2),
                  "gelem_per_s": round(P * N / (fused_ms * 1e-3) / 1e9, 2), "bytes": fused_b},
        "dequant_aggregate": {"ms": round(deq_ms, 4), "GBps": round(deq_b / (deq_ms * 1e-3) / 1e9, 1),
                              "pct_hbm_peak": round(100 * deq_b / (deq_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
                              "bytes": deq_b},
        "calibration": {"add_2r1w_GBps": round(12 * n_cal / (add_ms * 1e-3) / 1e9, 1),
                        "copy_1r1w_GBps": round(8 * n_cal / (copy_ms * 1e-3) / 1e9, 1),
                        "floats": n_cal,
                        "aggregate_pattern_GBps": round((P * E.row_bytes(N, wl.s) + 4 * N) / (gather_ms * 1e-3) / 1e9, 1),
                        "aggregate_pattern_ms": round(gather_ms, 4)},
        "roofline": {"bound": "hbm", "kernel": "ecq_quantize_update (fused single pass)",
                     "achieved": round(fused_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(fused_gbps / HBM_PEAK_GBPS, 4),
                     # HBM bytes per launch from a separate rocprofv3 counter run on the same kernel
                     # sources (not measured in this run); null when no such summary is committed.
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": fused_b},
    }
    if not args.no_entropy_coding:
        result["entropy_coding"] = entropy_coding(E, torch, sh, wl, codes, timed)
    if not args.no_cpu_baseline:
        n_s = min(N, max(wl.bucket, args.cpu_sample // wl.bucket * wl.bucket))
        result["cpu_baseline"] = cpu_baseline(wl, n_s, pool[0][:, :n_s].cpu().numpy())
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
