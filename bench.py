#!/usr/bin/env python3
"""Benchmark of libhfr on one MI355X.

A step is one pass of the whole hot path over one synthetic gradient batch of
the headline workload (K = 8 peer buffers, bf16, n = 64 Mi elements each):

  1. hfr_reduce_buckets: the flat gradient cut into 25 Mi-element buckets,
     every bucket reduced K-way in fp32 (in buffer order) and stored as bf16,
     chunk-pipelined over 4 HIP streams              -> (K+1) * n * 2 bytes
  2. hfr_combine_avg: the node partial combined with a received remote partial
     and scaled by 1 / (8 * 16), in place             -> 3 * n * 2 bytes

`value` is the metric as defined for this workload: (K+1) * n * 2 bytes divided
by the time of the K-way reduction (part 1 of the timed steps, run on its own
for the same number of passes, HIP events on the launch stream); `step` and
`ms_per_step` are the whole step (both parts, wall clock). Inputs are resident in HBM. `roofline` times the dominant kernel
(the K-way bf16 sum over the full 64 Mi buffer, one launch) with HIP events on
its launch stream and puts a ceiling measured in the same run beside it;
`cpu_baseline` times the CPU oracle on the same step on this host.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_BYTES_PER_S = 8.0e12  # MI355X published HBM3E peak

K = 8
N_ELEMS = 1 << 26
ELEM = 2
SCALE = 1.0 / (8 * 16)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--chunk-elems", type=int, default=0, help="chunk size of the bucket scheduler (0: one chunk per bucket)")
    ap.add_argument("--streams", type=int, default=4)
    ap.add_argument("--preheat-ms", type=float, default=PREHEAT_MS,
                    help="untimed device-busy time before every warm-up (brings the clocks to their steady state; 0 = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true",
                    help="run only the dominant-kernel launches (for rocprofv3 runs)")
    ap.add_argument("--roofline-launches", type=int, default=50)
    ap.add_argument("--config", default="",
                    help="instead of the default step, time one of the other workloads and print its own JSON "
                         "line: cfg1 (K=8 fp32 n=1Mi), cfg3 (bucketed transformer gradients), cfg4 (latency "
                         "regime table), cfg5 (combine, fp32 n=256Mi), ceilings (streaming probes: read-only, fill, "
                         "copy, 2:1, 8:1), f16 (headline shape in fp16), "
                         "sweep (sizes x K table), allk (every K, bf16 and fp32, against the shape before request pacing), placement (plain vs tuned kernel at ten buffer spacings), msg186 (186 MiB fp32 message), e4m3 / e5m2 (fp8, 128 MiB per buffer), avg (fused K-way average), slice (one rank's slice of eight), bcast (1-to-8 broadcast)")
    ap.add_argument("--no-placement-tuning", action="store_true",
                    help="skip hfr_tune_placement in the set-up: time the plain kernels whatever the buffers' placement")
    ap.add_argument("--separate-allocations", action="store_true",
                    help="leave every buffer where torch's allocator puts it instead of carving them from one "
                         "allocation at hfr_peer_stride (default line and cfg3)")
    ap.add_argument("--no-placement-spread", action="store_true",
                    help="skip the pass over ten random buffer placements (default line and cfg3)")
    ap.add_argument("--with-copy", action="store_true",
                    help="with --roofline-only: also launch the K=1 copy of one 128 MiB buffer (counter calibration)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "reduce_sum_k8_bf16_64mi_hbm_traffic.txt"),
                    help="summary of the committed rocprofv3 counter runs; its hbm_bytes_per_launch line is reported")
    return ap.parse_args()


_HFR_DT = {"torch.float32": 0, "torch.bfloat16": 1, "torch.float16": 2, "torch.float8_e4m3fn": 3, "torch.float8_e5m2": 4}


def carve(torch, hfr, count, n_elems, dtype, device, K, measure=True):
    """`count` buffers of n_elems elements, one after the other in ONE device
    allocation (a staging arena that the reduction's caller owns) at the
    distance hfr_tune_peer_stride measures for a K-way sum on that very
    allocation: hfr_peer_stride's value unless one of eight neighbouring
    distances is more than 1.5 % faster (measure=False: the rule's value as it
    is, no timing launches). Returns (allocation, views, stride in bytes, the
    rule's stride)."""
    es = torch.empty(0, dtype=dtype).element_size()
    nbytes = n_elems * es
    rule = hfr.hfr_peer_stride(nbytes)
    room = max(rule, (nbytes + (2 << 20) - 1) // (2 << 20) * (2 << 20) + (14 << 20))
    slab = torch.empty(room * count, dtype=torch.uint8, device=device)
    torch.cuda.synchronize()
    stride = rule
    if measure:
        _, stride = hfr.hfr_tune_peer_stride(slab, room * count, K, n_elems, _HFR_DT[str(dtype)])
    return slab, [slab[j * stride: j * stride + nbytes].view(dtype) for j in range(count)], stride, rule


def place(torch, hfr, args, tensors, n_outputs, device):
    """Copies of `tensors` plus n_outputs uninitialised buffers of the same
    shape, carved from one allocation at hfr_peer_stride (or the tensors
    themselves plus fresh allocations with --separate-allocations). Returns
    (buffers, outputs, text for the JSON line)."""
    t0 = tensors[0]
    if args.separate_allocations:
        return list(tensors), [torch.empty_like(t0) for _ in range(n_outputs)], "every buffer allocated on its own"
    slab, views, stride, rule = carve(torch, hfr, len(tensors) + n_outputs, t0.numel(), t0.dtype, device, len(tensors))
    for v, t in zip(views, tensors):
        v.copy_(t)
    torch.cuda.synchronize()
    return views[:len(tensors)], views[len(tensors):], ("buffers in one allocation at the measured stride of %d MiB "
                                                        "(hfr_peer_stride: %d MiB)" % (stride >> 20, rule >> 20))


def make_inputs(torch, hfr, synth, device, arena=True, measure=True):
    """The K peer buffers, the remote partial, the output and a second output
    (for the fused step). arena=True: all of them carved from one allocation at
    the library's stride; the separately allocated tensors the generators
    returned are kept as well (`separate`), for the comparison line."""
    ins = synth.peer_buffers_normal_bf16(K, N_ELEMS, 1e-3, 2000, device)
    remote = synth.normal_bf16(N_ELEMS, 1e-3 * (K ** 0.5), 2100, device)
    if not arena:
        out = torch.empty(N_ELEMS, dtype=torch.bfloat16, device=device)
        return ins, remote, out, torch.empty_like(out), None
    slab, views, stride, rule = carve(torch, hfr, K + 3, N_ELEMS, torch.bfloat16, device, K, measure)
    for j in range(K):
        views[j].copy_(ins[j])
    views[K + 1].copy_(remote)
    info = {"slab": slab, "stride": stride, "rule": rule, "separate": (ins, torch.empty(N_ELEMS, dtype=torch.bfloat16, device=device))}
    return views[:K], views[K + 1], views[K], views[K + 2], info


def time_dominant_kernel(torch, hfr, ins, out, stream, launches, warmup=5):
    """Average duration of one K=8 bf16 64 Mi launch, with HIP events recorded
    on the stream the kernel is launched on: one event pair around `launches`
    back-to-back launches (kernels on one stream start when the previous one
    ends, so elapsed / launches is the average launch duration). A second pass
    puts an event pair around every single launch; those figures include the
    event-to-kernel dispatch gap and are reported beside the average."""
    _preheat(torch, stream, lambda: hfr.hfr_reduce_sum(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream), PREHEAT_MS)
    with torch.cuda.stream(stream):
        for _ in range(warmup):
            hfr.hfr_reduce_sum(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(launches):
            hfr.hfr_reduce_sum(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream)
        e1.record(stream)
        pairs = []
        for _ in range(launches):
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record(stream)
            hfr.hfr_reduce_sum(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream)
            b.record(stream)
            pairs.append((a, b))
    stream.synchronize()
    avg = e0.elapsed_time(e1) / launches
    ms = sorted(a.elapsed_time(b) for a, b in pairs)
    return avg, ms[len(ms) // 2], ms[0]


def cpu_baseline(torch, synth, ins, remote, cuts):
    """The CPU oracle, as it stands, on the same step (all buckets + combine),
    single-threaded, on this host. Bounded to about 10-30 s of CPU work."""
    import numpy as np
    import oracle
    host_ins = [synth.as_numpy_bits(t) for t in ins]
    host_remote = synth.as_numpy_bits(remote)
    out = np.empty(N_ELEMS, dtype=np.uint16)
    buckets = [([a[o:o + l] for a in host_ins], out[o:o + l]) for o, l in cuts]
    oracle.reduce_buckets([([a[:4096] for a in host_ins], out[:4096])], oracle.BF16)  # page in the library
    times = []
    t_all = time.perf_counter()
    while True:
        t0 = time.perf_counter()
        oracle.reduce_buckets(buckets, oracle.BF16)
        oracle.combine_avg(out, host_remote, SCALE, oracle.BF16, out=out)
        times.append(time.perf_counter() - t0)
        if len(times) >= 3 and time.perf_counter() - t_all > 10.0:
            break
        if len(times) >= 8:
            break
    best = min(times)
    step_bytes = (K + 1 + 3) * N_ELEMS * ELEM

    # The same oracle functions on disjoint index slices from all host threads (elementwise
    # independence makes the result identical); context beside the single-thread baseline.
    from concurrent.futures import ThreadPoolExecutor
    threads = max(1, min(os.cpu_count() or 1, 16))
    bounds = [(N_ELEMS * t // threads, N_ELEMS * (t + 1) // threads) for t in range(threads)]
    out_mt = np.empty(N_ELEMS, dtype=np.uint16)

    def work(be):
        b, e = be
        oracle.reduce_sum([a[b:e] for a in host_ins], oracle.BF16, out=out_mt[b:e])
        oracle.combine_avg(out_mt[b:e], host_remote[b:e], SCALE, oracle.BF16, out=out_mt[b:e])

    mt_times = []
    with ThreadPoolExecutor(max_workers=threads) as pool:
        for _ in range(3):
            t0 = time.perf_counter()
            list(pool.map(work, bounds))
            mt_times.append(time.perf_counter() - t0)
    mt_best = min(mt_times)
    return {
        "value": step_bytes / best / 1e9,
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": "the full step (K=8 bf16 n=64Mi bucketed sum + combine), %d repetitions, best of them; "
                  "host has %d logical cpus" % (len(times), os.cpu_count() or 0),
        "seconds_per_step": best,
        "all_threads": {"value": step_bytes / mt_best / 1e9, "threads": threads, "seconds_per_step": mt_best,
                        "identical_to_single_thread": bool(np.array_equal(out_mt, out))},
    }, out


def _preheat(torch, stream, fn, ms):
    """Keeps the device busy with fn for about `ms` milliseconds, untimed, and
    leaves the work queued (no synchronisation at the end), so that what is
    timed next starts on a device at its steady clocks. Measured on MI355X:
    after an idle gap of 5 ms or more the next 10 to 15 ms of launches run 4 to
    9 % slower (K=8 bf16 64 Mi: 184-193 us per launch, then 177), whatever ran
    before the gap; a training loop never idles that long."""
    if ms <= 0:
        return
    with torch.cuda.stream(stream):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        fn()
        e1.record(stream)
    stream.synchronize()
    per_call = max(e0.elapsed_time(e1) / 2, 1e-3)
    # at most a few hundred calls: thousands of queued launches of a few microseconds each slow the
    # launches behind them down (4 MiB two- and four-operand sums: 5 -> 7.7 us per launch)
    calls = int(min(max(ms / per_call, 1), 400))
    with torch.cuda.stream(stream):
        for _ in range(calls):
            fn()


PREHEAT_MS = 100.0


def _event_time_ms(torch, stream, fn, reps, warmup=3, preheat_ms=None):
    """Average ms per call of fn, HIP events on `stream`. Synchronises the
    device first (the input generators ran on another stream), then brings it to
    its steady clocks (see _preheat) before the warm-up calls."""
    torch.cuda.synchronize()
    _preheat(torch, stream, fn, PREHEAT_MS if preheat_ms is None else preheat_ms)
    with torch.cuda.stream(stream):
        for _ in range(warmup):
            fn()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
    stream.synchronize()
    return e0.elapsed_time(e1) / reps


def measure_ceilings(torch, device, stream, full=False, reps=20):
    """What HBM delivers on this machine for plain streaming passes in the access
    shapes of the reduction kernels (libhfr_probe: XOR of the read streams, no
    arithmetic of the method): read-only over eight streams, fill, copy, 2:1 and
    8:1 read/write mixes, 128 MiB per buffer, HIP events on the launch stream.
    With full=False only what the default bench line quotes is measured."""
    from paper_2408_14158_amd import probe
    nbytes = 128 << 20
    bufs = [torch.empty(nbytes, dtype=torch.uint8, device=device) for _ in range(10)]
    for i, b in enumerate(bufs):
        b.fill_(i + 1)
    sink = torch.zeros(64, dtype=torch.uint8, device=device)
    cases = [("read_only_8_streams", 8, 0), ("fill", 0, 1), ("mix_8r_1w", 8, 1), ("mix_2r_1w", 2, 1)]
    if full:
        cases += [("copy_1r_1w", 1, 1), ("read_only_1_stream", 1, 0), ("read_only_2_streams", 2, 0),
                  ("read_only_16_streams", 16, 0), ("mix_9r_1w", 9, 1), ("mix_16r_1w", 16, 1), ("mix_1r_8w", 1, 8)]
    rows = {}
    # the bulk shape's two pacing knobs (workgroup size, pause after each trip), as the library's
    # kernels have them: the best of a small grid is what the shape can deliver for this mix
    paced_grid = [(lanes, pace) for lanes in (128, 192, 256, 320, 384) for pace in (0, 2, 8)]
    for label, R, W in cases:
        if R + W > len(bufs):
            extra = [torch.empty(nbytes, dtype=torch.uint8, device=device).fill_(3) for _ in range(R + W - len(bufs))]
            bufs += extra
        rd, wr = bufs[:R], bufs[R:R + W]
        row = {"reads": R, "writes": W, "bytes": (R + W) * nbytes}
        for shape, sname in ((probe.HFR_PROBE_WIDE, "wide"), (probe.HFR_PROBE_BULK, "bulk")):
            ms = _event_time_ms(torch, stream, lambda: probe.hfr_probe_stream(rd, wr, sink, nbytes, shape, stream), reps)
            row[sname + "_us"] = ms * 1e3
            row[sname + "_GBps"] = (R + W) * nbytes / ms / 1e6
        best = (0.0, 0, 0)
        for lanes, pace in paced_grid:
            ms = _event_time_ms(torch, stream, lambda: probe.hfr_probe_stream_paced(rd, wr, sink, nbytes, lanes, pace, stream),
                                max(reps // 2, 5), warmup=2)
            rate = (R + W) * nbytes / ms / 1e6
            if rate > best[0]:
                best = (rate, lanes, pace)
        row["paced_bulk_GBps"], row["paced_bulk_lanes"], row["paced_bulk_pace"] = best
        row["best_GBps"] = max(row["wide_GBps"], row["bulk_GBps"], row["paced_bulk_GBps"])
        rows[label] = row
    return {"config": "ceilings: streaming probes, 128 MiB per buffer, %d launches each, HIP events; paced_bulk = the best of the "
                      "bulk shape over workgroup sizes 128..384 and pauses 0, 2, 8 (x 64 clocks)" % reps,
            "cells": rows}


def placement_spread(torch, hfr, stream, K, n_elems, slab_gib, trials, seed, device, run=None):
    """GB/s of the K-way bf16 sum over `trials` random placements of its K + 1
    buffers (non-overlapping, 2 MiB-aligned offsets in one slab), each measured
    after the library has had its on-the-fly trial launches: min / median / max.
    run(ins, out) enqueues one pass (default: one hfr_reduce_sum)."""
    import random
    rng = random.Random(seed)
    unit = 1 << 20                                   # bf16 elements per 2 MiB
    per = (n_elems + unit - 1) // unit               # units per buffer
    slab_units = (slab_gib << 30) // (2 << 20)
    slab = torch.empty(slab_units * unit, dtype=torch.bfloat16, device=device)
    slab.view(torch.int16).fill_(0x3A00)             # a small normal bf16 value everywhere
    rates, patterns = [], []
    for _ in range(trials):
        while True:                                  # K + 1 starts, no two closer than one buffer
            starts = sorted(rng.randrange(0, slab_units - per) for _ in range(K + 1))
            if all(b - a >= per for a, b in zip(starts, starts[1:])):
                break
        rng.shuffle(starts)
        bufs = [slab[u * unit: u * unit + n_elems] for u in starts]
        ins, out = bufs[:K], bufs[K]
        fn = (lambda: run(ins, out)) if run else (lambda: hfr.hfr_reduce_sum(ins, K, out, n_elems, hfr.HFR_BF16, stream))
        _event_time_ms(torch, stream, fn, 14, warmup=0)      # the library's trial launches on this placement
        ms = _event_time_ms(torch, stream, fn, 10, warmup=1)
        rates.append((K + 1) * n_elems * 2 / ms / 1e6)
        patterns.append(hfr.hfr_placement_query(ins, K, out, hfr.HFR_BF16)[2])
    rates_sorted = sorted(rates)
    del slab
    return {"what": "K=%d bf16 sum, %d random placements of the %d buffers in a %d GiB slab, after on-the-fly placement "
                    "tuning" % (K, trials, K + 1, slab_gib),
            "min_GBps": rates_sorted[0], "median_GBps": rates_sorted[len(rates_sorted) // 2],
            "max_GBps": rates_sorted[-1], "GBps": rates, "recorded_patterns": patterns}


def oracle_sample_baseline(fn, bytes_moved, what, min_seconds=8.0, max_reps=6):
    """cpu_baseline entry: the oracle call fn() timed single-threaded on this
    host, best of a few repetitions of a bounded sample."""
    fn()                                             # page in the library and the sample
    times, t_all = [], time.perf_counter()
    while len(times) < max_reps and (len(times) < 2 or time.perf_counter() - t_all < min_seconds):
        t0 = time.perf_counter()
        fn()
        times.append(time.perf_counter() - t0)
    return {"value": bytes_moved / min(times) / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%s, %d repetitions, best of them; host has %d logical cpus" % (what, len(times), os.cpu_count() or 0),
            "seconds_per_sample": min(times)}


def composite_ceiling(rows, n_read, n_write):
    """Serial model: reads at the read-only rate of eight streams, then writes at
    the fill rate (reads and writes share the one DRAM bus). GB/s."""
    rd, wr = rows["read_only_8_streams"]["best_GBps"], rows["fill"]["best_GBps"]
    return (n_read + n_write) / (n_read / rd + n_write / wr)


def run_other_config(args, torch, hfr, synth, device, stream):
    """Secondary workloads (parity-test shapes), one JSON line each."""
    peak = HBM_PEAK_BYTES_PER_S
    name = args.config
    if name == "cfg1":
        Kc, n = 8, 1 << 20
        ins = synth.peer_buffers_uniform_f32(Kc, n, 1000, device)
        out = torch.empty(n, dtype=torch.float32, device=device)
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, hfr.HFR_F32, stream), 200)
        b = (Kc + 1) * n * 4
        print(json.dumps({"config": "cfg1: K=8 fp32 n=1Mi (cache-resident, launch-bound)", "us_per_launch": ms * 1e3,
                          "GBps": b / ms / 1e6, "note": "working set 36 MiB fits the 256 MiB Infinity Cache"}))
    elif name == "cfg3":
        Kc = 8
        tensors = synth.transformer_grad_tensors()
        total = sum(t.numel for t in tensors)
        if args.separate_allocations:
            flats = [synth.flat_gradient_bf16(tensors, 3000 + j, device) for j in range(Kc)]
            out = torch.empty(total, dtype=torch.bfloat16, device=device)
            stride = None
        else:
            # the K flat gradient buffers and the output, one after the other in one allocation
            slab, views, stride, rule = carve(torch, hfr, Kc + 1, total, torch.bfloat16, device, Kc)
            for j in range(Kc):
                views[j].copy_(synth.flat_gradient_bf16(tensors, 3000 + j, device))
            flats, out = views[:Kc], views[Kc]
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
        b = (Kc + 1) * total * 2
        # primary packing: flat cuts every 25Mi elements; secondary: whole tensors, greedy
        whole = synth.bucket_cuts_whole_tensors(tensors)
        flat_cuts = synth.bucket_cuts(total)
        lines = []
        for label, cuts, chunk in (("flat buckets of 25Mi", flat_cuts, synth.BUCKET_CAP_ELEMS),
                                   ("whole-tensor buckets closed at >= 25Mi, chunks of 25Mi", whole, synth.BUCKET_CAP_ELEMS),
                                   ("whole-tensor buckets closed at >= 25Mi, one chunk per bucket", whole, 1 << 28)):
            arr = hfr.make_bucket_array([([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in cuts])
            run = lambda: hfr.hfr_reduce_buckets(arr, len(cuts), Kc, hfr.HFR_BF16, chunk, args.streams, stream)
            _event_time_ms(torch, stream, run, 2, warmup=0)      # the library's on-the-fly placement trials
            ms = _event_time_ms(torch, stream, run, 10, warmup=2)
            lines.append({"config": "cfg3: K=8 bf16, 74 transformer gradient tensors, %d elements in %d %s"
                                    % (total, len(cuts), label), "ms_per_pass": ms, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                          "placement_pattern": hfr.hfr_placement_query([f[:1 << 20] for f in flats], Kc, out[:1 << 20],
                                                                       hfr.HFR_BF16)[2]})
        primary = lines[0]
        primary["buffer_placement"] = ("nine flat buffers in one allocation at the measured stride of %d MiB (hfr_peer_stride: "
                                       "%d MiB)" % (stride >> 20, rule >> 20) if stride else "every flat buffer allocated on its own")
        # the flat buckets follow each other in memory: the library runs them as one sum, cut into
        # equal launches of at most 128 MiB per buffer
        n_launches = -(-total * 2 // (128 << 20))
        primary["roofline"] = {
            "bound": "hbm", "kernel": "reduce_sum_bulk_kernel<BF16Traits, 8, ...>; the %d adjacent buckets of a pass run as "
                                      "%d equal launches of %.1f MiB per buffer" % (len(flat_cuts), n_launches,
                                                                                   total * 2 / n_launches / 2 ** 20),
            "achieved": primary["GBps"], "peak": peak / 1e9, "unit": "GB/s", "frac": primary["GBps"] * 1e9 / peak,
            "traffic": None, "algorithmic_bytes_per_launch": (Kc + 1) * total * 2 / n_launches,
            "avg_launch_ms": primary["ms_per_pass"] / n_launches,
            "note": "pass time / launches: HIP events around 10 whole passes on the launch stream, scheduling gaps included"}
        # the same pass with one launch per bucket (the schedule the merged one is measured against)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, -1)
        arr = hfr.make_bucket_array([([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in flat_cuts])
        ms1 = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_buckets(arr, len(flat_cuts), Kc, hfr.HFR_BF16,
                                                                          synth.BUCKET_CAP_ELEMS, args.streams, stream), 10, warmup=2)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, 0)
        primary["one_launch_per_bucket"] = {"ms_per_pass": ms1, "GBps": b / ms1 / 1e6, "launches": len(flat_cuts)}
        if not args.no_cpu_baseline:
            import oracle
            sample = flat_cuts[:4] + flat_cuts[-1:]              # four full buckets and the ragged last one
            host = [([synth.as_numpy_bits(f[o:o + l]) for f in flats], None) for o, l in sample]
            import numpy as np
            hb = [(ins, np.empty(len(ins[0]), dtype=np.uint16)) for ins, _ in host]
            sb = (Kc + 1) * 2 * sum(l for _, l in sample)
            primary["cpu_baseline"] = oracle_sample_baseline(
                lambda: oracle.reduce_buckets(hb, oracle.BF16), sb,
                "the oracle bucket by bucket on 5 of the 67 buckets (4 full ones and the ragged last, %d bytes moved)" % sb)
            with torch.cuda.stream(stream):
                arr = hfr.make_bucket_array([([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in flat_cuts])
                hfr.hfr_reduce_buckets(arr, len(flat_cuts), Kc, hfr.HFR_BF16, synth.BUCKET_CAP_ELEMS, args.streams, stream)
            stream.synchronize()
            primary["matches_oracle_on_sample"] = all(
                bool(np.array_equal(synth.as_numpy_bits(out[o:o + l]), w[1])) for (o, l), w in zip(sample, hb))
        del flats, out
        torch.cuda.empty_cache()
        if not args.no_placement_spread:
            def run_pass(ins, o):
                cuts = synth.bucket_cuts(total)
                arr2 = hfr.make_bucket_array([([f[a:a + l] for f in ins], o[a:a + l], l) for a, l in cuts])
                hfr.hfr_reduce_buckets(arr2, len(cuts), Kc, hfr.HFR_BF16, synth.BUCKET_CAP_ELEMS, args.streams, stream)
            primary["placement_spread"] = placement_spread(torch, hfr, stream, Kc, total, 64, 10, 33, device, run=run_pass)
        for ln in lines:
            print(json.dumps(ln))
    elif name == "cfg4":
        # Per cell: (a) hfr_reduce_buckets on the contiguous buffers (Algorithm 1's chunk list: adjacent
        # chunks, which the library merges); (a') the same 256 chunks lying 4 KiB apart, which cannot be
        # merged and are folded into batched launches; (a'') one launch per chunk; (b) call (a)
        # captured once into a HIP graph and replayed; (c) the batched entry point (chunk table in the
        # kernel arguments, a handful of launches); (d) the chunk table in device memory (one launch);
        # (e) one plain launch over the whole buffer.
        cells = []
        for Kc in (2, 4, 8, 16):
            for cb in (64 << 10, 256 << 10, 1 << 20, 4 << 20):
                ce = cb // 4
                n = 256 * ce
                ins = synth.peer_buffers_uniform_f32(Kc, n, 4000, device)
                out = torch.empty(n, dtype=torch.float32, device=device)
                arr = hfr.make_bucket_array([(ins, out, n)])
                chunks = hfr.make_bucket_array([([t[c * ce:(c + 1) * ce] for t in ins], out[c * ce:(c + 1) * ce], ce)
                                                for c in range(256)])
                ring = lambda: hfr.hfr_reduce_buckets(arr, 1, Kc, hfr.HFR_F32, ce, 4, stream)
                ms = _event_time_ms(torch, stream, ring, 10, warmup=2)
                one_stream = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_buckets(
                    arr, 1, Kc, hfr.HFR_F32, ce, 1, stream), 10, warmup=2)
                pitch = ce + 1024                                    # 4 KiB between chunks: nothing to merge
                wide_ins = [torch.empty(256 * pitch, dtype=torch.float32, device=device) for _ in range(Kc)]
                wide_out = torch.empty(256 * pitch, dtype=torch.float32, device=device)
                for w, t in zip(wide_ins, ins):
                    w.view(256, pitch)[:, :ce].copy_(t.view(256, ce))
                apart = hfr.make_bucket_array([([w[c * pitch: c * pitch + ce] for w in wide_ins],
                                                wide_out[c * pitch: c * pitch + ce], ce) for c in range(256)])
                torch.cuda.synchronize()
                scattered = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_buckets(
                    apart, 256, Kc, hfr.HFR_F32, ce, 4, stream), 10, warmup=2)
                del wide_ins, wide_out, apart
                hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, -1)     # the schedule before folding: a launch per chunk
                unfolded = _event_time_ms(torch, stream, ring, 10, warmup=2)
                hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, 0)
                one = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(
                    ins, Kc, out, n, hfr.HFR_F32, stream), 10, warmup=2)
                bat = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_buckets_batched(
                    chunks, 256, Kc, hfr.HFR_F32, stream), 10, warmup=2)
                table = hfr.make_chunk_table([([t[c * ce:(c + 1) * ce] for t in ins], out[c * ce:(c + 1) * ce], ce)
                                              for c in range(256)], device)
                tab = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_chunk_table(
                    table, 256, ce, Kc, hfr.HFR_F32, stream), 10, warmup=2)
                graph_ms = None
                try:
                    ref = out.clone()
                    g = torch.cuda.CUDAGraph()
                    torch.cuda.synchronize()
                    with torch.cuda.graph(g, stream=stream):
                        ring()
                    ok = True
                    for _ in range(3):          # replays interleaved with eager work, checked every time
                        out.zero_()
                        g.replay()
                        torch.cuda.synchronize()
                        ok = ok and bool(torch.equal(out.view(torch.int32), ref.view(torch.int32)))
                    if ok:
                        graph_ms = _event_time_ms(torch, stream, g.replay, 10, warmup=2)
                    del g
                except Exception as exc:  # graph capture is an extra, never the product path
                    graph_ms = None
                    sys.stderr.write("graph capture skipped: %r\n" % (exc,))
                b = (Kc + 1) * n * 4
                cells.append({"K": Kc, "chunk_KiB": cb >> 10, "us_per_chunk": ms * 1e3 / 256,
                              "one_stream_us_per_chunk": one_stream * 1e3 / 256,
                              "chunks_4KiB_apart_us_per_chunk": scattered * 1e3 / 256,
                              "launch_per_chunk_us_per_chunk": unfolded * 1e3 / 256,
                              "chunks_per_s": 256 / (ms * 1e-3), "GBps": b / ms / 1e6,
                              "graph_replay_us_per_chunk": None if graph_ms is None else graph_ms * 1e3 / 256,
                              "batched_us_per_chunk": bat * 1e3 / 256, "batched_GBps": b / bat / 1e6,
                              "device_table_us_per_chunk": tab * 1e3 / 256, "device_table_GBps": b / tab / 1e6,
                              "one_launch_us": one * 1e3, "ratio_to_one_launch": ms / one,
                              "batched_ratio_to_one_launch": bat / one})
                del ins, out
        print(json.dumps({"config": "cfg4: fp32, 256 chunks per run through hfr_reduce_buckets on 4 streams (adjacent chunks "
                                    "merged; chunks_4KiB_apart = the same chunks where nothing can be merged: small chunks "
                                    "folded into batched launches); launch_per_chunk = the same call with merging and folding off",
                          "cells": cells}))
    elif name in ("f16", "avg", "e4m3", "e5m2"):
        # the headline shape with fp16 / fp8 storage, and the fused K-way average (bf16)
        Kc, n = 8, 1 << 26
        es = 2
        if name == "f16":
            ins = synth.peer_buffers_normal_f16(Kc, n, 1e-3, 2400, device)
            fn = lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, hfr.HFR_F16, stream)
            label = "K=8 fp16 n=64Mi, hfr_reduce_sum"
        elif name in ("e4m3", "e5m2"):
            n, es = 1 << 27, 1          # 128 MiB per buffer, as the bf16 headline
            ins = synth.peer_buffers_normal_fp8(Kc, n, 1.0, 2600, name, device)
            code = hfr.HFR_FP8_E4M3 if name == "e4m3" else hfr.HFR_FP8_E5M2
            fn = lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, code, stream)
            label = "K=8 fp8 %s n=128Mi (128 MiB per buffer), hfr_reduce_sum" % name
        else:
            ins = synth.peer_buffers_normal_bf16(Kc, n, 1e-3, 2000, device)
            fn = lambda: hfr.hfr_reduce_avg(ins, Kc, out, n, 1.0 / Kc, hfr.HFR_BF16, stream)
            label = "K=8 bf16 n=64Mi, hfr_reduce_avg (sum and mean in one pass)"
        ins, (out,), where = place(torch, hfr, args, ins, 1, device)
        pattern = None
        if not args.no_placement_tuning:
            code = {"f16": hfr.HFR_F16, "avg": hfr.HFR_BF16, "e4m3": hfr.HFR_FP8_E4M3, "e5m2": hfr.HFR_FP8_E5M2}[name]
            _, pattern = hfr.hfr_tune_placement(ins, Kc, out, n, code, stream)
        ms = _event_time_ms(torch, stream, fn, 50, warmup=5)
        b = (Kc + 1) * n * es
        print(json.dumps({"config": label, "us_per_launch": ms * 1e3, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                          "placement_pattern": pattern, "buffer_placement": where}))
    elif name == "msg186":
        # the message size of the paper's allreduce test (Section IV-B: 186 MiB), as K=8 fp32 buffers
        Kc, n = 8, 48758784
        ins, (out,), where = place(torch, hfr, args, synth.peer_buffers_uniform_f32(Kc, n, 6000, device), 1, device)
        pattern = None
        if not args.no_placement_tuning:
            _, pattern = hfr.hfr_tune_placement(ins, Kc, out, n, hfr.HFR_F32, stream)
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, hfr.HFR_F32, stream), 30)
        b = (Kc + 1) * n * 4
        print(json.dumps({"config": "K=8 fp32 n=48,758,784 (186 MiB per buffer), hfr_reduce_sum",
                          "us_per_launch": ms * 1e3, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                          "placement_pattern": pattern, "buffer_placement": where}))
    elif name == "placement":
        # nine 128 MiB buffers cut from one allocation at a uniform spacing: the plain bulk kernel, then the
        # variant hfr_tune_placement records for that placement (same bits; see the header)
        Kc, n = 8, 1 << 26
        mib = 1 << 20
        slab = torch.empty(36 * 1024 * mib // 2, device=device, dtype=torch.bfloat16)
        slab.view(torch.int16).fill_(0x3C00)
        rows = []
        for sp_mib in (128, 129, 130, 256, 258, 512, 1024, 2048, 3342, 4096):
            sp = sp_mib * mib // 2
            ins = [slab[j * sp: j * sp + n] for j in range(Kc)]
            out = slab[Kc * sp: Kc * sp + n]
            run = lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, hfr.HFR_BF16, stream)
            hfr.hfr_shutdown()                      # forget earlier placements
            hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)    # no trial launches inside the plain timing
            plain = _event_time_ms(torch, stream, run, 20)
            hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, 0)
            _, pattern = hfr.hfr_tune_placement(ins, Kc, out, n, hfr.HFR_BF16, stream)
            tuned = _event_time_ms(torch, stream, run, 20)
            b = (Kc + 1) * n * 2
            rows.append({"spacing_MiB": sp_mib, "plain_us": plain * 1e3, "plain_GBps": b / plain / 1e6,
                         "pattern": pattern, "tuned_us": tuned * 1e3, "tuned_GBps": b / tuned / 1e6})
        print(json.dumps({"config": "placement tuning: K=8 bf16 n=64Mi, nine buffers at a uniform spacing in one "
                                    "allocation; plain bulk kernel vs the recorded variant", "cells": rows}))
    elif name == "sweep":
        # library defaults across sizes and input counts (bf16), one line per cell
        rows = []
        pool = [synth.normal_bf16((256 << 20) // 2, 1e-3, 2700 + j, device) for j in range(17)]
        for Kc in (2, 4, 8, 16):
            for mib in (1, 4, 16, 32, 64, 128, 256):
                n = (mib << 20) // 2
                ins = [t[:n] for t in pool[:Kc]]
                outb = pool[16][:n]
                reps = 200 if mib <= 16 else 40
                ms = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(ins, Kc, outb, n, hfr.HFR_BF16, stream), reps)
                b = (Kc + 1) * n * 2
                rows.append({"K": Kc, "MiB_per_buffer": mib, "us": ms * 1e3, "GBps": b / ms / 1e6})
        print(json.dumps({"config": "hfr_reduce_sum, bf16, library defaults, buffers carved from 256 MiB tensors", "cells": rows}))
    elif name == "allk":
        # every input count, bf16 and fp32, 128 MiB per buffer: median over random placements of the K + 1
        # buffers in one slab (the same placements for both columns); library defaults against the shape
        # before request pacing (256 lanes, no pause, no bound on resident workgroups)
        import random
        mib, trials, slab_gib = 128, 6, 40
        unit_b = 2 << 20
        slab = torch.empty((slab_gib << 30) // 2, dtype=torch.bfloat16, device=device)
        slab.view(torch.int16).fill_(0x3A00)
        slab_units, per = (slab_gib << 30) // unit_b, (mib << 20) // unit_b
        hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
        former = ((hfr.HFR_TUNE_BULK_BLOCK, 256), (hfr.HFR_TUNE_BULK_PACE, -1), (hfr.HFR_TUNE_WIDE_WGS_PER_CU, -1))
        rows = []
        for dt_name, code, es, view in (("bf16", hfr.HFR_BF16, 2, torch.bfloat16), ("f32", hfr.HFR_F32, 4, torch.float32)):
            n = (mib << 20) // es
            typed = slab.view(view)
            for Kc in range(1, 17):
                rng = random.Random(1000 + Kc)
                rates = {"default": [], "former": []}
                for _ in range(trials):
                    while True:
                        starts = sorted(rng.randrange(0, slab_units - per) for _ in range(Kc + 1))
                        if all(b - a >= per for a, b in zip(starts, starts[1:])):
                            break
                    rng.shuffle(starts)
                    bufs = [typed[u * (unit_b // es): u * (unit_b // es) + n] for u in starts]
                    ins, outb = bufs[:Kc], bufs[Kc]
                    for mode in ("default", "former"):
                        for knob, v in former:
                            hfr.hfr_set_tuning(knob, v if mode == "former" else 0)
                        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(ins, Kc, outb, n, code, stream), 10, warmup=2)
                        rates[mode].append((Kc + 1) * n * es / ms / 1e6)
                med = lambda v: sorted(v)[len(v) // 2]
                rows.append({"dtype": dt_name, "K": Kc, "GBps": med(rates["default"]), "min_GBps": min(rates["default"]),
                             "former_shape_GBps": med(rates["former"]), "former_shape_min_GBps": min(rates["former"])})
        for knob, _ in former:
            hfr.hfr_set_tuning(knob, 0)
        print(json.dumps({"config": "hfr_reduce_sum, every K, 128 MiB per buffer, median over %d random placements in a %d GiB "
                                    "slab; former_shape = 256 lanes, no pause, no bound on resident workgroups" % (trials, slab_gib),
                          "cells": rows}))
    elif name == "slice":
        # the share of one GPU in the sharded form: rank r sums slice r of `world` out of the K full
        # buffers; all eight slices in turn cover the buffer, so the pass compares with one launch
        Kc, n, world = 8, 1 << 26, 8
        ins, (out,), where = place(torch, hfr, args, synth.peer_buffers_normal_bf16(Kc, n, 1e-3, 2000, device), 1, device)
        b = (Kc + 1) * n * 2
        def all_slices():
            for r in range(world):
                hfr.hfr_reduce_scatter_slice(ins, Kc, out, n, r, world, hfr.HFR_BF16, stream)
        one = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_scatter_slice(ins, Kc, out, n, 3, world, hfr.HFR_BF16, stream), 200)
        ms = _event_time_ms(torch, stream, all_slices, 50, warmup=5)
        whole = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, hfr.HFR_BF16, stream), 50, warmup=5)
        print(json.dumps({"config": "K=8 bf16 n=64Mi, hfr_reduce_scatter_slice with world=8 (16 MiB per buffer and slice)",
                          "us_per_slice": one * 1e3, "slice_GBps": b / world / one / 1e6,
                          "us_all_eight_slices": ms * 1e3, "all_slices_GBps": b / ms / 1e6,
                          "us_whole_buffer_one_call": whole * 1e3, "whole_GBps": b / whole / 1e6,
                          "buffer_placement": where}))
    elif name == "apart":
        # gradient buckets that are allocations of their own (25 MiB per buffer, the default bucket size of
        # PyTorch's DistributedDataParallel), so that nothing can be merged: bulk launches over a list of
        # chunks against one launch per bucket
        Kc, nb, count = 8, 25 << 20, 40
        n = nb // 2
        pitch = nb + 4096
        bufs = [torch.empty(count * pitch, dtype=torch.uint8, device=device) for _ in range(Kc + 1)]
        for j, bb in enumerate(bufs[:Kc]):
            bb.view(torch.bfloat16).copy_(synth.normal_bf16(count * pitch // 2, 1e-3, 7000 + j, device))
        arr = hfr.make_bucket_array([([bb[c * pitch: c * pitch + nb].view(torch.bfloat16) for bb in bufs[:Kc]],
                                      bufs[Kc][c * pitch: c * pitch + nb].view(torch.bfloat16), n) for c in range(count)])
        run = lambda: hfr.hfr_reduce_buckets(arr, count, Kc, hfr.HFR_BF16, 1 << 40, args.streams, stream)
        b = (Kc + 1) * nb * count
        res = {}
        for label, knob in (("default", 0), ("one_launch_per_bucket", -1), ("list_launches_forced", 1)):
            hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_LIST, knob)
            _event_time_ms(torch, stream, run, 2, warmup=0)      # on-the-fly placement trials
            ms = _event_time_ms(torch, stream, run, 10, warmup=2)
            res[label] = {"ms_per_pass": ms, "GBps": b / ms / 1e6}
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_LIST, 0)
        pattern = hfr.hfr_placement_query([bb[:nb].view(torch.bfloat16) for bb in bufs[:Kc]], Kc, bufs[Kc][:nb].view(torch.bfloat16),
                                          hfr.HFR_BF16)[2]
        print(json.dumps({"config": "K=8 bf16, 40 buckets of 25 MiB per buffer lying 4 KiB apart (nothing to merge), "
                                    "hfr_reduce_buckets; default = list launches where the placement table holds pattern 0, "
                                    "else a launch per bucket with the recorded variant",
                          "placement_pattern": pattern, "bytes_moved": b, **res}))
    elif name == "bcast":
        Kc, n = 8, 1 << 26
        src = synth.normal_bf16(n, 1e-3, 2500, device)
        dsts = [torch.empty_like(src) for _ in range(Kc)]
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_broadcast(src, dsts, Kc, n, hfr.HFR_BF16, stream), 30)
        b = (Kc + 1) * n * 2
        print(json.dumps({"config": "broadcast of one bf16 buffer of 64Mi elements to K=8 destinations (1 read, 8 writes)",
                          "us_per_launch": ms * 1e3, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b}))
    elif name == "ceilings":
        print(json.dumps(measure_ceilings(torch, device, stream, full=True)))
    elif name == "cfg5":
        n = 1 << 28
        (a, b_), (out,), where = place(torch, hfr, args, [synth.normal_f32(n, 1.0, 5000, device),
                                                           synth.normal_f32(n, 1.0, 5001, device)], 1, device)
        torch.cuda.empty_cache()
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_combine_avg(a, b_, out, n, SCALE, hfr.HFR_F32, stream), 30)
        b = 3 * n * 4
        seg = 256 << 20                                          # bytes per buffer of one launch of this call
        line = {"config": "cfg5: combine-and-average fp32 n=256Mi, scale 2^-7", "us_per_launch": ms * 1e3,
                "GBps": b / ms / 1e6, "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                "buffer_placement": where,
                "roofline": {"bound": "hbm", "kernel": "combine_avg_kernel<F32Traits, 4, ...>, %d launches of 256 MiB per buffer per call"
                                                       % (n * 4 // seg),
                             "achieved": b / ms / 1e6, "peak": peak / 1e9, "unit": "GB/s", "frac": b / (ms * 1e-3) / peak,
                             "traffic": None, "algorithmic_bytes_per_launch": 3 * seg,
                             "avg_launch_ms": ms / (n * 4 // seg),
                             "note": "call time / launches: HIP events around 30 whole calls on the launch stream"}}
        if not args.no_cpu_baseline:
            import numpy as np
            import oracle
            m = 1 << 26                                          # a quarter of the workload
            ha, hb = synth.as_numpy_bits(a[:m]), synth.as_numpy_bits(b_[:m])
            ho = np.empty(m, dtype=np.float32)
            line["cpu_baseline"] = oracle_sample_baseline(
                lambda: oracle.combine_avg(ha, hb, SCALE, oracle.F32, out=ho), 3 * m * 4,
                "the oracle on the first 2^26 of the 2^28 elements (%d bytes moved)" % (3 * m * 4))
            stream.synchronize()
            line["matches_oracle_on_sample"] = bool(np.array_equal(synth.as_numpy_bits(out[:m]), ho))
        print(json.dumps(line))
    else:
        print("unknown --config %r" % name, file=sys.stderr)
        return 2
    return 0


def main():
    global PREHEAT_MS
    args = parse_args()
    PREHEAT_MS = max(0.0, args.preheat_ms)
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the K peer buffers live in one GPU's HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2408_14158_amd import hfr, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; libhfr has no CPU fallback", file=sys.stderr)
        return 3
    hfr.lib()  # fail loudly if the HIP library is not built
    device = "cuda:0"
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    # what the driver reports: memory clock and bus width
    _, mem_khz, bus_bits = hfr.hfr_device_info()
    # one transfer per reported clock; the published 8 TB/s is the roofline's denominator whatever this reads
    reported_peak = mem_khz * 1e3 * (bus_bits / 8) / 1e9 if mem_khz and bus_bits else None

    if args.config:
        stream = torch.cuda.Stream()
        if args.no_placement_tuning:
            hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
        rc = run_other_config(args, torch, hfr, synth, device, stream)
        hfr.hfr_shutdown()
        return rc

    # a profiling run of the headline kernel takes the rule's stride as it is: the timing launches of the
    # measured form are launches of that same kernel and would mix into its trace
    ins, remote, out, out_fused, arena = make_inputs(torch, hfr, synth, device, arena=not args.separate_allocations,
                                                     measure=not args.roofline_only)
    torch.cuda.synchronize()  # the generators and the copies ran on the default stream
    cuts = synth.bucket_cuts(N_ELEMS)
    chunk_elems = args.chunk_elems if args.chunk_elems > 0 else synth.BUCKET_CAP_ELEMS
    bucket_arr = hfr.make_bucket_array([([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts])
    stream = torch.cuda.Stream()
    hfr.hfr_init()

    reduce_bytes = (K + 1) * N_ELEMS * ELEM
    step_bytes = reduce_bytes + 3 * N_ELEMS * ELEM

    if args.no_placement_tuning:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)

    def settle(fn, passes=14):
        """Untimed set-up passes: the library measures an unseen buffer placement
        on the fly during its first twelve bulk launches (no host block), as it
        would during the first iterations of a training loop."""
        with torch.cuda.stream(stream):
            for _ in range(passes):
                fn()
        stream.synchronize()

    if args.roofline_only:
        settle(lambda: hfr.hfr_reduce_sum(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream))
        avg_ms, med_ms, best_ms = time_dominant_kernel(torch, hfr, ins, out, stream, args.roofline_launches)
        if args.with_copy:
            # a plain copy of known size (K = 1: 128 MiB read, 128 MiB written) for scaling the counters
            with torch.cuda.stream(stream):
                for _ in range(args.roofline_launches):
                    hfr.hfr_reduce_sum(ins[:1], 1, out, N_ELEMS, hfr.HFR_BF16, stream)
            stream.synchronize()
        print(json.dumps({"kernel": "reduce_sum K=8 bf16 n=64Mi", "launches": args.roofline_launches,
                          "avg_ms": avg_ms, "single_pair_median_ms": med_ms, "single_pair_best_ms": best_ms,
                          "GBps": reduce_bytes / (avg_ms * 1e-3) / 1e9,
                          "placement_pattern": hfr.hfr_placement_query(ins, K, out, hfr.HFR_BF16)[2]}))
        return 0

    def reduce_part():
        hfr.hfr_reduce_buckets(bucket_arr, len(cuts), K, hfr.HFR_BF16, chunk_elems, args.streams, stream)

    def step():
        reduce_part()
        hfr.hfr_combine_avg(out, remote, out, N_ELEMS, SCALE, hfr.HFR_BF16, stream)

    if not args.no_placement_tuning:
        settle(step, 7)     # two trial launches per step
    _preheat(torch, stream, step, PREHEAT_MS)
    with torch.cuda.stream(stream):
        for _ in range(args.warmup):
            step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    with torch.cuda.stream(stream):
        for _ in range(args.steps):
            step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    step_GBps = step_bytes / (elapsed / args.steps) / 1e9
    # the K-way reduction of the same steps on its own (the metric is defined on it): the same number of
    # passes, one HIP event pair on the launch stream around all of them (events between the kernels of a
    # step would open gaps of several microseconds each)
    reduce_ms = _event_time_ms(torch, stream, reduce_part, args.steps, warmup=2)
    value = reduce_bytes / (reduce_ms * 1e-3) / 1e9

    st, state, pattern = hfr.hfr_placement_query(ins, K, out, hfr.HFR_BF16)
    placement = {"what": "buffer placement measured by the library on the fly during the untimed set-up passes "
                         "(state 2 = recorded; pattern 0 = plain kernel, 1-3 = skewed variant)",
                 "state": state, "pattern": pattern}
    if not args.no_placement_tuning:
        # the same loop with the plain kernels only, for comparison (after the timed region)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, -1)
        _preheat(torch, stream, step, PREHEAT_MS)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        with torch.cuda.stream(stream):
            for _ in range(args.steps):
                step()
        torch.cuda.synchronize()
        plain_ms = (time.perf_counter() - t1) * 1e3 / args.steps
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, 0)
        placement["plain_kernels_ms_per_step"] = plain_ms
        placement["plain_kernels_step_GBps"] = step_bytes / (plain_ms * 1e-3) / 1e9

    avg_ms, med_ms, best_ms = time_dominant_kernel(torch, hfr, ins, out, stream, args.roofline_launches)
    achieved = reduce_bytes / (avg_ms * 1e-3) / 1e9

    # The same step through the fused entry point (sum and combine in one kernel): the node partial never
    # goes to HBM and back, so a step moves (K + 2) * n * 2 bytes. Reported beside `value`, as one call
    # over the buffers (what the merged bucket list of the step amounts to) and as one call per bucket.
    def fused_step():
        hfr.hfr_reduce_combine_avg(ins, K, remote, out_fused, N_ELEMS, SCALE, hfr.HFR_BF16, stream)
    def fused_step_per_bucket():
        for o, l in cuts:
            hfr.hfr_reduce_combine_avg([t[o:o + l] for t in ins], K, remote[o:o + l], out_fused[o:o + l], l,
                                       SCALE, hfr.HFR_BF16, stream)
    if not args.no_placement_tuning:
        settle(fused_step, 14)
    fused_ms = _event_time_ms(torch, stream, fused_step, args.steps, warmup=args.warmup)
    fused_bucket_ms = _event_time_ms(torch, stream, fused_step_per_bucket, args.steps, warmup=args.warmup)
    fused_bytes = (K + 2) * N_ELEMS * ELEM

    # the same launch on buffers that torch's allocator placed one by one
    separate = None
    if arena is not None:
        sep_ins, sep_out = arena["separate"]
        settle(lambda: hfr.hfr_reduce_sum(sep_ins, K, sep_out, N_ELEMS, hfr.HFR_BF16, stream))
        sep_ms, _, _ = time_dominant_kernel(torch, hfr, sep_ins, sep_out, stream, args.roofline_launches)
        separate = {"what": "the roofline launch on nine separately allocated buffers (torch's allocator; where they land "
                            "differs from process to process), after on-the-fly placement tuning",
                    "avg_launch_ms": sep_ms, "GBps": reduce_bytes / (sep_ms * 1e-3) / 1e9,
                    "placement_pattern": hfr.hfr_placement_query(sep_ins, K, sep_out, hfr.HFR_BF16)[2]}
        del sep_ins, sep_out
        arena["separate"] = None

    # what HBM delivers on this machine for the same traffic in plain streaming passes
    ceil = measure_ceilings(torch, device, stream, full=False, reps=10)["cells"]
    ceiling_sum = composite_ceiling(ceil, K, 1)

    traffic = None
    if os.path.exists(args.traffic_file):
        try:
            with open(args.traffic_file) as f:
                for line in f:
                    if line.strip().startswith("hbm_bytes_per_launch"):
                        traffic = float(line.split("=")[1].split()[0])
        except (OSError, ValueError, IndexError):
            traffic = None

    result = {
        "metric": "reduced GB/s (bytes moved = (K+1)*n*2) of the K-way reduction, K=8 bf16 n=64Mi, 1 GPU",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "preheat_ms": PREHEAT_MS,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: K=8 bf16 gradient buffers, n=67108864 each, N(0,1e-3); "
                        "step = bucketed K-way sum (25Mi-element buckets through hfr_reduce_buckets, %d streams) "
                        "+ combine-and-average; buffers %s" % (args.streams, (
                            "carved from one allocation at the measured stride of %d MiB" % (arena["stride"] >> 20)) if arena
                            else "allocated one by one"),
            "K": K, "n": N_ELEMS, "storage": "bf16", "accumulate": "f32",
            "bucket_elems": synth.BUCKET_CAP_ELEMS, "chunk_elems": chunk_elems, "streams": args.streams,
            "bytes_per_reduction": reduce_bytes, "bytes_per_step": step_bytes,
            "device": props.name, "compute_units": props.multi_processor_count,
            "device_reported_clock_x_bus_GBps": reported_peak, "memory_clock_kHz": mem_khz, "memory_bus_bits": bus_bits,
        },
        "pct_of_hbm_peak": 100.0 * value * 1e9 / HBM_PEAK_BYTES_PER_S,
        "value_is": "(K+1)*n*2 bytes / reduce_ms_per_step: the bucketed K-way reduction of the timed steps (hfr_reduce_buckets "
                    "over the three buckets, which lie one after the other in the buffers and are merged into one launch) run on its own for the same number of passes, one HIP event pair on the launch "
                    "stream around them; `step` and ms_per_step are the whole hot path (sum + combine), wall clock",
        "reduce_ms_per_step": reduce_ms,
        "step": {
            "what": "whole hot path: bucketed K-way sum + combine-and-average in place, wall clock over the timed steps",
            "ms_per_step": ms_per_step, "bytes_per_step": step_bytes, "GBps": step_GBps,
            "pct_of_hbm_peak": 100.0 * step_GBps * 1e9 / HBM_PEAK_BYTES_PER_S,
        },
        "placement_tuning": placement,
        "buffer_placement": {
            "what": "inputs, output and remote partial lie in one allocation (a staging arena owned by the caller of the "
                    "reduction) at the distance hfr_tune_peer_stride measured on it: hfr_peer_stride's value unless a "
                    "neighbouring distance is more than 1.5 % faster" if arena else "every buffer allocated on its own",
            "stride_bytes": arena["stride"] if arena else None,
            "hfr_peer_stride_bytes": arena["rule"] if arena else None,
            "base_address_mod_2MiB": (ins[0].data_ptr() % (2 << 20)) if arena else None,
            "separate_allocations": separate,
        },
        "fused_step": {
            "what": "the same step through hfr_reduce_combine_avg (one call over the buffers, bit-identical output; "
                    "per_bucket = one call per 25Mi-element bucket)",
            "ms_per_step": fused_ms, "bytes_per_step": fused_bytes,
            "per_bucket_ms_per_step": fused_bucket_ms, "per_bucket_GBps": fused_bytes / (fused_bucket_ms * 1e-3) / 1e9,
            "GBps": fused_bytes / (fused_ms * 1e-3) / 1e9, "speedup_vs_step": ms_per_step / fused_ms,
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "hfr_reduce_sum K=8 bf16 on the full 64Mi buffers, one launch of reduce_sum_bulk_kernel<BF16Traits, 8, ...>",
            "achieved": achieved,
            "peak": HBM_PEAK_BYTES_PER_S / 1e9,
            "unit": "GB/s",
            "frac": achieved * 1e9 / HBM_PEAK_BYTES_PER_S,
            "traffic": traffic,
            "traffic_source": "%s (committed rocprofv3 --pmc summary; not measured in this run)"
                              % os.path.relpath(args.traffic_file, ROOT) if traffic is not None else None,
            "algorithmic_bytes_per_launch": reduce_bytes,
            "avg_launch_ms": avg_ms, "single_launch_event_pair_median_ms": med_ms,
            "single_launch_event_pair_best_ms": best_ms,
            "launches": args.roofline_launches,
            "measured_ceiling_GBps": ceiling_sum,
            "frac_of_measured_ceiling": achieved / ceiling_sum,
            "measured_ceiling_probe": "serial model from two streaming probes timed in this run (libhfr_probe, 128 MiB "
                                      "per buffer): 8 parts read at the read-only rate of eight streams (%.0f GB/s) + 1 part "
                                      "written at the fill rate (%.0f GB/s); the 8-read:1-write XOR probe itself: %.0f GB/s"
                                      % (ceil["read_only_8_streams"]["best_GBps"], ceil["fill"]["best_GBps"],
                                         ceil["mix_8r_1w"]["best_GBps"]),
        },
    }
    if not args.no_placement_spread:
        result["placement_spread"] = placement_spread(torch, hfr, stream, K, N_ELEMS, 24, 12, 21, device)

    if not args.no_cpu_baseline:
        base, host_out = cpu_baseline(torch, synth, ins, remote, cuts)
        result["cpu_baseline"] = base
        # the step's GPU result must be the oracle's, bit for bit
        with torch.cuda.stream(stream):
            step()
        torch.cuda.synchronize()
        import numpy as np
        got = synth.as_numpy_bits(out)
        result["matches_oracle"] = bool(np.array_equal(got, host_out))
        out_fused.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            fused_step()
        torch.cuda.synchronize()
        result["fused_step"]["matches_oracle"] = bool(np.array_equal(synth.as_numpy_bits(out_fused), host_out))

    hfr.hfr_shutdown()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
