#!/usr/bin/env python3
"""Benchmark of libhfr on one MI355X.

A step is one pass of the whole hot path over one synthetic gradient batch of
the headline workload (K = 8 peer buffers, bf16, n = 64 Mi elements each):

  1. hfr_reduce_buckets: the flat gradient cut into 25 Mi-element buckets,
     every bucket reduced K-way in fp32 (in buffer order) and stored as bf16,
     chunk-pipelined over 4 HIP streams              -> (K+1) * n * 2 bytes
  2. hfr_combine_avg: the node partial combined with a received remote partial
     and scaled by 1 / (8 * 16), in place             -> 3 * n * 2 bytes

`value` is bytes moved per second over whole steps, inputs resident in HBM.
`roofline` times the dominant kernel (the K-way bf16 sum over the full 64 Mi
buffer, one launch) with HIP events on its launch stream; `cpu_baseline` times
the CPU oracle on the same step on this host.

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
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--roofline-only", action="store_true",
                    help="run only the dominant-kernel launches (for rocprofv3 runs)")
    ap.add_argument("--roofline-launches", type=int, default=50)
    ap.add_argument("--config", default="",
                    help="instead of the default step, time one of the other workloads and print its own JSON "
                         "line: cfg1 (K=8 fp32 n=1Mi), cfg3 (bucketed transformer gradients), cfg4 (latency "
                         "regime table), cfg5 (combine, fp32 n=256Mi), f16 (headline shape in fp16), "
                         "sweep (sizes x K table), placement (plain vs tuned kernel at ten buffer spacings), msg186 (186 MiB fp32 message), e4m3 / e5m2 (fp8, 128 MiB per buffer), avg (fused K-way average), bcast (1-to-8 broadcast)")
    ap.add_argument("--no-placement-tuning", action="store_true",
                    help="skip hfr_tune_placement in the set-up: time the plain kernels whatever the buffers' placement")
    ap.add_argument("--with-copy", action="store_true",
                    help="with --roofline-only: also launch the K=1 copy of one 128 MiB buffer (counter calibration)")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "reduce_sum_k8_bf16_64mi_hbm_traffic.txt"),
                    help="summary of the committed rocprofv3 counter runs; its hbm_bytes_per_launch line is reported")
    return ap.parse_args()


def make_inputs(torch, synth, device):
    ins = synth.peer_buffers_normal_bf16(K, N_ELEMS, 1e-3, 2000, device)
    remote = synth.normal_bf16(N_ELEMS, 1e-3 * (K ** 0.5), 2100, device)
    out = torch.empty(N_ELEMS, dtype=torch.bfloat16, device=device)
    return ins, remote, out


def time_dominant_kernel(torch, hfr, ins, out, stream, launches, warmup=5):
    """Average duration of one K=8 bf16 64 Mi launch, with HIP events recorded
    on the stream the kernel is launched on: one event pair around `launches`
    back-to-back launches (kernels on one stream start when the previous one
    ends, so elapsed / launches is the average launch duration). A second pass
    puts an event pair around every single launch; those figures include the
    event-to-kernel dispatch gap and are reported beside the average."""
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


def _event_time_ms(torch, stream, fn, reps, warmup=3):
    """Average ms per call of fn, HIP events on `stream`. Synchronises the
    device first: the input generators ran on another stream."""
    torch.cuda.synchronize()
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
        flats = [synth.flat_gradient_bf16(tensors, 3000 + j, device) for j in range(Kc)]
        out = torch.empty(total, dtype=torch.bfloat16, device=device)
        b = (Kc + 1) * total * 2
        # primary packing: flat cuts every 25Mi elements; secondary: whole tensors, greedy
        whole = synth.bucket_cuts_whole_tensors(tensors)
        pattern = None
        if not args.no_placement_tuning:   # once for the eight flat gradient buffers; every bucket shares the placement
            _, pattern = hfr.hfr_tune_placement(flats, Kc, out, 1 << 26, hfr.HFR_BF16, stream)
        for label, cuts, chunk in (("flat buckets of 25Mi", synth.bucket_cuts(total), synth.BUCKET_CAP_ELEMS),
                                   ("whole-tensor buckets closed at >= 25Mi, chunks of 25Mi", whole, synth.BUCKET_CAP_ELEMS),
                                   ("whole-tensor buckets closed at >= 25Mi, one chunk per bucket", whole, 1 << 28)):
            arr = hfr.make_bucket_array([([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in cuts])
            ms = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_buckets(
                arr, len(cuts), Kc, hfr.HFR_BF16, chunk, args.streams, stream), 10, warmup=2)
            print(json.dumps({"config": "cfg3: K=8 bf16, 74 transformer gradient tensors, %d elements in %d %s"
                                        % (total, len(cuts), label), "ms_per_pass": ms, "GBps": b / ms / 1e6,
                              "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                              "placement_pattern": pattern}))
    elif name == "cfg4":
        # Per cell: (a) the stream-ring schedule, one launch per chunk; (b) the same call captured
        # once into a HIP graph and replayed; (c) the batched entry point (chunk table in the kernel
        # arguments, a handful of launches); (d) the chunk table in device memory (one launch);
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
                              "launch_per_chunk_us_per_chunk": unfolded * 1e3 / 256,
                              "chunks_per_s": 256 / (ms * 1e-3), "GBps": b / ms / 1e6,
                              "graph_replay_us_per_chunk": None if graph_ms is None else graph_ms * 1e3 / 256,
                              "batched_us_per_chunk": bat * 1e3 / 256, "batched_GBps": b / bat / 1e6,
                              "device_table_us_per_chunk": tab * 1e3 / 256, "device_table_GBps": b / tab / 1e6,
                              "one_launch_us": one * 1e3, "ratio_to_one_launch": ms / one,
                              "batched_ratio_to_one_launch": bat / one})
                del ins, out
        print(json.dumps({"config": "cfg4: fp32, 256 chunks per run through hfr_reduce_buckets on 4 streams (small chunks "
                                    "folded into batched launches); launch_per_chunk = the same call with folding off",
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
        out = torch.empty_like(ins[0])
        pattern = None
        if not args.no_placement_tuning:
            code = {"f16": hfr.HFR_F16, "avg": hfr.HFR_BF16, "e4m3": hfr.HFR_FP8_E4M3, "e5m2": hfr.HFR_FP8_E5M2}[name]
            _, pattern = hfr.hfr_tune_placement(ins, Kc, out, n, code, stream)
        ms = _event_time_ms(torch, stream, fn, 50, warmup=5)
        b = (Kc + 1) * n * es
        print(json.dumps({"config": label, "us_per_launch": ms * 1e3, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                          "placement_pattern": pattern}))
    elif name == "msg186":
        # the message size of the paper's allreduce test (Section VI-B: 186 MiB), as K=8 fp32 buffers
        Kc, n = 8, 48758784
        ins = synth.peer_buffers_uniform_f32(Kc, n, 6000, device)
        out = torch.empty(n, dtype=torch.float32, device=device)
        pattern = None
        if not args.no_placement_tuning:
            _, pattern = hfr.hfr_tune_placement(ins, Kc, out, n, hfr.HFR_F32, stream)
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_reduce_sum(ins, Kc, out, n, hfr.HFR_F32, stream), 30)
        b = (Kc + 1) * n * 4
        print(json.dumps({"config": "K=8 fp32 n=48,758,784 (186 MiB per buffer), hfr_reduce_sum",
                          "us_per_launch": ms * 1e3, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b,
                          "placement_pattern": pattern}))
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
            plain = _event_time_ms(torch, stream, run, 20)
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
    elif name == "bcast":
        Kc, n = 8, 1 << 26
        src = synth.normal_bf16(n, 1e-3, 2500, device)
        dsts = [torch.empty_like(src) for _ in range(Kc)]
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_broadcast(src, dsts, Kc, n, hfr.HFR_BF16, stream), 30)
        b = (Kc + 1) * n * 2
        print(json.dumps({"config": "broadcast of one bf16 buffer of 64Mi elements to K=8 destinations (1 read, 8 writes)",
                          "us_per_launch": ms * 1e3, "GBps": b / ms / 1e6,
                          "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b}))
    elif name == "cfg5":
        n = 1 << 28
        a = synth.normal_f32(n, 1.0, 5000, device)
        b_ = synth.normal_f32(n, 1.0, 5001, device)
        out = torch.empty_like(a)
        ms = _event_time_ms(torch, stream, lambda: hfr.hfr_combine_avg(a, b_, out, n, SCALE, hfr.HFR_F32, stream), 30)
        b = 3 * n * 4
        print(json.dumps({"config": "cfg5: combine-and-average fp32 n=256Mi, scale 2^-7", "us_per_launch": ms * 1e3,
                          "GBps": b / ms / 1e6, "pct_of_hbm_peak": 100 * b / (ms * 1e-3) / peak, "bytes_moved": b}))
    else:
        print("unknown --config %r" % name, file=sys.stderr)
        return 2
    return 0


def main():
    args = parse_args()
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
        rc = run_other_config(args, torch, hfr, synth, device, stream)
        hfr.hfr_shutdown()
        return rc

    ins, remote, out = make_inputs(torch, synth, device)
    torch.cuda.synchronize()  # the generators ran on the default stream
    cuts = synth.bucket_cuts(N_ELEMS)
    chunk_elems = args.chunk_elems if args.chunk_elems > 0 else synth.BUCKET_CAP_ELEMS
    bucket_arr = hfr.make_bucket_array([([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts])
    stream = torch.cuda.Stream()
    hfr.hfr_init()

    reduce_bytes = (K + 1) * N_ELEMS * ELEM
    step_bytes = reduce_bytes + 3 * N_ELEMS * ELEM

    if args.roofline_only:
        if not args.no_placement_tuning:
            hfr.hfr_tune_placement(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream)
        avg_ms, med_ms, best_ms = time_dominant_kernel(torch, hfr, ins, out, stream, args.roofline_launches)
        if args.with_copy:
            # a plain copy of known size (K = 1: 128 MiB read, 128 MiB written) for scaling the counters
            with torch.cuda.stream(stream):
                for _ in range(args.roofline_launches):
                    hfr.hfr_reduce_sum(ins[:1], 1, out, N_ELEMS, hfr.HFR_BF16, stream)
            stream.synchronize()
        print(json.dumps({"kernel": "reduce_sum K=8 bf16 n=64Mi", "launches": args.roofline_launches,
                          "avg_ms": avg_ms, "single_pair_median_ms": med_ms, "single_pair_best_ms": best_ms,
                          "GBps": reduce_bytes / (avg_ms * 1e-3) / 1e9}))
        return 0

    def step():
        hfr.hfr_reduce_buckets(bucket_arr, len(cuts), K, hfr.HFR_BF16, chunk_elems, args.streams, stream)
        hfr.hfr_combine_avg(out, remote, out, N_ELEMS, SCALE, hfr.HFR_BF16, stream)

    # Set-up, outside the timed region, as a training loop would do once for its gradient buffers:
    # let the library time its kernel variants on these buffers' placement (K peers, and K peers plus
    # the remote partial for the fused entry point). The untimed-variant figure is reported beside it.
    placement = None
    if not args.no_placement_tuning:
        _, pat_k = hfr.hfr_tune_placement(ins, K, out, N_ELEMS, hfr.HFR_BF16, stream)
        _, pat_k1 = hfr.hfr_tune_placement(list(ins) + [remote], K + 1, out, N_ELEMS, hfr.HFR_BF16, stream)
        placement = {"what": "hfr_tune_placement once before the warm-up (not timed); skew pattern recorded for "
                             "the K peers / for the K peers plus the remote partial (0 = plain kernel)",
                     "pattern_k_inputs": pat_k, "pattern_k_plus_remote": pat_k1}

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
    value = step_bytes / (elapsed / args.steps) / 1e9

    if placement is not None:
        # the same loop with the plain kernels only, for comparison (after the timed region)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, -1)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        with torch.cuda.stream(stream):
            for _ in range(args.steps):
                step()
        torch.cuda.synchronize()
        plain_ms = (time.perf_counter() - t1) * 1e3 / args.steps
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, 0)
        placement["plain_kernels_ms_per_step"] = plain_ms
        placement["plain_kernels_GBps"] = step_bytes / (plain_ms * 1e-3) / 1e9

    avg_ms, med_ms, best_ms = time_dominant_kernel(torch, hfr, ins, out, stream, args.roofline_launches)
    achieved = reduce_bytes / (avg_ms * 1e-3) / 1e9

    # The same step through the fused entry point (sum and combine in one kernel per bucket): the node
    # partial never goes to HBM and back, so a step moves (K + 2) * n * 2 bytes. Reported beside `value`.
    out_fused = torch.empty_like(out)
    def fused_step():
        for o, l in cuts:
            hfr.hfr_reduce_combine_avg([t[o:o + l] for t in ins], K, remote[o:o + l], out_fused[o:o + l], l,
                                       SCALE, hfr.HFR_BF16, stream)
    fused_ms = _event_time_ms(torch, stream, fused_step, args.steps, warmup=args.warmup)
    fused_bytes = (K + 2) * N_ELEMS * ELEM

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
        "metric": "reduced GB/s (bytes moved), K=8 bf16 n=64Mi, 1 GPU",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": "configs[1]: K=8 bf16 gradient buffers, n=67108864 each, N(0,1e-3); "
                        "step = bucketed K-way sum (25Mi-element buckets, %d streams) + combine-and-average"
                        % args.streams,
            "K": K, "n": N_ELEMS, "storage": "bf16", "accumulate": "f32",
            "bucket_elems": synth.BUCKET_CAP_ELEMS, "chunk_elems": chunk_elems, "streams": args.streams,
            "bytes_per_step": step_bytes,
            "device": props.name, "compute_units": props.multi_processor_count,
            "device_reported_clock_x_bus_GBps": reported_peak, "memory_clock_kHz": mem_khz, "memory_bus_bits": bus_bits,
        },
        "pct_of_hbm_peak": 100.0 * value * 1e9 / HBM_PEAK_BYTES_PER_S,
        "placement_tuning": placement,
        "fused_step": {
            "what": "the same step through hfr_reduce_combine_avg (one kernel per bucket, bit-identical output)",
            "ms_per_step": fused_ms, "bytes_per_step": fused_bytes,
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
            "algorithmic_bytes_per_launch": reduce_bytes,
            "avg_launch_ms": avg_ms, "single_launch_event_pair_median_ms": med_ms,
            "single_launch_event_pair_best_ms": best_ms,
            "launches": args.roofline_launches,
        },
    }

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
        result["fused_step"]["matches_oracle"] = bool(np.array_equal(synth.as_numpy_bits(out_fused), host_out))

    hfr.hfr_shutdown()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
