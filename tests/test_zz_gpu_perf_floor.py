"""Throughput floors, far below what the kernels reach (about 75 % of it), so
that a launch shape that silently stopped working - a fallback to a slow path,
loads serialised by a compiler change - fails a test instead of only showing up
in the benchmark. Every floor is a ratio to a plain launch timed in the same
run, not an absolute figure: boxes of one pool differ. Collected after the
parity tests."""
import pytest
import torch

from paper_2408_14158_amd import hfr, synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _median_us(fn, stream, reps=15, warm=4):
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        for _ in range(warm):
            fn()
        pairs = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fn()
            b.record(stream)
            pairs.append((a, b))
    stream.synchronize()
    ms = sorted(x.elapsed_time(y) for x, y in pairs)
    return ms[len(ms) // 2] * 1e3


def test_headline_sum_combine_and_broadcast_floors():
    """Floors relative to a plain copy (K = 1, 128 MiB in, 128 MiB out) timed in
    the same run on the same box: boxes of one pool differ by several per cent,
    the ratios between kernels on one box do not."""
    K, n = 8, 1 << 26
    s = torch.cuda.Stream()
    ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 2000, DEV)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    remote = synth.normal_bf16(n, 1e-3, 2100, DEV)
    us = _median_us(lambda: hfr.hfr_reduce_sum(ins[:1], 1, out, n, hfr.HFR_BF16, s), s)
    copy = 2 * n * 2 / us / 1e6
    assert copy > 2.0, "K=1 copy of 128 MiB: %.2f TB/s (%.1f us)" % (copy, us)     # sanity only: any working GPU
    for _ in range(14):                       # the library's on-the-fly placement trials, untimed
        hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16, s)
        hfr.hfr_reduce_combine_avg(ins, K, remote, out, n, 1.0 / 128, hfr.HFR_BF16, s)
    us = _median_us(lambda: hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16, s), s)
    tbps = (K + 1) * n * 2 / us / 1e6
    assert tbps > 0.80 * copy, "K=8 bf16 64Mi sum: %.2f TB/s (%.1f us), copy %.2f TB/s" % (tbps, us, copy)
    us = _median_us(lambda: hfr.hfr_combine_avg(out, remote, out, n, 1.0 / 128, hfr.HFR_BF16, s), s)
    tbps = 3 * n * 2 / us / 1e6
    assert tbps > 0.75 * copy, "bf16 64Mi combine: %.2f TB/s (%.1f us), copy %.2f TB/s" % (tbps, us, copy)
    us = _median_us(lambda: hfr.hfr_reduce_combine_avg(ins, K, remote, out, n, 1.0 / 128, hfr.HFR_BF16, s), s)
    tbps = (K + 2) * n * 2 / us / 1e6
    assert tbps > 0.80 * copy, "fused sum + combine: %.2f TB/s (%.1f us), copy %.2f TB/s" % (tbps, us, copy)
    del remote
    dsts = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for _ in range(K)]
    us = _median_us(lambda: hfr.hfr_broadcast(out, dsts, K, n, hfr.HFR_BF16, s), s)
    tbps = (K + 1) * n * 2 / us / 1e6
    assert tbps > 0.60 * copy, "1-to-8 broadcast: %.2f TB/s (%.1f us), copy %.2f TB/s" % (tbps, us, copy)


def test_latency_regime_floors():
    """256 chunks of 64 KiB, K = 8, fp32, relative to ONE plain launch over the
    same 16 MiB buffers timed in the same run: the bucket scheduler (which folds
    such chunks into batched launches), the batched and the device-table entry
    points each stay within a small multiple of it; with folding switched off
    the scheduler pays a launch per chunk and is many times slower."""
    K, ce = 8, 16384
    n = 256 * ce
    s = torch.cuda.Stream()
    ins = synth.peer_buffers_uniform_f32(K, n, 4000, DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    chunk_list = [([t[c * ce:(c + 1) * ce] for t in ins], out[c * ce:(c + 1) * ce], ce) for c in range(256)]
    arr = hfr.make_bucket_array([(ins, out, n)])
    chunks = hfr.make_bucket_array(chunk_list)
    table = hfr.make_chunk_table(chunk_list, DEV)
    one = _median_us(lambda: hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_F32, s), s, reps=8, warm=2)
    sched = _median_us(lambda: hfr.hfr_reduce_buckets(arr, 1, K, hfr.HFR_F32, ce, 4, s), s, reps=8, warm=2)
    batched = _median_us(lambda: hfr.hfr_reduce_buckets_batched(chunks, 256, K, hfr.HFR_F32, s), s, reps=8, warm=2)
    tab = _median_us(lambda: hfr.hfr_reduce_chunk_table(table, 256, ce, K, hfr.HFR_F32, s), s, reps=8, warm=2)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, -1)
    try:
        per_chunk = _median_us(lambda: hfr.hfr_reduce_buckets(arr, 1, K, hfr.HFR_F32, ce, 4, s), s, reps=4, warm=1)
    finally:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, 0)
    budget = 4 * one + 60.0                   # microseconds for all 256 chunks
    assert sched < budget, "bucket scheduler: %.1f us for 256 chunks, one launch %.1f us" % (sched, one)
    assert batched < budget, "batched: %.1f us for 256 chunks, one launch %.1f us" % (batched, one)
    assert tab < budget, "device table: %.1f us for 256 chunks, one launch %.1f us" % (tab, one)
    assert per_chunk > 3 * sched, "folding buys nothing: %.1f us with a launch per chunk, %.1f us folded" % (per_chunk, sched)
