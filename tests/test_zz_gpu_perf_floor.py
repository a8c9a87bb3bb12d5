"""Throughput floors, far below what the kernels reach (about 75 % of it), so
that a launch shape that silently stopped working - a fallback to a slow path,
loads serialised by a compiler change - fails a test instead of only showing up
in the benchmark. Collected last: a slow box must not hide the parity tests."""
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
    K, n = 8, 1 << 26
    s = torch.cuda.Stream()
    ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 2000, DEV)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    remote = synth.normal_bf16(n, 1e-3, 2100, DEV)
    us = _median_us(lambda: hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16, s), s)
    tbps = (K + 1) * n * 2 / us / 1e6
    assert tbps > 5.0, "K=8 bf16 64Mi sum: %.2f TB/s (%.1f us)" % (tbps, us)
    us = _median_us(lambda: hfr.hfr_combine_avg(out, remote, out, n, 1.0 / 128, hfr.HFR_BF16, s), s)
    tbps = 3 * n * 2 / us / 1e6
    assert tbps > 4.7, "bf16 64Mi combine: %.2f TB/s (%.1f us)" % (tbps, us)
    us = _median_us(lambda: hfr.hfr_reduce_combine_avg(ins, K, remote, out, n, 1.0 / 128, hfr.HFR_BF16, s), s)
    tbps = (K + 2) * n * 2 / us / 1e6
    assert tbps > 5.0, "fused sum + combine: %.2f TB/s (%.1f us)" % (tbps, us)
    del remote
    dsts = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for _ in range(K)]
    us = _median_us(lambda: hfr.hfr_broadcast(out, dsts, K, n, hfr.HFR_BF16, s), s)
    tbps = (K + 1) * n * 2 / us / 1e6
    assert tbps > 3.8, "1-to-8 broadcast: %.2f TB/s (%.1f us)" % (tbps, us)


def test_latency_regime_floors():
    """256 chunks of 64 KiB, K = 8, fp32: one launch per chunk stays under 8 us per
    chunk, the batched and the device-table entry points under 1 us per chunk."""
    K, ce = 8, 16384
    n = 256 * ce
    s = torch.cuda.Stream()
    ins = synth.peer_buffers_uniform_f32(K, n, 4000, DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    chunk_list = [([t[c * ce:(c + 1) * ce] for t in ins], out[c * ce:(c + 1) * ce], ce) for c in range(256)]
    arr = hfr.make_bucket_array([(ins, out, n)])
    chunks = hfr.make_bucket_array(chunk_list)
    table = hfr.make_chunk_table(chunk_list, DEV)
    ring = _median_us(lambda: hfr.hfr_reduce_buckets(arr, 1, K, hfr.HFR_F32, ce, 4, s), s, reps=8, warm=2) / 256
    batched = _median_us(lambda: hfr.hfr_reduce_buckets_batched(chunks, 256, K, hfr.HFR_F32, s), s, reps=8, warm=2) / 256
    tab = _median_us(lambda: hfr.hfr_reduce_chunk_table(table, 256, ce, K, hfr.HFR_F32, s), s, reps=8, warm=2) / 256
    assert ring < 8.0, "stream ring: %.2f us per chunk" % ring
    assert batched < 1.0, "batched: %.2f us per chunk" % batched
    assert tab < 1.0, "device table: %.2f us per chunk" % tab
