"""GPU parity for the fp8 storage types (OCP E4M3 and E5M2): libhfr against the
CPU oracle, bit for bit, including every ordered pair of patterns and the
narrowing of arbitrary binary32 values."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import DT, assert_bitwise, check_reduce_sum, gpu_reduce_sum, make_peers, oracle_reduce_sum

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
DEV = "cuda"
FMTS = [("e4m3", torch.float8_e4m3fn), ("e5m2", torch.float8_e5m2)]


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    for knob, v in ((hfr.HFR_TUNE_GRID_CAP, 0), (hfr.HFR_TUNE_UNROLL, 0), (hfr.HFR_TUNE_BULK_GRID, 0),
                    (hfr.HFR_TUNE_BULK_MIN_BYTES, 0)):
        hfr.hfr_set_tuning(knob, v)


def dev_bytes(arr, tdt):
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.uint8).copy()).to(DEV).view(tdt)


@pytest.mark.parametrize("name,tdt", FMTS)
def test_fp8_every_ordered_pair_and_identity(name, tdt):
    hdt, odt = DT[tdt]
    a = np.tile(np.arange(256, dtype=np.uint8), 256)
    b = np.repeat(np.arange(256, dtype=np.uint8), 256)
    ta, tb = dev_bytes(a, tdt), dev_bytes(b, tdt)
    out = gpu_reduce_sum([ta, tb])
    ident = gpu_reduce_sum([ta])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum([a, b], odt), "fp8 pairs", fp8=name)
    assert_bitwise(synth.as_numpy_bits(ident), oracle.reduce_sum([a], odt), "fp8 identity", fp8=name)
    # all pairs again, three deep: (a + b) + a
    out3 = gpu_reduce_sum([ta, tb, ta])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out3), oracle.reduce_sum([a, b, a], odt), "fp8 triples", fp8=name)


@pytest.mark.parametrize("name,tdt", FMTS)
def test_fp8_narrowing_of_arbitrary_binary32_values(name, tdt):
    """fl((x + 0) * scale) for every x and many scales: the hardware narrowing
    sees binary32 values with all 24 significand bits in use, on and around
    every rounding boundary, beyond the largest number and in the subnormal band."""
    hdt, odt = DT[tdt]
    x = np.arange(256, dtype=np.uint8)
    zero = np.zeros(256, dtype=np.uint8)
    tx, tz = dev_bytes(x, tdt), dev_bytes(zero, tdt)
    out = torch.empty_like(tx)
    rng = np.random.default_rng(440)
    scales = np.concatenate([
        rng.uniform(0.5, 2.0, size=600).astype(np.float32),
        (2.0 ** rng.integers(-12, 12, size=200) * rng.uniform(1, 2, size=200)).astype(np.float32),
        np.array([1.0, 0.5, 1.5, 1.0625, 1.03125, 1.09375, 1.125, 1.1875, 0.75, 3.0, 1e-3, 1e3], dtype=np.float32)])
    for s in scales.tolist():
        hfr.hfr_combine_avg(tx, tz, out, 256, s, hdt)
        got = synth.as_numpy_bits(out)           # synchronises
        want = oracle.combine_avg(x, zero, s, odt)
        assert_bitwise(got, want, "narrow scale=%r" % s, fp8=name)


@pytest.mark.parametrize("name,tdt", FMTS)
@pytest.mark.parametrize("K", [1, 2, 3, 5, 8, 13, 16])
def test_fp8_every_shape(name, tdt, K):
    n = 256 * 16 * 8 * 24 + 1777
    ins = make_peers(tdt, K, n, 470 + K, DEV, std=1.0)
    check_reduce_sum(ins, "fp8 wide K=%d" % K)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 5)
    check_reduce_sum(ins, "fp8 bulk K=%d" % K)
    views = [t[3:n - 2] for t in ins]                # odd byte offsets: element alignment only
    want = oracle_reduce_sum(views)
    gpu_reduce_sum(views, views[0])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(views[0]), want, "fp8 bulk misaligned in place K=%d" % K, fp8=name)


@pytest.mark.parametrize("name,tdt", FMTS)
@pytest.mark.parametrize("n", [1, 15, 16, 17, 4099, (1 << 20) + 1])
def test_fp8_ragged_combine_avg_slice_batched_broadcast(name, tdt, n):
    K = 4
    hdt, odt = DT[tdt]
    ins = make_peers(tdt, K, n, 480, DEV, std=2.0)
    host = [synth.as_numpy_bits(t) for t in ins]
    check_reduce_sum(ins, "fp8 ragged")
    out = torch.empty_like(ins[0])
    hfr.hfr_combine_avg(ins[0], ins[1], out, n, 0.3, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.combine_avg(host[0], host[1], 0.3, odt), "fp8 combine", fp8=name)
    hfr.hfr_reduce_avg(ins, K, out, n, 0.25, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, 0.25, odt), "fp8 reduce_avg", fp8=name)
    out.view(torch.uint8).zero_()
    for r in range(3):
        hfr.hfr_reduce_scatter_slice(ins, K, out, n, r, 3, hdt)
    torch.cuda.synchronize()
    full = oracle.reduce_sum(host, odt)
    assert_bitwise(synth.as_numpy_bits(out), full, "fp8 slices", fp8=name)
    cuts = synth.bucket_cuts(n, max(1, n // 5))
    out.view(torch.uint8).zero_()
    hfr.hfr_reduce_buckets_batched([([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts], len(cuts), K, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), full, "fp8 batched", fp8=name)
    out.view(torch.uint8).zero_()
    hfr.hfr_reduce_buckets([([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts], len(cuts), K, hdt, 4099, 4)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), full, "fp8 buckets", fp8=name)
    bufs = [torch.zeros(n + 5, dtype=torch.uint8, device=DEV) for _ in range(3)]
    dsts = [b[j:j + n].view(tdt) for j, b in enumerate(bufs)]
    hfr.hfr_broadcast(ins[0][:n], dsts, 3, n, hdt)
    torch.cuda.synchronize()
    for j, b in enumerate(bufs):
        assert np.array_equal(b[j:j + n].cpu().numpy(), host[0])
        assert not b[:j].any() and not b[j + n:].any()


def _load_cases(name, nfields):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([p.strip() for p in line.split(";", nfields - 1)])
    return rows


def test_fp8_golden_fixtures_on_the_gpu():
    n = 1029
    tds = dict(FMTS)
    for dt, ins, exp, why in _load_cases("reduce_sum_cases.txt", 4):
        if dt not in tds:
            continue
        bufs = [dev_bytes(np.full(n, int(x, 16), dtype=np.uint8), tds[dt]) for x in ins.split()]
        out = gpu_reduce_sum(bufs)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), np.full(n, int(exp, 16), dtype=np.uint8), why, fp8=dt)
    for dt, a, b, s, exp, why in _load_cases("combine_avg_cases.txt", 6):
        if dt not in tds:
            continue
        ta = dev_bytes(np.full(n, int(a, 16), dtype=np.uint8), tds[dt])
        tb = dev_bytes(np.full(n, int(b, 16), dtype=np.uint8), tds[dt])
        out = torch.empty_like(ta)
        scale = float(np.array([int(s, 16)], dtype=np.uint32).view(np.float32)[0])
        hfr.hfr_combine_avg(ta, tb, out, n, scale, DT[tds[dt]][0])
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), np.full(n, int(exp, 16), dtype=np.uint8), why, fp8=dt)


@pytest.mark.parametrize("name,tdt", FMTS)
def test_fp8_headline_shape_full_size(name, tdt):
    n = 1 << 26
    ins = make_peers(tdt, 8, n, 2600, DEV, std=1.0)
    out = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "fp8 K=8 64Mi", fp8=name)
