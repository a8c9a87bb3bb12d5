"""GPU parity for the fp16 storage type: libhfr against the CPU oracle, bit for
bit, including every ordered pair of fp16 bit patterns."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import assert_bitwise, check_reduce_sum, from_bits, gpu_reduce_sum, make_peers, oracle_reduce_sum

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
DEV = "cuda"
F16 = torch.float16


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    for knob, v in ((hfr.HFR_TUNE_GRID_CAP, 0), (hfr.HFR_TUNE_UNROLL, 0), (hfr.HFR_TUNE_BULK_GRID, 0),
                    (hfr.HFR_TUNE_BULK_MIN_BYTES, 0)):
        hfr.hfr_set_tuning(knob, v)


def test_f16_every_ordered_pair_of_patterns():
    """K=2 over all 2^32 ordered pairs of fp16 bit patterns: every tie, carry,
    overflow and subnormal case of the hardware conversions and the add."""
    from concurrent.futures import ThreadPoolExecutor
    lo = torch.arange(65536, dtype=torch.int32, device=DEV)
    n = 1 << 26
    threads = 8

    def oracle_slice(args):
        a, b, k = args
        sl = slice(k * (n // threads), (k + 1) * (n // threads))
        return oracle.reduce_sum([a[sl], b[sl]], oracle.F16)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        for blk in range(64):
            hi = torch.arange(blk * 1024, (blk + 1) * 1024, dtype=torch.int32, device=DEV)
            a = lo.repeat(1024).to(torch.int16).view(F16)
            b = hi.repeat_interleave(65536).to(torch.int16).view(F16)
            out = gpu_reduce_sum([a, b])
            torch.cuda.synchronize()
            ha, hb = synth.as_numpy_bits(a), synth.as_numpy_bits(b)
            want = np.concatenate(list(pool.map(oracle_slice, [(ha, hb, k) for k in range(threads)])))
            assert_bitwise(synth.as_numpy_bits(out), want, "f16 pairs block %d" % blk, f16=True)


def test_f16_narrowing_of_full_precision_sums():
    """K=8 with close exponents: fp32 accumulators with all 24 bits in use are
    narrowed; plus the subnormal band and the overflow edge."""
    rng = np.random.default_rng(225)
    K, n = 8, 600001
    h = rng.integers(0, 1 << 16, size=(K, n)).astype(np.uint16)
    e0 = ((h[0] >> 10) & 0x1F).astype(np.int64)
    for j in range(1, K):
        ej = np.clip(e0 + rng.integers(-3, 4, size=n), 0, 30).astype(np.uint16)
        h[j] = (h[j] & np.uint16(0x83FF)) | (ej << 10)
    h[0] = (h[0] & np.uint16(0x83FF)) | (np.clip(e0, 0, 30).astype(np.uint16) << 10)
    ins = [from_bits(np.ascontiguousarray(h[j]), f16=True) for j in range(K)]
    check_reduce_sum(ins, "f16 wide exponent")
    sub = h & np.uint16(0x83FF)
    ins = [from_bits(np.ascontiguousarray(sub[j]), f16=True) for j in range(K)]
    out = check_reduce_sum(ins, "f16 subnormals")
    assert torch.count_nonzero(out) > n // 2
    big = (h & np.uint16(0x83FF)) | np.uint16(28 << 10)       # 8192 .. 16383: sums overflow to inf
    ins = [from_bits(np.ascontiguousarray(big[j] & np.uint16(0x7FFF)), f16=True) for j in range(K)]
    out = check_reduce_sum(ins, "f16 overflow")
    assert torch.isinf(out).any()


@pytest.mark.parametrize("K", [1, 2, 3, 5, 8, 13, 16])
def test_f16_every_shape(K):
    n = 256 * 8 * 8 * 40 + 777
    ins = make_peers(F16, K, n, 370 + K, DEV, std=1.0)
    check_reduce_sum(ins, "f16 wide K=%d" % K)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 5)
    check_reduce_sum(ins, "f16 bulk K=%d" % K)
    views = [t[1:n - 2] for t in ins]
    want = oracle_reduce_sum(views)
    gpu_reduce_sum(views, views[0])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(views[0]), want, "f16 bulk misaligned in place K=%d" % K, f16=True)


@pytest.mark.parametrize("n", [1, 7, 8, 9, 2049, (1 << 20) + 1])
def test_f16_ragged_combine_avg_slice_batched(n):
    K = 4
    ins = make_peers(F16, K, n, 380, DEV, std=1.0)
    host = [synth.as_numpy_bits(t) for t in ins]
    check_reduce_sum(ins, "f16 ragged")
    out = torch.empty_like(ins[0])
    hfr.hfr_combine_avg(ins[0], ins[1], out, n, 0.1, hfr.HFR_F16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.combine_avg(host[0], host[1], 0.1, oracle.F16), "f16 combine", f16=True)
    hfr.hfr_reduce_avg(ins, K, out, n, 0.25, hfr.HFR_F16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, 0.25, oracle.F16), "f16 reduce_avg", f16=True)
    out.zero_()
    for r in range(3):
        hfr.hfr_reduce_scatter_slice(ins, K, out, n, r, 3, hfr.HFR_F16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum(host, oracle.F16), "f16 slices", f16=True)
    cuts = synth.bucket_cuts(n, max(1, n // 5))
    out.zero_()
    hfr.hfr_reduce_buckets_batched([([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts], len(cuts), K, hfr.HFR_F16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum(host, oracle.F16), "f16 batched", f16=True)
    out.zero_()
    hfr.hfr_reduce_buckets([([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts], len(cuts), K, hfr.HFR_F16, 4096, 4)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum(host, oracle.F16), "f16 buckets", f16=True)


def _load_cases(name, nfields):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([p.strip() for p in line.split(";", nfields - 1)])
    return rows


def test_f16_golden_fixtures_on_the_gpu():
    n = 1029
    for dt, ins, exp, why in _load_cases("reduce_sum_cases.txt", 4):
        if dt != "f16":
            continue
        bufs = [from_bits(np.full(n, int(x, 16), dtype=np.uint16), f16=True) for x in ins.split()]
        out = gpu_reduce_sum(bufs)
        torch.cuda.synchronize()
        assert np.all(synth.as_numpy_bits(out) == int(exp, 16)), why
    for dt, a, b, s, exp, why in _load_cases("combine_avg_cases.txt", 6):
        if dt != "f16":
            continue
        ta = from_bits(np.full(n, int(a, 16), dtype=np.uint16), f16=True)
        tb = from_bits(np.full(n, int(b, 16), dtype=np.uint16), f16=True)
        out = torch.empty_like(ta)
        scale = float(np.array([int(s, 16)], dtype=np.uint32).view(np.float32)[0])
        hfr.hfr_combine_avg(ta, tb, out, n, scale, hfr.HFR_F16)
        torch.cuda.synchronize()
        assert np.all(synth.as_numpy_bits(out) == int(exp, 16)), why


def test_f16_headline_shape_full_size():
    n = 1 << 26
    ins = make_peers(F16, 8, n, 2400, DEV, std=1e-3)
    out = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "f16 K=8 64Mi", f16=True)
