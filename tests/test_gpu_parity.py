"""GPU parity: libhfr (through its C ABI) against the CPU oracle, bit for bit
(0 ULP; any NaN matches any NaN). Inputs are seeded and synthetic."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import (assert_bitwise, bits, check_reduce_sum, from_bits, gpu_reduce_sum,
                               oracle_reduce_sum, oracle_reduce_sum_threaded)

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
DEV = "cuda"


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    for knob, v in ((hfr.HFR_TUNE_GRID_CAP, 0), (hfr.HFR_TUNE_UNROLL, 0), (hfr.HFR_TUNE_BULK_GRID, 0),
                    (hfr.HFR_TUNE_BULK_MIN_BYTES, 0), (hfr.HFR_TUNE_BUCKET_FOLD, 0), (hfr.HFR_TUNE_SEGMENT_MIB, 0)):
        hfr.hfr_set_tuning(knob, v)


# ------------------------------------------------------- the five workloads

def test_config1_k8_f32_1m():
    ins = synth.peer_buffers_uniform_f32(8, 1 << 20, 1000, DEV)
    check_reduce_sum(ins, "cfg1")


@pytest.mark.parametrize("n", [(1 << 20) + 12345, 3 * 256 * 2 * 8 * 5 + 3])
def test_config2_shape_small_bf16(n):
    ins = synth.peer_buffers_normal_bf16(8, n, 1e-3, 2000, DEV)
    check_reduce_sum(ins, "cfg2-small n=%d" % n)


def test_config2_full_size_k8_bf16_64m():
    """The headline workload at full size, every element compared."""
    n = 1 << 26
    ins = synth.peer_buffers_normal_bf16(8, n, 1e-3, 2000, DEV)
    out = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    want = oracle_reduce_sum(ins)
    assert_bitwise(synth.as_numpy_bits(out), want, "cfg2 full")


def _small_transformer():
    return synth.transformer_grad_tensors(n_layers=8, d_model=128, ffn=344, vocab=1000)


@pytest.mark.parametrize("chunk_elems,n_streams", [(1 << 30, 1), (1 << 30, 4), (20000, 4), (4096, 3), (777, 16)])
def test_config3_bucketed_gradients_scaled_down(chunk_elems, n_streams):
    """Same tensor list and packing rule as the bucketed workload at 1/32 of
    the widths; bucket cap chosen so that there are many buckets and a ragged
    last one."""
    K = 8
    tensors = _small_transformer()
    total = sum(t.numel for t in tensors)
    flats = [synth.flat_gradient_bf16(tensors, 3000 + j, DEV) for j in range(K)]
    out = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    cap = 25 * 1024
    cuts = synth.bucket_cuts(total, cap)
    assert len(cuts) > 20 and cuts[-1][1] != cap
    buckets = [([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in cuts]
    hfr.hfr_reduce_buckets(buckets, len(buckets), K, hfr.HFR_BF16, chunk_elems, n_streams)
    torch.cuda.synchronize()
    want = oracle.reduce_buckets(
        [([synth.as_numpy_bits(f[o:o + l]) for f in flats], np.empty(l, dtype=np.uint16)) for o, l in cuts],
        oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), np.concatenate(want), "cfg3 small")


@pytest.mark.parametrize("chunk_elems,n_streams", [(1 << 30, 4), (20000, 4), (777, 3)])
def test_config3_whole_tensor_buckets_scaled_down(chunk_elems, n_streams):
    """The secondary packing of the bucketed workload: whole tensors appended
    until a bucket holds at least the cap, so buckets are uneven and some hold
    a single matrix. The result must equal the oracle's on the same cuts and
    the flat sum (packing is invisible in the result)."""
    K = 8
    tensors = _small_transformer()
    total = sum(t.numel for t in tensors)
    flats = [synth.flat_gradient_bf16(tensors, 3000 + j, DEV) for j in range(K)]
    out = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
    cuts = synth.bucket_cuts_whole_tensors(tensors, 25 * 1024)
    assert len(cuts) > 10 and len({l for _, l in cuts}) > 2
    buckets = [([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in cuts]
    hfr.hfr_reduce_buckets(buckets, len(buckets), K, hfr.HFR_BF16, chunk_elems, n_streams)
    torch.cuda.synchronize()
    want = oracle.reduce_buckets(
        [([synth.as_numpy_bits(f[o:o + l]) for f in flats], np.empty(l, dtype=np.uint16)) for o, l in cuts],
        oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), np.concatenate(want), "cfg3 whole-tensor small")
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(flats), "cfg3 whole-tensor vs flat")


def test_config3_full_size_every_bucket_of_both_packings():
    """Full-size bucketed workload (8 peers x 1.75e9 bf16 elements): all 67 flat
    buckets of 25 Mi elements, and then all 41 whole-tensor buckets of the
    secondary packing, compared element by element with the oracle, which runs
    bucket by bucket on the host's threads."""
    from concurrent.futures import ThreadPoolExecutor
    K = 8
    tensors = synth.transformer_grad_tensors()
    total = sum(t.numel for t in tensors)
    assert total == 1_750_142_976
    flats = [synth.flat_gradient_bf16(tensors, 3000 + j, DEV) for j in range(K)]
    out = torch.empty(total, dtype=torch.bfloat16, device=DEV)
    cuts = synth.bucket_cuts(total)
    assert len(cuts) == 67 and cuts[-1][1] == 19_992_576
    buckets = [([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in cuts]
    hfr.hfr_reduce_buckets(buckets, len(buckets), K, hfr.HFR_BF16, synth.BUCKET_CAP_ELEMS, 4)
    torch.cuda.synchronize()
    host = [synth.as_numpy_bits(f) for f in flats]
    want = np.empty(total, dtype=np.uint16)

    def one_bucket(cut):
        o, l = cut
        oracle.reduce_sum([h[o:o + l] for h in host], oracle.BF16, out=want[o:o + l])

    with ThreadPoolExecutor(max_workers=16) as pool:
        list(pool.map(one_bucket, cuts))
    got = synth.as_numpy_bits(out)
    for b, (o, l) in enumerate(cuts):
        assert_bitwise(got[o:o + l], want[o:o + l], "cfg3 flat bucket %d" % b)
    # secondary packing at full size: 41 uneven whole-tensor buckets, every one against the oracle
    cuts2 = synth.bucket_cuts_whole_tensors(tensors)
    assert len(cuts2) == 41
    out.zero_()
    buckets2 = [([f[o:o + l] for f in flats], out[o:o + l], l) for o, l in cuts2]
    hfr.hfr_reduce_buckets(buckets2, len(buckets2), K, hfr.HFR_BF16, synth.BUCKET_CAP_ELEMS, 4)
    torch.cuda.synchronize()
    got = synth.as_numpy_bits(out)
    for b, (o, l) in enumerate(cuts2):
        assert_bitwise(got[o:o + l], want[o:o + l], "cfg3 whole-tensor bucket %d" % b)


@pytest.mark.parametrize("K", [2, 4, 8, 16])
@pytest.mark.parametrize("chunk_bytes", [64 << 10, 256 << 10, 1 << 20, 4 << 20])
def test_config4_latency_regime(K, chunk_bytes):
    """256 chunks per run through hfr_reduce_buckets with 4 streams; every
    chunk of every cell compared with the oracle (host threads)."""
    chunk_elems = chunk_bytes // 4
    n = 256 * chunk_elems
    ins = synth.peer_buffers_uniform_f32(K, n, 4000, DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    hfr.hfr_reduce_buckets([(ins, out, n)], 1, K, hfr.HFR_F32, chunk_elems, 4)
    torch.cuda.synchronize()
    want = oracle_reduce_sum_threaded([synth.as_numpy_bits(t) for t in ins], oracle.F32)
    got = synth.as_numpy_bits(out)
    for c in range(256):
        sl = slice(c * chunk_elems, (c + 1) * chunk_elems)
        assert_bitwise(got[sl], want[sl], "cfg4 chunk %d" % c)


def test_config5_combine_full_size_f32_256m():
    n = 1 << 28
    a = synth.normal_f32(n, 1.0, 5000, DEV)
    b = synth.normal_f32(n, 1.0, 5001, DEV)
    out = torch.empty_like(a)
    scale = 1.0 / (8 * 16)
    hfr.hfr_combine_avg(a, b, out, n, scale, hfr.HFR_F32)
    torch.cuda.synchronize()
    want = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), scale, oracle.F32)
    assert_bitwise(synth.as_numpy_bits(out), want, "cfg5")


def test_inputs_longer_than_one_launch_segment():
    """Inputs beyond 128 MiB per buffer are cut into several launches inside
    the library; a ragged remainder lands in a last, tiny launch."""
    n = (1 << 26) + 12345                       # bf16: 128 MiB + a bit
    ins = synth.peer_buffers_normal_bf16(8, n, 1e-3, 2300, DEV)
    out = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "two segments bf16 K8")
    n = 2 * (1 << 25) + (1 << 24) + 4099        # fp32: 2.5 segments + ragged
    a = synth.normal_f32(n, 1.0, 2310, DEV)
    b = synth.normal_f32(n, 1.0, 2311, DEV)
    out = torch.empty_like(a)
    hfr.hfr_combine_avg(a, b, out, n, 0.1, hfr.HFR_F32)
    s2 = gpu_reduce_sum([a, b, a])
    torch.cuda.synchronize()
    want = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), 0.1, oracle.F32)
    assert_bitwise(synth.as_numpy_bits(out), want, "combine over segments")
    assert_bitwise(synth.as_numpy_bits(s2), oracle_reduce_sum([a, b, a]), "K3 over segments")
    # shifted views: every segment start stays element aligned only
    v = [a[1:], b[1:]]
    want = oracle_reduce_sum(v)
    gpu_reduce_sum(v, v[0])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(v[0]), want, "segments, shifted, in place")


@pytest.mark.parametrize("bulk", [False, True])
def test_every_entry_point_across_many_short_segments(bulk):
    """The segment length forced down to 1 MiB per buffer: every entry point
    that cuts long inputs runs as a chain of many launches with a ragged last
    one, in the wide and in the bulk launch shape, and must give the oracle's
    bits (segment cuts are invisible in the result)."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_SEGMENT_MIB, 1)
    if bulk:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 6)
    n = 5 * (1 << 19) + 70001                    # bf16: five whole segments and a ragged sixth
    for K in (2, 8, 16):
        ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 2400 + K, DEV)
        check_reduce_sum(ins, "segments K=%d bulk=%s" % (K, bulk))
    ins = synth.peer_buffers_normal_bf16(9, n, 1e-3, 2450, DEV)
    h = [synth.as_numpy_bits(t) for t in ins]
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_avg(ins[:8], 8, out, n, 0.125, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(h[:8], 0.125, oracle.BF16), "avg over segments")
    hfr.hfr_reduce_combine_avg(ins[:8], 8, ins[8], out, n, 1.0 / 128, hfr.HFR_BF16)
    torch.cuda.synchronize()
    want = oracle.combine_avg(oracle.reduce_sum(h[:8], oracle.BF16), h[8], 1.0 / 128, oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), want, "fused sum + combine over segments")
    hfr.hfr_combine_avg(ins[0], ins[1], out, n, 0.3, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.combine_avg(h[0], h[1], 0.3, oracle.BF16), "combine over segments")
    hfr.hfr_reduce_scatter_slice(ins[:8], 8, out, n, 1, 2, hfr.HFR_BF16)
    torch.cuda.synchronize()
    b, e = hfr.hfr_slice_bounds(n, 1, 2)
    assert_bitwise(synth.as_numpy_bits(out)[b:e], oracle.reduce_sum(h[:8], oracle.BF16)[b:e], "slice over segments")
    dsts = [torch.zeros_like(ins[0]) for _ in range(3)]
    hfr.hfr_broadcast(ins[0], dsts, 3, n, hfr.HFR_BF16)
    torch.cuda.synchronize()
    for d in dsts:
        assert_bitwise(synth.as_numpy_bits(d), h[0], "broadcast over segments")


# ------------------------------------------------------------- edge cases

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n", [1, 2, 3, 7, 8, 9, 255, 256, 2047, 2049, 4096 + 5, (1 << 20) - 1, (1 << 20) + 1])
def test_ragged_sizes(dtype, n):
    K = 5
    if dtype == torch.float32:
        ins = synth.peer_buffers_uniform_f32(K, n, 60, DEV)
    else:
        ins = synth.peer_buffers_normal_bf16(K, n, 1.0, 60, DEV)
    check_reduce_sum(ins, "ragged n=%d" % n)
    a, b = ins[0], ins[1]
    _, odt = (None, oracle.F32) if dtype == torch.float32 else (None, oracle.BF16)
    hdt = hfr.HFR_F32 if dtype == torch.float32 else hfr.HFR_BF16
    out = torch.empty_like(a)
    hfr.hfr_combine_avg(a, b, out, n, 0.1, hdt)
    torch.cuda.synchronize()
    want = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), 0.1, odt)
    assert_bitwise(synth.as_numpy_bits(out), want, "combine ragged n=%d" % n)


def test_empty_input_is_a_no_op():
    out = torch.full((16,), 7.0, device=DEV)
    assert hfr.hfr_reduce_sum([out, out], 2, out, 0, hfr.HFR_F32) == hfr.HFR_OK
    assert hfr.hfr_combine_avg(out, out, out, 0, 1.0, hfr.HFR_F32) == hfr.HFR_OK
    assert hfr.hfr_reduce_buckets([([out, out], out, 0)], 1, 2, hfr.HFR_F32, 4, 4) == hfr.HFR_OK
    torch.cuda.synchronize()
    assert torch.all(out == 7.0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K", list(range(1, 17)))
def test_every_k(dtype, K):
    n = 70001
    if dtype == torch.float32:
        ins = synth.peer_buffers_uniform_f32(K, n, 70 + K, DEV)
    else:
        ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 70 + K, DEV)
    check_reduce_sum(ins, "K=%d" % K)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_misaligned_views(dtype):
    """Pointers with element alignment only (views shifted by 1..3 elements),
    in every mix of aligned / shifted inputs and output."""
    K, n = 4, 300007
    gen = synth.peer_buffers_uniform_f32 if dtype == torch.float32 else \
        (lambda K, n, s, d: synth.peer_buffers_normal_bf16(K, n, 1.0, s, d))
    base = gen(K, n + 8, 80, DEV)
    for shifts, oshift in (((1, 1, 1, 1), 1), ((0, 1, 2, 3), 0), ((0, 0, 0, 0), 3), ((3, 0, 1, 0), 2)):
        ins = [b[s:s + n] for b, s in zip(base, shifts)]
        obuf = torch.zeros(n + 8, dtype=dtype, device=DEV)
        out = obuf[oshift:oshift + n]
        gpu_reduce_sum(ins, out)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "misaligned %s/%d" % (shifts, oshift))
        # nothing outside the view was written
        assert torch.all(obuf[:oshift] == 0) and torch.all(obuf[oshift + n:] == 0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_in_place_output_aliases_an_input(dtype):
    K, n = 8, 1 << 18
    gen = synth.peer_buffers_uniform_f32 if dtype == torch.float32 else \
        (lambda K, n, s, d: synth.peer_buffers_normal_bf16(K, n, 1.0, s, d))
    ins = gen(K, n + 3, 90, DEV)
    ins = [t[:n + 3] for t in ins]
    want = oracle_reduce_sum(ins)
    for j in (0, 3, 7):
        work = [t.clone() for t in ins]
        gpu_reduce_sum(work, work[j])
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(work[j]), want, "in place j=%d" % j)
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    a, b = ins[0].clone(), ins[1].clone()
    wantc = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), 0.125, odt)
    hfr.hfr_combine_avg(a, b, b, n + 3, 0.125, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(b), wantc, "combine in place")


def test_adjacent_buffers_are_not_an_overlap():
    n = 4096
    buf = synth.uniform_pm1(3 * n, 91, DEV)
    ins = [buf[:n], buf[n:2 * n]]
    out = buf[2 * n:]
    want = oracle_reduce_sum(ins)
    gpu_reduce_sum(ins, out)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "adjacent")
    assert hfr.hfr_reduce_sum(ins, 2, buf[n - 1:2 * n - 1], n, hfr.HFR_F32, check=False) == hfr.HFR_ERR_OVERLAP


def _load_cases(name, nfields):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([p.strip() for p in line.split(";", nfields - 1)])
    return rows


def test_golden_fixtures_on_the_gpu():
    """The hand-derived tie / carry / overflow / signed-zero / subnormal cases,
    placed at several positions of a buffer (vector body and scalar tail)."""
    for dt, ins, exp, why in _load_cases("reduce_sum_cases.txt", 4):
        if dt not in ("f32", "bf16"):
            continue  # fp16 / fp8 rows are covered by their own test files
        in_bits = [int(x, 16) for x in ins.split()]
        np_t = np.uint32 if dt == "f32" else np.uint16
        n = 1029
        bufs = [from_bits(np.full(n, b, dtype=np_t)) for b in in_bits]
        out = gpu_reduce_sum(bufs)
        torch.cuda.synchronize()
        got = synth.as_numpy_bits(out)
        got = got.view(np.uint32) if dt == "f32" else got
        assert np.all(got == int(exp, 16)), why
    for dt, a, b, s, exp, why in _load_cases("combine_avg_cases.txt", 6):
        if dt not in ("f32", "bf16"):
            continue
        np_t = np.uint32 if dt == "f32" else np.uint16
        n = 1029
        ta = from_bits(np.full(n, int(a, 16), dtype=np_t))
        tb = from_bits(np.full(n, int(b, 16), dtype=np_t))
        out = torch.empty_like(ta)
        scale = float(np.array([int(s, 16)], dtype=np.uint32).view(np.float32)[0])
        hfr.hfr_combine_avg(ta, tb, out, n, scale, hfr.HFR_F32 if dt == "f32" else hfr.HFR_BF16)
        torch.cuda.synchronize()
        got = synth.as_numpy_bits(out)
        got = got.view(np.uint32) if dt == "f32" else got
        assert np.all(got == int(exp, 16)), why


def test_special_values_f32_all_exponents():
    """Random bit patterns over every exponent incl. subnormals, infinities and
    NaNs; close exponents so that adds round; no flush to zero on either side."""
    rng = np.random.default_rng(123)
    K, n = 8, 200003
    u = rng.integers(0, 1 << 32, size=(K, n), dtype=np.uint64).astype(np.uint32)
    e0 = ((u[0] >> 23) & 0xFF).astype(np.int64)
    for j in range(1, K):
        ej = np.clip(e0 + rng.integers(-2, 3, size=n), 0, 255).astype(np.uint32)
        u[j] = (u[j] & np.uint32(0x807FFFFF)) | (ej << 23)
    ins = [from_bits(np.ascontiguousarray(u[j])) for j in range(K)]
    check_reduce_sum(ins, "all exponents f32")
    sub = (u & np.uint32(0x807FFFFF))  # exponent field 0: all subnormal
    ins = [from_bits(np.ascontiguousarray(sub[j])) for j in range(K)]
    out = check_reduce_sum(ins, "subnormals f32")
    assert torch.count_nonzero(out) > n // 2  # really not flushed


def test_special_values_bf16_all_patterns_pairs():
    """K=2 over every bf16 pattern against 2048 partner patterns (specials and
    random): 2^27 ordered pairs, exercising every tie / carry of the narrowing."""
    rng = np.random.default_rng(124)
    partners = np.concatenate([
        np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x3F80, 0xBF80, 0x3B80, 0x3F81,
                  0x4380, 0x7F7F, 0xFF7F, 0x7B00, 0x7F80, 0xFF80, 0x7FC0], dtype=np.uint16),
        rng.integers(0, 1 << 16, size=2048 - 17).astype(np.uint16)])
    a = np.tile(np.arange(65536, dtype=np.uint32).astype(np.uint16), 2048)
    b = np.repeat(partners, 65536)
    ta, tb = from_bits(a), from_bits(b)
    out = gpu_reduce_sum([ta, tb])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum([a, b], oracle.BF16), "bf16 pairs")
    outc = torch.empty_like(ta)
    hfr.hfr_combine_avg(ta, tb, outc, a.shape[0], 0.1, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(outc), oracle.combine_avg(a, b, 0.1, oracle.BF16), "bf16 pairs combine")


def test_bf16_every_ordered_pair_of_patterns():
    """K=2 over all 2^32 ordered pairs of bf16 bit patterns, 2^26 at a time:
    every tie, carry, overflow and subnormal case of a two-operand sum. The
    oracle's slices run on a few host threads (same single-threaded function on
    disjoint index ranges)."""
    from concurrent.futures import ThreadPoolExecutor
    lo = torch.arange(65536, dtype=torch.int32, device=DEV)
    n = 1 << 26
    threads = 8

    def oracle_slice(args):
        a, b, k = args
        sl = slice(k * (n // threads), (k + 1) * (n // threads))
        return oracle.reduce_sum([a[sl], b[sl]], oracle.BF16)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        for blk in range(64):
            # a runs over all patterns (fast index), b over 1024 patterns of this block
            hi = torch.arange(blk * 1024, (blk + 1) * 1024, dtype=torch.int32, device=DEV)
            a = lo.repeat(1024).to(torch.int16).view(torch.bfloat16)
            b = hi.repeat_interleave(65536).to(torch.int16).view(torch.bfloat16)
            out = gpu_reduce_sum([a, b])
            torch.cuda.synchronize()
            ha, hb = synth.as_numpy_bits(a), synth.as_numpy_bits(b)
            want = np.concatenate(list(pool.map(oracle_slice, [(ha, hb, k) for k in range(threads)])))
            assert_bitwise(synth.as_numpy_bits(out), want, "pairs block %d" % blk)


def _bf16_dev(u16):
    return torch.from_numpy(u16.view(np.int16).copy()).view(torch.bfloat16).to(DEV)


def test_bf16_narrowing_of_arbitrary_binary32_values():
    """The device's bf16 narrowing (a carry trick, a different formulation from
    the oracle's) fed with binary32 values that use all 24 significand bits:
    fl((x + 0) * scale) for EVERY bf16 pattern x and many scales, through the
    combine and through the fused average, against the oracle."""
    x = np.arange(65536, dtype=np.uint16)
    zero = np.zeros(65536, dtype=np.uint16)
    tx, tz = _bf16_dev(x), _bf16_dev(zero)
    out = torch.empty_like(tx)
    rng = np.random.default_rng(441)
    scales = np.concatenate([
        rng.uniform(0.5, 2.0, size=150).astype(np.float32),
        (2.0 ** rng.integers(-20, 20, size=60) * rng.uniform(1, 2, size=60)).astype(np.float32),
        np.array([1.0, 0.5, 1.5, 1.00390625, 1.001953125, 1.005859375, 1.0078125, 0.75, 3.0, 1e-3, 1e3,
                  1.0 / 128, 1.0 / 3, 2.0 ** -120, 2.0 ** 100], dtype=np.float32)])
    for s in scales.tolist():
        hfr.hfr_combine_avg(tx, tz, out, 65536, s, hfr.HFR_BF16)
        got = synth.as_numpy_bits(out)               # synchronises
        assert_bitwise(got, oracle.combine_avg(x, zero, s, oracle.BF16), "combine narrow scale=%r" % s)
        hfr.hfr_reduce_avg([tx, tz], 2, out, 65536, s, hfr.HFR_BF16)
        got = synth.as_numpy_bits(out)
        assert_bitwise(got, oracle.reduce_avg([x, zero], s, oracle.BF16), "average narrow scale=%r" % s)


@pytest.mark.parametrize("nudge", [0, 1, -1])
def test_bf16_narrowing_on_and_around_every_tie(nudge):
    """For every bf16 pattern p with room below it: p + half an ulp of p is a
    binary32 value exactly between two bf16 neighbours (a tie, for even and
    for odd kept mantissas alike); one binary32 ulp more or less is just off
    the tie. Built as exact three-operand sums ((p + h) + t), so the only
    rounding is the narrowing under test."""
    p = np.arange(65536, dtype=np.uint16)
    e = (p >> 7) & 0xFF
    ok = (e >= 24) & (e < 255)                       # h and t are normal bf16 numbers, p is finite
    sign = p & 0x8000
    h = np.where(ok, sign | ((e - 8).astype(np.uint16) << 7), 0).astype(np.uint16)     # half an ulp of p, same sign
    tsign = sign if nudge > 0 else (sign ^ 0x8000)
    t = np.where(ok & (nudge != 0), tsign | ((e - 23).astype(np.uint16) << 7), 0).astype(np.uint16)  # one fp32 ulp
    ins_h = [p, h, t]
    ins = [_bf16_dev(a) for a in ins_h]
    out = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    want = oracle.reduce_sum(ins_h, oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), want, "ties nudge=%d" % nudge)
    if nudge == 0:
        # the construction does what it says: on a tie the result has an even kept mantissa
        w = want[ok]
        assert not (w & 1).any()
        assert ((w == p[ok]) | (w == p[ok] + 1)).all()
    # the same sums through the fused average with scale 1 and the combine of (p + h) with t
    hfr.hfr_reduce_avg(ins, 3, out, 65536, 1.0, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "ties through the average, nudge=%d" % nudge)


def test_bf16_wide_exponent_k8():
    rng = np.random.default_rng(125)
    K, n = 8, 400001
    h = rng.integers(0, 1 << 16, size=(K, n)).astype(np.uint16)
    e0 = ((h[0] >> 7) & 0xFF).astype(np.int64)
    for j in range(1, K):
        ej = np.clip(e0 + rng.integers(-3, 4, size=n), 0, 254).astype(np.uint16)
        h[j] = (h[j] & np.uint16(0x807F)) | (ej << 7)
    ins = [from_bits(np.ascontiguousarray(h[j])) for j in range(K)]
    check_reduce_sum(ins, "bf16 wide exponent")


def test_order_discriminator_on_the_gpu():
    vals = [2.0 ** 24, 1, 1, 1, 1, 1, 1, -(2.0 ** 24)]
    n = 5000
    ins = [torch.full((n,), v, dtype=torch.float32, device=DEV) for v in vals]
    out = gpu_reduce_sum(ins)
    rev = gpu_reduce_sum(list(reversed(ins)))
    torch.cuda.synchronize()
    assert torch.all(out == 0.0) and torch.all(rev == 6.0)


def test_combine_scale_one_equals_two_way_sum_and_no_fma():
    n = (1 << 20) + 3
    a = synth.normal_f32(n, 1.0, 51, DEV)
    b = synth.normal_f32(n, 1.0, 52, DEV)
    out = torch.empty_like(a)
    hfr.hfr_combine_avg(a, b, out, n, 1.0, hfr.HFR_F32)
    s = gpu_reduce_sum([a, b])
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int32), s.view(torch.int32))
    # non power-of-two scale: two roundings, as the oracle does them
    hfr.hfr_combine_avg(a, b, out, n, 0.1, hfr.HFR_F32)
    torch.cuda.synchronize()
    want = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), 0.1, oracle.F32)
    assert_bitwise(synth.as_numpy_bits(out), want, "combine 0.1")


def test_combine_bf16_gradient_shape():
    n = (1 << 22) + 5
    a = synth.normal_bf16(n, 8e-3, 53, DEV)
    b = synth.normal_bf16(n, 8e-3, 54, DEV)
    out = torch.empty_like(a)
    hfr.hfr_combine_avg(a, b, out, n, 1.0 / 128, hfr.HFR_BF16)
    torch.cuda.synchronize()
    want = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), 1.0 / 128, oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), want, "combine bf16")


# ------------------------------------------ fused average and slice variants

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K,n,force_bulk", [(8, (1 << 20) + 13, False), (2, 4099, False), (16, 300001, False),
                                            (8, 256 * 8 * 8 * 40 + 777, True), (3, 256 * 8 * 8 * 9 + 5, True)])
def test_reduce_avg(dtype, K, n, force_bulk):
    if force_bulk:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 7)
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    if dtype == torch.float32:
        ins = synth.peer_buffers_uniform_f32(K, n, 700 + K, DEV)
    else:
        ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 700 + K, DEV)
    host = [synth.as_numpy_bits(t) for t in ins]
    out = torch.empty_like(ins[0])
    for scale in (1.0 / K, 0.1, 1.0):
        hfr.hfr_reduce_avg(ins, K, out, n, scale, hdt)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, scale, odt), "reduce_avg s=%g" % scale)
    # scale 1 is the plain sum, bit for bit
    assert torch.equal(out.view(torch.int16 if dtype == torch.bfloat16 else torch.int32),
                       gpu_reduce_sum(ins).view(torch.int16 if dtype == torch.bfloat16 else torch.int32))


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_nvlink_variant_shape_pair_prereduce_then_slice_reduce(dtype):
    """The shape of the paper's NVLink variant (Section IV-C) on one GPU: the
    eight buffers are pre-reduced in four pairs (K = 2 sums), then every rank of
    a group of four reduces its own slice of the four pair partials (K = 4,
    slice only); the slices together are the full result. Each stage is compared
    with the oracle run the same way (the pair partials are stored, hence
    rounded, before the second stage)."""
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    n, world = 1_000_003, 4
    if dtype == torch.float32:
        ins = synth.peer_buffers_uniform_f32(8, n, 780, DEV)
    else:
        ins = synth.peer_buffers_normal_bf16(8, n, 1e-3, 780, DEV)
    host = [synth.as_numpy_bits(t) for t in ins]
    pairs = [torch.empty_like(ins[0]) for _ in range(4)]
    for p in range(4):
        hfr.hfr_reduce_sum([ins[2 * p], ins[2 * p + 1]], 2, pairs[p], n, hdt)
    out = torch.zeros_like(ins[0])
    for rank in range(world):
        hfr.hfr_reduce_scatter_slice(pairs, 4, out, n, rank, world, hdt)
    torch.cuda.synchronize()
    want_pairs = [oracle.reduce_sum([host[2 * p], host[2 * p + 1]], odt) for p in range(4)]
    for p in range(4):
        assert_bitwise(synth.as_numpy_bits(pairs[p]), want_pairs[p], "pair %d" % p)
    want = np.zeros_like(want_pairs[0])
    for rank in range(world):
        oracle.reduce_scatter_slice(want_pairs, rank, world, odt, want)
    assert_bitwise(synth.as_numpy_bits(out), want, "slices of the pair partials")
    assert_bitwise(want, oracle.reduce_sum(want_pairs, odt), "the slices cover [0, n)")


def test_reduce_avg_golden_and_config2_size():
    # 256 + 7 ones, times 1/128: one narrowing after the multiply -> 0x4004
    col = [from_bits(np.full(1029, b, dtype=np.uint16)) for b in [0x4380] + [0x3F80] * 7]
    out = torch.empty_like(col[0])
    hfr.hfr_reduce_avg(col, 8, out, 1029, 1.0 / 128, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert np.all(synth.as_numpy_bits(out) == 0x4004)
    # headline shape, full size (bulk launch shape by default)
    n = 1 << 26
    ins = synth.peer_buffers_normal_bf16(8, n, 1e-3, 2000, DEV)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_avg(ins, 8, out, n, 1.0 / 8, hfr.HFR_BF16)
    torch.cuda.synchronize()
    want = oracle.reduce_avg([synth.as_numpy_bits(t) for t in ins], 1.0 / 8, oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), want, "reduce_avg cfg2 size")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("n,world", [(100003, 7), (1 << 20, 8), (5, 16), (4096 * 3 + 1, 2)])
def test_reduce_scatter_slice(dtype, n, world):
    K = 4
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    if dtype == torch.float32:
        ins = synth.peer_buffers_uniform_f32(K, n, 800, DEV)
    else:
        ins = synth.peer_buffers_normal_bf16(K, n, 1.0, 800, DEV)
    host = [synth.as_numpy_bits(t) for t in ins]
    full = oracle.reduce_sum(host, odt)
    gathered = torch.zeros(n, dtype=dtype, device=DEV)
    for r in range(world):
        out = torch.full((n,), 3.0, dtype=dtype, device=DEV)
        hfr.hfr_reduce_scatter_slice(ins, K, out, n, r, world, hdt)
        hfr.hfr_reduce_scatter_slice(ins, K, gathered, n, r, world, hdt)
        torch.cuda.synchronize()
        want = np.full(n, 3.0, dtype=np.float32)
        want = want if dtype == torch.float32 else synth.as_numpy_bits(torch.full((n,), 3.0, dtype=torch.bfloat16))
        want = oracle.reduce_scatter_slice(host, r, world, odt, want.copy())
        assert_bitwise(synth.as_numpy_bits(out), want, "slice %d/%d" % (r, world))
        assert hfr.hfr_slice_bounds(n, r, world) == oracle.slice_bounds(n, r, world)
    assert_bitwise(synth.as_numpy_bits(gathered), full, "all slices gathered")


# ----------------------------------------------- fused sum + combine-and-average

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.float8_e4m3fn, torch.float8_e5m2])
@pytest.mark.parametrize("K,n,force_bulk", [(1, 4099, False), (2, 70001, False), (8, (1 << 20) + 13, False),
                                            (15, 300001, False), (8, 256 * 16 * 8 * 24 + 777, True),
                                            (3, 256 * 16 * 8 * 9 + 5, True)])
def test_reduce_combine_avg_equals_the_two_calls(dtype, K, n, force_bulk):
    """One kernel against the oracle's reduce_sum followed by its combine_avg:
    the node partial is rounded to storage in between on both sides."""
    from tests.parity_util import DT, FP8_NAME, make_peers
    if force_bulk:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 7)
    hdt, odt = DT[dtype]
    std = 1.0 if dtype in FP8_NAME else 1e-3
    ins = make_peers(dtype, K, n, 1100 + K, DEV, std=std)
    remote = make_peers(dtype, 1, n, 1150 + K, DEV, std=std * 2)[0]
    host = [synth.as_numpy_bits(t) for t in ins]
    hrem = synth.as_numpy_bits(remote)
    kw = dict(f16=dtype == torch.float16, fp8=FP8_NAME.get(dtype, ""))
    for scale in (1.0 / 128, 0.3):
        want = oracle.combine_avg(oracle.reduce_sum(host, odt), hrem, scale, odt)
        out = torch.empty_like(ins[0])
        hfr.hfr_reduce_combine_avg(ins, K, remote, out, n, scale, hdt)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), want, "fused K=%d s=%g" % (K, scale), **kw)
        # and against the library's own two calls
        two = torch.empty_like(ins[0])
        hfr.hfr_reduce_sum(ins, K, two, n, hdt)
        hfr.hfr_combine_avg(two, remote, two, n, scale, hdt)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(two), want, "two calls K=%d" % K, **kw)
    # in place on the remote partial
    rem2 = remote.clone()
    hfr.hfr_reduce_combine_avg(ins, K, rem2, rem2, n, 0.3, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(rem2), want, "fused in place", **kw)


def test_reduce_combine_avg_intermediate_rounding_matters():
    """256 + 7 ones is 263 in fp32 but 264 once stored as bf16; adding a remote 1
    and scaling by 1 must give narrow(265) = 264, not narrow(263 + 1) = 264 ...
    so use a remote of 2: 264 + 2 = 266 -> tie -> 264? no: 266 = 256 * 1.0390625,
    between 264 and 268 -> exactly half-way -> even mantissa -> 264; whereas the
    unrounded 263 + 2 = 265 would narrow to 264 as well. A remote of 4 separates
    them: 264 + 4 = 268 (exact) against 263 + 4 = 267 -> 268. Use remote = -8:
    264 - 8 = 256 (exact), 263 - 8 = 255 (exact, differs)."""
    n = 1029
    col = [from_bits(np.full(n, b, dtype=np.uint16)) for b in [0x4380] + [0x3F80] * 7]
    remote = from_bits(np.full(n, 0xC100, dtype=np.uint16))     # -8.0
    out = torch.empty_like(col[0])
    hfr.hfr_reduce_combine_avg(col, 8, remote, out, n, 1.0, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert np.all(synth.as_numpy_bits(out) == 0x4380)           # 256, not 255 (0x437F)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.float8_e4m3fn, torch.float8_e5m2])
def test_scaled_operations_on_the_scalar_tail_path(dtype):
    """Thousands of calls shorter than one 16-byte vector, so that every element
    goes through the scalar tail code of the scaled operations (a place where a
    compiler may fuse "multiply, then narrow" into a single rounding)."""
    from tests.parity_util import DT, FP8_NAME, make_peers
    hdt, odt = DT[dtype]
    es = hfr.ELEM_SIZE[hdt]
    m = 16 // es - 1                      # elements per call: one less than a vector
    calls, K = 1500, 3
    n = calls * 16                        # every call starts 16-byte aligned
    std = 1.0 if dtype in FP8_NAME else 1e-2
    ins = make_peers(dtype, K, n, 1300, DEV, std=std)
    remote = make_peers(dtype, 1, n, 1310, DEV, std=std)[0]
    o_avg, o_comb, o_fused = (torch.zeros(n, dtype=torch.uint8, device=DEV).view(dtype) if dtype in FP8_NAME
                              else torch.zeros(n, dtype=dtype, device=DEV) for _ in range(3))
    scale = 0.3
    for c in range(calls):
        sl = slice(c * 16, c * 16 + m)
        hfr.hfr_reduce_avg([t[sl] for t in ins], K, o_avg[sl], m, scale, hdt)
        hfr.hfr_combine_avg(ins[0][sl], remote[sl], o_comb[sl], m, scale, hdt)
        hfr.hfr_reduce_combine_avg([t[sl] for t in ins], K, remote[sl], o_fused[sl], m, scale, hdt)
    torch.cuda.synchronize()
    host = [synth.as_numpy_bits(t) for t in ins]
    hrem = synth.as_numpy_bits(remote)
    keep = (np.arange(n) % 16) < m
    kw = dict(f16=dtype == torch.float16, fp8=FP8_NAME.get(dtype, ""))
    assert_bitwise(synth.as_numpy_bits(o_avg)[keep], oracle.reduce_avg(host, scale, odt)[keep], "tail reduce_avg", **kw)
    assert_bitwise(synth.as_numpy_bits(o_comb)[keep], oracle.combine_avg(host[0], hrem, scale, odt)[keep], "tail combine", **kw)
    want = oracle.combine_avg(oracle.reduce_sum(host, odt), hrem, scale, odt)
    assert_bitwise(synth.as_numpy_bits(o_fused)[keep], want[keep], "tail fused", **kw)


# ---------------------------------------------------------------- broadcast

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
@pytest.mark.parametrize("K,n", [(1, 5), (2, 4099), (8, (1 << 20) + 7), (16, 70001), (3, 1)])
def test_broadcast(dtype, K, n):
    from tests.parity_util import DT, make_peers
    hdt, odt = DT[dtype]
    src = make_peers(dtype, 1, n + 3, 950 + K, DEV, std=1.0)[0]
    for shift_src, shift_dst in ((0, 0), (1, 0), (0, 1), (1, 2)):
        s = src[shift_src:shift_src + n]
        bufs = [torch.zeros(n + 8, dtype=dtype, device=DEV) for _ in range(K)]
        dsts = [b[(shift_dst + j) % 3:(shift_dst + j) % 3 + n] for j, b in enumerate(bufs)]
        hfr.hfr_broadcast(s, dsts, K, n, hdt)
        torch.cuda.synchronize()
        want = oracle.broadcast(synth.as_numpy_bits(s), K, odt)
        for j in range(K):
            got = synth.as_numpy_bits(dsts[j])
            assert np.array_equal(got.view(np.uint32) if dtype == torch.float32 else got,
                                  want[j].view(np.uint32) if dtype == torch.float32 else want[j]), (j, shift_src, shift_dst)
            o = (shift_dst + j) % 3
            assert not bufs[j][:o].any() and not bufs[j][o + n:].any()    # nothing outside the view
    # a destination equal to the source is allowed
    d2 = torch.zeros(n, dtype=dtype, device=DEV)
    s = src[:n]
    keep = s.clone()
    hfr.hfr_broadcast(s, [s, d2], 2, n, hdt)
    torch.cuda.synchronize()
    assert torch.equal(s.view(torch.int16 if dtype != torch.float32 else torch.int32),
                       keep.view(torch.int16 if dtype != torch.float32 else torch.int32))
    assert torch.equal(d2.view(torch.int16 if dtype != torch.float32 else torch.int32),
                       keep.view(torch.int16 if dtype != torch.float32 else torch.int32))


@pytest.mark.parametrize("grid", [1, 3, 256, 0])
@pytest.mark.parametrize("K", [3, 8, 16])
def test_broadcast_bulk_shape(K, grid):
    """The broadcast's bulk shape (tiles parked in registers, one destination
    after the other) forced onto small inputs: several bursts per workgroup, an
    uneven last burst, a partial tile, a byte tail, nothing written outside."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, grid)
    for n in (256 * 16 * 70 + 16 * 9 + 5, 256 * 16 * 33 * 3, 4096 * 3 + 1, 100, 16):   # bytes (fp8 elements)
        src = synth.normal_fp8(n, 1.0, 940 + K, "e5m2", DEV)
        bufs = [torch.zeros(n + 32, dtype=torch.float8_e5m2, device=DEV) for _ in range(K)]
        dsts = [b[16:16 + n] for b in bufs]                  # 16-byte aligned views with guard bands
        hfr.hfr_broadcast(src, dsts, K, n, hfr.HFR_FP8_E5M2)
        torch.cuda.synchronize()
        want = synth.as_numpy_bits(src)
        for j, b in enumerate(bufs):
            got = synth.as_numpy_bits(b)
            assert np.array_equal(got[16:16 + n], want), (K, grid, n, j)
            assert not got[:16].any() and not got[16 + n:].any(), (K, grid, n, j)


def test_broadcast_bulk_shape_full_size():
    """128 MiB to eight destinations: the default launch of the bulk shape."""
    n = 1 << 26
    src = synth.normal_bf16(n, 1e-3, 945, DEV)
    dsts = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for _ in range(8)]
    hfr.hfr_broadcast(src, dsts, 8, n, hfr.HFR_BF16)
    torch.cuda.synchronize()
    for d in dsts:
        assert torch.equal(d.view(torch.int16), src.view(torch.int16))


def test_broadcast_large_over_segments():
    n = (1 << 25) + (1 << 23) + 4099       # fp32: more than one 128 MiB launch segment
    src = synth.uniform_pm1(n, 960, DEV)
    dsts = [torch.empty(n, dtype=torch.float32, device=DEV) for _ in range(3)]
    hfr.hfr_broadcast(src, dsts, 3, n, hfr.HFR_F32)
    torch.cuda.synchronize()
    for d in dsts:
        assert torch.equal(d.view(torch.int32), src.view(torch.int32))


# ------------------------------------------------- chunk table on the device

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.float8_e4m3fn])
@pytest.mark.parametrize("K", [1, 3, 8, 16])
def test_chunk_table_in_device_memory(dtype, K):
    """One launch over a table of chunks of every awkward size (empty, shorter
    than a vector, ragged, element-aligned views, one long chunk far above the
    hint, in place), written to device memory by a copy on the same stream."""
    from tests.parity_util import DT, make_peers
    hdt, odt = DT[dtype]
    rng = np.random.default_rng(1200 + K)
    sizes = [0, 1, 3, 15, 16, 17, 255, 4096, 4099, 70001] + [int(x) for x in rng.integers(1, 30000, size=120)]
    sizes[50] = (3 << 20) + 11                   # far above the hint: the tile loop strides
    total = sum(s + 19 for s in sizes)
    flats = make_peers(dtype, K, total, 1210, DEV, std=1.0)
    out = torch.zeros(total, dtype=dtype, device=DEV)
    chunks, off = [], 0
    for i, sz in enumerate(sizes):
        shift = (0, 0, 1, 3)[i % 4]              # half of the chunks are 16-byte aligned (offsets are multiples of 16 elements + shift)
        o = (off + 15) // 16 * 16 + shift
        dst = flats[0][o:o + sz] if i % 7 == 3 else out[o:o + sz]      # some chunks in place on input 0
        chunks.append(([f[o:o + sz] for f in flats], dst, sz))
        off = o + sz
    want = [oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt) if n else None for ins, _, n in chunks]
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        table = hfr.make_chunk_table(chunks, DEV)                         # the copy is ordered before the launch
        hfr.hfr_reduce_chunk_table(table, len(chunks), 8192, K, hdt, s)
    s.synchronize()
    f16 = dtype == torch.float16
    fp8 = "e4m3" if dtype == torch.float8_e4m3fn else ""
    for i, (ins, dst, n) in enumerate(chunks):
        if n:
            assert_bitwise(synth.as_numpy_bits(dst), want[i], "chunk %d n=%d" % (i, n), f16=f16, fp8=fp8)
    # nothing was written between the chunks
    mask = torch.ones(total, dtype=torch.bool, device=DEV)
    for ins, dst, n in chunks:
        if n and dst.data_ptr() >= out.data_ptr() and dst.data_ptr() < out.data_ptr() + total * out.element_size():
            o = (dst.data_ptr() - out.data_ptr()) // out.element_size()
            mask[o:o + n] = False
    assert not out.view(torch.uint8 if out.element_size() == 1 else (torch.int16 if out.element_size() == 2 else torch.int32))[mask].any()


def test_chunk_table_latency_workload_and_long_table():
    """The latency workload (256 chunks of 64 KiB, K = 8, fp32) in one launch,
    and a table longer than the launch's grid is tall (70000 tiny chunks)."""
    K, ce = 8, 16384
    n = 256 * ce
    ins = synth.peer_buffers_uniform_f32(K, n, 4000, DEV)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    table = hfr.make_chunk_table([([t[c * ce:(c + 1) * ce] for t in ins], out[c * ce:(c + 1) * ce], ce) for c in range(256)], DEV)
    hfr.hfr_reduce_chunk_table(table, 256, ce, K, hfr.HFR_F32)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "256 chunks")
    out.zero_()
    small = 40
    nch = 70000
    table = hfr.make_chunk_table([([t[c * small:(c + 1) * small] for t in ins[:2]], out[c * small:(c + 1) * small], small)
                                  for c in range(nch)], DEV)
    hfr.hfr_reduce_chunk_table(table, nch, small, 2, hfr.HFR_F32)
    torch.cuda.synchronize()
    want = oracle_reduce_sum([t[:nch * small] for t in ins[:2]])
    assert_bitwise(synth.as_numpy_bits(out[:nch * small]), want, "70000 chunks")
    assert not out[nch * small:].any()


# ------------------------------------------------------- batched launches

@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K", [1, 2, 8, 16])
def test_batched_many_small_buckets(dtype, K):
    """More buckets than one launch's table holds, of every awkward size
    (empty, shorter than a vector, ragged, shifted views, one big bucket in the
    middle), against the oracle bucket by bucket."""
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    rng = np.random.default_rng(900 + K)
    sizes = [0, 1, 3, 7, 8, 9, 255, 256, 257, 2048, 4099, 70001] + [int(x) for x in rng.integers(1, 20000, size=150)]
    sizes[100] = (5 << 20) + 11          # above the 8 MiB folding limit: gets a launch of its own
    sizes[60] = 0
    total = sum(s + 3 for s in sizes)
    if dtype == torch.float32:
        flats = synth.peer_buffers_uniform_f32(K, total, 910, DEV)
    else:
        flats = synth.peer_buffers_normal_bf16(K, total, 1.0, 910, DEV)
    out = torch.zeros(total, dtype=dtype, device=DEV)
    buckets, host = [], []
    off = 0
    for i, sz in enumerate(sizes):
        sh = i % 3                       # 0..2 elements of shift: mixed alignment classes
        ins = [f[off + sh: off + sh + sz] for f in flats]
        buckets.append((ins, out[off + sh: off + sh + sz], sz))
        host.append(([synth.as_numpy_bits(t) for t in ins], np.empty(sz, dtype=np.float32 if dtype == torch.float32 else np.uint16)))
        off += sz + 3
    hfr.hfr_reduce_buckets_batched(buckets, len(buckets), K, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_buckets(host, odt)
    for i, (b, w) in enumerate(zip(buckets, want)):
        assert_bitwise(synth.as_numpy_bits(b[1]), w, "batched bucket %d (n=%d)" % (i, sizes[i]))
    # the gaps between buckets were never written
    o = synth.as_numpy_bits(out)
    off = 0
    for i, sz in enumerate(sizes):
        sh = i % 3
        assert not o[off:off + sh].any() and not o[off + sh + sz: off + sz + 3].any()
        off += sz + 3


@pytest.mark.parametrize("K,chunk_bytes", [(2, 64 << 10), (8, 256 << 10), (16, 1 << 20), (4, 4 << 20)])
def test_batched_equals_chunked_schedule_on_the_latency_workload(K, chunk_bytes):
    chunk_elems = chunk_bytes // 4
    n = 256 * chunk_elems
    ins = synth.peer_buffers_uniform_f32(K, n, 4000, DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    chunks = [([t[c * chunk_elems:(c + 1) * chunk_elems] for t in ins], out[c * chunk_elems:(c + 1) * chunk_elems],
               chunk_elems) for c in range(256)]
    hfr.hfr_reduce_buckets_batched(chunks, 256, K, hfr.HFR_F32)
    flat = gpu_reduce_sum(ins)
    torch.cuda.synchronize()
    assert torch.equal(flat.view(torch.int32), out.view(torch.int32))
    for c in (0, 100, 255):
        sl = slice(c * chunk_elems, (c + 1) * chunk_elems)
        want = oracle.reduce_sum([synth.as_numpy_bits(t[sl]) for t in ins], oracle.F32)
        assert_bitwise(synth.as_numpy_bits(out[sl]), want, "batched chunk %d" % c)


@pytest.mark.parametrize("fold", [0, 1, -1])
@pytest.mark.parametrize("K,dtype", [(2, torch.float32), (8, torch.bfloat16), (16, torch.float32), (5, torch.bfloat16)])
def test_buckets_fold_small_chunks_across_table_capacity_with_mixed_alignment(K, dtype, fold):
    """One hfr_reduce_buckets call whose small chunks fill several batched
    launches (more chunks than one kernel-argument table holds), with buckets
    that start at shifted, element-aligned addresses next to 16-byte aligned
    ones, ragged last chunks, a bucket shorter than a vector, an empty bucket
    and one chunk too large to fold. Every schedule (folded on the caller's
    stream, folded over the worker streams, one launch per chunk) must give the
    oracle's bits and leave the gaps between buckets untouched."""
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    es = 4 if dtype == torch.float32 else 2
    chunk = 3000
    # the chunks of one bucket follow each other in memory and are merged into one table entry, so the
    # tables are filled by many buckets (each at most a few chunks long, 8 elements apart)
    sizes = ([20 * chunk + 17, 5, 0, 33 * chunk, 1, 4099, 64 * chunk + 2999, (9 << 20) // es + 11, 7 * chunk + 1] +
             [chunk, chunk - 1, 17, 2 * chunk + 5, 1, chunk // 2, 0, chunk] * 40)
    n_entries = sum(1 for sz in sizes if sz > 0)
    assert n_entries > 3 * (3824 // (8 * (K + 3)))         # several full tables
    pad = 8
    total = sum(sz + pad for sz in sizes)
    if dtype == torch.float32:
        flats = synth.peer_buffers_uniform_f32(K, total, 1700 + K, DEV)
    else:
        flats = synth.peer_buffers_normal_bf16(K, total, 1.0, 1700 + K, DEV)
    out = torch.zeros(total, dtype=dtype, device=DEV)
    buckets, host, off = [], [], 0
    for i, sz in enumerate(sizes):
        sh = (0, 1, 3, 0, 2)[i % 5]                      # element shifts: mixed 16-byte alignment inside one table
        ins = [f[off + sh: off + sh + sz] for f in flats]
        buckets.append((ins, out[off + sh: off + sh + sz], sz))
        host.append(([synth.as_numpy_bits(t) for t in ins], np.empty(sz, dtype=np.float32 if es == 4 else np.uint16)))
        off += sz + pad
    want = oracle.reduce_buckets(host, odt)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, fold)
    try:
        hfr.hfr_reduce_buckets(buckets, len(buckets), K, hdt, chunk, 4)
        torch.cuda.synchronize()
    finally:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, 0)
    for i, (b, w) in enumerate(zip(buckets, want)):
        assert_bitwise(synth.as_numpy_bits(b[1]), w, "fold=%d bucket %d (n=%d)" % (fold, i, sizes[i]))
    o = synth.as_numpy_bits(out)
    off = 0
    for i, sz in enumerate(sizes):
        sh = (0, 1, 3, 0, 2)[i % 5]
        assert not o[off:off + sh].any() and not o[off + sh + sz: off + sz + pad].any(), "gap after bucket %d" % i
        off += sz + pad


@pytest.mark.parametrize("fold", [0, -1])
@pytest.mark.parametrize("K,dtype,seg_mib", [(6, torch.bfloat16, 1), (8, torch.float32, 0), (13, torch.bfloat16, 2)])
def test_buckets_merge_adjacent_bulk_chunks_into_longer_launches(K, dtype, seg_mib, fold):
    """Bulk chunks that follow each other in memory (every input and the output)
    run as one longer launch, cut into equal segments: chunks of one bucket with
    a ragged last chunk, a second bucket cut from the same flat buffers right
    behind it, a bucket behind a gap, one whose output lies elsewhere, an
    element-shifted bucket (wide shape) between two runs, two adjacent in-place
    buckets. Merged (default) and one launch per chunk must both give the
    oracle's bits and leave everything around the buckets untouched."""
    hdt, odt = (hfr.HFR_F32, oracle.F32) if dtype == torch.float32 else (hfr.HFR_BF16, oracle.BF16)
    es = 4 if dtype == torch.float32 else 2
    npdt = np.float32 if es == 4 else np.uint16
    chunk = (300 << 10) // es                                  # 300 KiB per buffer and chunk
    a, b, c, d, e, f, g = 5 * chunk + 4096, 3 * chunk, 2 * chunk + 64, 4 * chunk, chunk + 8, 2 * chunk, 3 * chunk + 16
    gap = 64
    total = a + b + gap + c + d + gap + e + 1 + f + g + gap
    if dtype == torch.float32:
        flats = synth.peer_buffers_uniform_f32(K, total, 2300 + K, DEV)
    else:
        flats = synth.peer_buffers_normal_bf16(K, total, 1.0, 2300 + K, DEV)
    out = torch.zeros(total, dtype=dtype, device=DEV)
    other = torch.zeros(d + 2 * gap, dtype=dtype, device=DEV)
    spans, off = [], 0
    for name, sz, lead in (("a", a, 0), ("b", b, 0), ("c", c, gap), ("d", d, 0), ("e", e, gap + 1), ("f", f, 0), ("g", g, 0)):
        off += lead
        spans.append((name, off, sz))
        off += sz
    buckets, host, keep = [], [], []
    for name, o, sz in spans:
        ins = [t[o:o + sz] for t in flats]
        if name == "d":
            dst = other[gap:gap + sz]                          # inputs continue the run, the output does not
        elif name in ("f", "g"):
            dst = ins[1]                                       # in place on input 1, f and g adjacent
        else:
            dst = out[o:o + sz]
        buckets.append((ins, dst, sz))
        host.append(([synth.as_numpy_bits(t).copy() for t in ins], np.empty(sz, dtype=npdt)))
        keep.append(dst)
    want = oracle.reduce_buckets(host, odt)
    untouched = synth.as_numpy_bits(flats[1]).copy()
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)          # every 16-byte aligned chunk of K >= 5 inputs is bulk
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 5)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_SEGMENT_MIB, seg_mib)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, fold)
    try:
        hfr.hfr_reduce_buckets(buckets, len(buckets), K, hdt, chunk, 4)
        torch.cuda.synchronize()
    finally:
        for knob in (hfr.HFR_TUNE_BULK_MIN_BYTES, hfr.HFR_TUNE_BULK_GRID, hfr.HFR_TUNE_SEGMENT_MIB, hfr.HFR_TUNE_BUCKET_FOLD):
            hfr.hfr_set_tuning(knob, 0)
    for (name, o, sz), dst, w in zip(spans, keep, want):
        assert_bitwise(synth.as_numpy_bits(dst), w, "fold=%d bucket %s (n=%d)" % (fold, name, sz))
    o_bits = synth.as_numpy_bits(out)
    covered = np.zeros(total, dtype=bool)
    for name, o, sz in spans:
        if name not in ("d", "f", "g"):
            covered[o:o + sz] = True
    assert not o_bits[~covered].any(), "bytes of `out` outside the buckets were written"
    ob = synth.as_numpy_bits(other)
    assert not ob[:gap].any() and not ob[gap + d:].any(), "bytes around the stray output were written"
    inplace = np.zeros(total, dtype=bool)
    for name, o, sz in spans:
        if name in ("f", "g"):
            inplace[o:o + sz] = True
    assert np.array_equal(bits(synth.as_numpy_bits(flats[1]))[~inplace], bits(untouched)[~inplace]), "input 1 outside f and g changed"


@pytest.mark.parametrize("fold", [0, -1])
def test_a_ragged_tail_joins_the_run_it_continues(fold):
    """Library defaults, sizes that take the bulk shape by themselves: a bucket
    of 55 MiB per buffer in chunks of 25Mi elements (50 MiB, bulk, and a 5 MiB
    tail that is not) and a second bucket of 30 MiB right behind it in the same
    flat buffers. By default the three chunks run as one sum of 85 MiB; with
    folding off as three launches. Same bits, nothing written past the end."""
    K, mib = 8, 1 << 20
    n1, n2, pad = 55 * mib // 2, 30 * mib // 2 + 24, 4096
    flats = synth.peer_buffers_normal_bf16(K, n1 + n2 + pad, 1e-3, 2600, DEV)
    out = torch.zeros(n1 + n2 + pad, dtype=torch.bfloat16, device=DEV)
    buckets = [([f[:n1] for f in flats], out[:n1], n1), ([f[n1:n1 + n2] for f in flats], out[n1:n1 + n2], n2)]
    want = oracle_reduce_sum([f[:n1 + n2] for f in flats])
    hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, fold)
    try:
        hfr.hfr_reduce_buckets(buckets, 2, K, hfr.HFR_BF16, synth.BUCKET_CAP_ELEMS, 4)
        torch.cuda.synchronize()
    finally:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, 0)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, 0)
    assert_bitwise(synth.as_numpy_bits(out[:n1 + n2]), want, "fold=%d" % fold)
    assert not synth.as_numpy_bits(out[n1 + n2:]).any(), "bytes past the last bucket were written"


def test_long_inputs_are_cut_into_equal_segments_to_the_mib():
    """2.3 MiB per buffer with 1 MiB segments: three launches of 1 MiB, 1 MiB
    and the rest; 5 MiB + 3 elements with 2 MiB segments: three of 2, 2 and the
    rest (segments are rounded up to whole MiB). The bits do not depend on it."""
    for K, n, seg in ((8, (2300 << 10) // 2, 1), (5, (5 << 20) // 2 + 3, 2), (3, (3 << 20) // 2 + 1, 1)):
        ins = synth.peer_buffers_normal_bf16(K, n, 1e-2, 2400 + K, DEV)
        out = torch.empty_like(ins[0])
        hfr.hfr_set_tuning(hfr.HFR_TUNE_SEGMENT_MIB, seg)
        try:
            hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16)
            torch.cuda.synchronize()
        finally:
            hfr.hfr_set_tuning(hfr.HFR_TUNE_SEGMENT_MIB, 0)
        assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "K=%d n=%d segments of %d MiB" % (K, n, seg))


def test_a_stale_runtime_error_is_not_blamed_on_a_launch():
    """An unrelated HIP call that failed earlier on this thread leaves its code
    in the runtime's last-error slot; the library's launches report their own
    status, so the next entry point must still return HFR_OK."""
    import ctypes
    hip = None
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                hip = ctypes.CDLL(line.split()[-1])
                break
    assert hip is not None
    hip.hipDeviceGetAttribute.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.c_int, ctypes.c_int]
    hip.hipDeviceGetAttribute.restype = ctypes.c_int
    ins = synth.peer_buffers_uniform_f32(3, 70001, 1800, DEV)
    out = torch.empty_like(ins[0])
    torch.cuda.synchronize()
    v = ctypes.c_int(0)
    assert hip.hipDeviceGetAttribute(ctypes.byref(v), 987654, 0) != 0      # an attribute that does not exist
    assert hfr.hfr_reduce_sum(ins, 3, out, 70001, hfr.HFR_F32, check=False) == hfr.HFR_OK
    assert hfr.hfr_combine_avg(ins[0], ins[1], out, 70001, 0.5, hfr.HFR_F32, check=False) == hfr.HFR_OK
    assert hfr.hfr_broadcast(ins[0], [out], 1, 70001, hfr.HFR_F32, check=False) == hfr.HFR_OK
    hip.hipGetLastError.restype = ctypes.c_int
    hip.hipGetLastError()                                                   # leave the slot clean for later tests
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), synth.as_numpy_bits(ins[0]), "after a stale error")


# ----------------------------------------------- launch shape never matters

def _check_all_ops(n, tag):
    ins = synth.peer_buffers_normal_bf16(8, n, 1e-3, 300, DEV)
    check_reduce_sum(ins, tag + " bf16 K8")
    ins = synth.peer_buffers_uniform_f32(3, n, 301, DEV)
    check_reduce_sum(ins, tag + " f32 K3")
    a, b = ins[0], ins[1]
    out = torch.empty_like(a)
    hfr.hfr_combine_avg(a, b, out, n, 0.3, hfr.HFR_F32)
    torch.cuda.synchronize()
    want = oracle.combine_avg(synth.as_numpy_bits(a), synth.as_numpy_bits(b), 0.3, oracle.F32)
    assert_bitwise(synth.as_numpy_bits(out), want, tag + " combine")


@pytest.mark.parametrize("unroll", [1, 2, 4])
@pytest.mark.parametrize("grid_cap", [1, 7, 256, 0])
def test_wide_shape_knobs_do_not_change_results(unroll, grid_cap):
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, -1)  # wide shape only
    hfr.hfr_set_tuning(hfr.HFR_TUNE_UNROLL, unroll)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_GRID_CAP, grid_cap)
    n = 256 * 4 * 8 * 9 + 1234  # several tiles of every unroll plus a ragged end
    _check_all_ops(n, "wide u%d g%d" % (unroll, grid_cap))


@pytest.mark.parametrize("bulk_grid", [1, 3, 64, 256, 1000, 0])
@pytest.mark.parametrize("n", [256 * 8 * 8 * 70 + 4321, 256 * 8 * 5 + 9, 100])
def test_bulk_shape_knobs_do_not_change_results(bulk_grid, n):
    """The lock-step shape forced onto small inputs: whole tiles spread over
    several store bursts, a partial tile, a scalar tail, idle workgroups."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)   # bulk shape always
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, bulk_grid)
    _check_all_ops(n, "bulk g%d n%d" % (bulk_grid, n))


@pytest.mark.parametrize("trips_per_wg", [31, 33, 36, 47, 65, 100])
def test_bulk_shape_bursts_split_evenly(trips_per_wg):
    """A workgroup's trips are split evenly over its store bursts (33 trips run
    as 17 + 16, not 32 + 1): sizes that give every burst fewer trips than the
    kernel's register tile holds, a last burst that is shorter still, and a
    last workgroup with one trip less."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 3)
    n = 256 * 8 * (3 * trips_per_wg - 1) + 777
    _check_all_ops(n, "bulk %d trips" % trips_per_wg)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("K", list(range(1, 17)))
def test_every_k_bulk_shape(dtype, K):
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 5)        # many trips and bursts per workgroup
    n = 256 * 8 * 8 * 40 + 777
    if dtype == torch.float32:
        ins = synth.peer_buffers_uniform_f32(K, n, 170 + K, DEV)
    else:
        ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 170 + K, DEV)
    check_reduce_sum(ins, "bulk K=%d" % K)
    # shifted views: element alignment only (such buffers take the wide shape whatever the knob says),
    # in place on input 0
    base = [t for t in ins]
    views = [t[1:n - 2] for t in base]
    want = oracle_reduce_sum(views)
    gpu_reduce_sum(views, views[0])
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(views[0]), want, "bulk misaligned in place K=%d" % K)


# ------------------------------------------------------- stream semantics

def test_buckets_respect_stream_order_and_buffer_reuse():
    """The ring forks from and joins back into the caller's stream: work
    enqueued before is seen, work enqueued after sees every chunk. The same
    output buffer is reused back to back with different inputs."""
    K, n = 4, 1 << 20
    s = torch.cuda.Stream()
    sets = [synth.peer_buffers_uniform_f32(K, n, 500 + 10 * r, DEV) for r in range(3)]
    wants = [oracle_reduce_sum(ins) for ins in sets]
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    copies = []
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for r, ins in enumerate(sets):
            staged = [torch.empty_like(t) for t in ins]
            for d, t in zip(staged, ins):
                d.copy_(t, non_blocking=True)       # producer on the caller's stream
            hfr.hfr_reduce_buckets([(staged, out, n)], 1, K, hfr.HFR_F32, 8192, 4, s)
            copies.append(out.clone())              # consumer on the caller's stream
    s.synchronize()
    for r in range(3):
        assert_bitwise(synth.as_numpy_bits(copies[r]), wants[r], "round %d" % r)


def test_buckets_mixed_bulk_and_small_chunks_keep_stream_order():
    """A list that mixes buckets large enough for the bulk launch shape (kept on
    the caller's stream), mid-size ones (kept there too when bulk chunks are
    present) and tiny ones (dealt over the worker ring): producer work enqueued
    before the call is seen by every chunk, consumer work enqueued after it
    sees every chunk, whichever stream a chunk ran on."""
    K = 8
    sizes = [1 << 20, 25 * (1 << 20), 3 << 20, 777, 25 * (1 << 20), 1 << 19, 5]
    total = sum(sizes)
    s = torch.cuda.Stream()
    src = synth.peer_buffers_normal_bf16(K, total, 1e-3, 1400, DEV)
    want = oracle_reduce_sum(src)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        staged = [torch.empty_like(t) for t in src]
        for d, t in zip(staged, src):
            d.copy_(t, non_blocking=True)                  # producer on the caller's stream
        out = torch.zeros(total, dtype=torch.bfloat16, device=DEV)
        buckets, off = [], 0
        for sz in sizes:
            buckets.append(([t[off:off + sz] for t in staged], out[off:off + sz], sz))
            off += sz
        hfr.hfr_reduce_buckets(buckets, len(buckets), K, hfr.HFR_BF16, 1 << 30, 4, s)
        snapshot = out.clone()                             # consumer on the caller's stream
        # second call right behind the first, chunked finely: small chunks everywhere
        out2 = torch.zeros_like(out)
        b2 = [([t[o:o + l] for t in staged], out2[o:o + l], l) for o, l in synth.bucket_cuts(total, 6 << 20)]
        hfr.hfr_reduce_buckets(b2, len(b2), K, hfr.HFR_BF16, 1 << 19, 4, s)
        snapshot2 = out2.clone()
    s.synchronize()
    assert_bitwise(synth.as_numpy_bits(snapshot), want, "mixed bulk/small")
    assert_bitwise(synth.as_numpy_bits(snapshot2), want, "fine chunks")


def test_bucket_schedule_can_be_captured_into_a_hip_graph():
    """The fork / join of the worker ring is plain event work, so a caller may
    capture the call into a HIP graph. Replayed several times, with eager work
    and synchronisations in between, every replay must give the oracle's bits."""
    K, chunk = 4, 1 << 16
    n = 64 * chunk
    ins = synth.peer_buffers_uniform_f32(K, n, 1500, DEV)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    want = oracle_reduce_sum(ins)
    s = torch.cuda.Stream()
    hfr.hfr_init()                                         # worker streams exist before the capture
    arr = hfr.make_bucket_array([(ins, out, n)])
    with torch.cuda.stream(s):
        hfr.hfr_reduce_buckets(arr, 1, K, hfr.HFR_F32, chunk, 4, s)   # eager once
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "eager")
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        hfr.hfr_reduce_buckets(arr, 1, K, hfr.HFR_F32, chunk, 4, s)
    for rep in range(4):
        out.zero_()                                        # eager work between replays
        scratch = torch.rand(1 << 20, device=DEV).sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), want, "graph replay %d" % rep)
    del g


def test_device_info_matches_the_runtime():
    cus, clock_khz, bus_bits = hfr.hfr_device_info()
    assert cus == torch.cuda.get_device_properties(0).multi_processor_count
    assert clock_khz >= 0 and bus_bits >= 0
    if clock_khz and bus_bits:                       # HBM3E: thousands of bits wide, GHz-class clock
        assert bus_bits >= 1024 and clock_khz >= 100_000
    L = hfr.lib()                                    # every pointer may be NULL
    assert L.hfr_device_info(None, None, None) == hfr.HFR_OK


def test_init_shutdown_cycle():
    assert hfr.hfr_init() == hfr.HFR_OK
    n = 100000
    ins = synth.peer_buffers_uniform_f32(2, n, 600, DEV)
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    hfr.hfr_reduce_buckets([(ins, out, n)], 1, 2, hfr.HFR_F32, 1000, 8)
    torch.cuda.synchronize()
    assert hfr.hfr_shutdown() == hfr.HFR_OK
    assert hfr.hfr_shutdown() == hfr.HFR_OK
    hfr.hfr_reduce_buckets([(ins, out, n)], 1, 2, hfr.HFR_F32, 1000, 8)  # pool comes back on demand
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "after shutdown")
