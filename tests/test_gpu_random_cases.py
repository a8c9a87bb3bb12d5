"""Seeded random sweep over the whole C ABI: entry point, element type, K, n,
element misalignment, in-place output, chunking and every launch-shape knob
drawn at random; each case is compared with the oracle bit for bit. The cases
are reproducible from the seed printed on failure."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import assert_bitwise

pytestmark = pytest.mark.gpu
DEV = "cuda"

KINDS = {
    "f32": (torch.float32, hfr.HFR_F32, oracle.F32, 4),
    "bf16": (torch.bfloat16, hfr.HFR_BF16, oracle.BF16, 2),
    "f16": (torch.float16, hfr.HFR_F16, oracle.F16, 2),
    "e4m3": (torch.float8_e4m3fn, hfr.HFR_FP8_E4M3, oracle.FP8_E4M3, 1),
    "e5m2": (torch.float8_e5m2, hfr.HFR_FP8_E5M2, oracle.FP8_E5M2, 1),
}
KNOBS = (hfr.HFR_TUNE_GRID_CAP, hfr.HFR_TUNE_UNROLL, hfr.HFR_TUNE_BULK_GRID, hfr.HFR_TUNE_BULK_MIN_BYTES,
         hfr.HFR_TUNE_BULK_SKEW, hfr.HFR_TUNE_BULK_BLOCK, hfr.HFR_TUNE_BULK_PACE, hfr.HFR_TUNE_WIDE_WGS_PER_CU,
         hfr.HFR_TUNE_BUCKET_FOLD, hfr.HFR_TUNE_SEGMENT_MIB, hfr.HFR_TUNE_BUCKET_LIST)


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    for knob in KNOBS:
        hfr.hfr_set_tuning(knob, 0)
    hfr.hfr_shutdown()


def _buffer(kind, n, seed, shift):
    """n elements of `kind` starting `shift` elements into a fresh allocation."""
    if kind == "f32":
        t = synth.normal_f32(n + shift, 1.0, seed, DEV)
    elif kind == "bf16":
        t = synth.normal_bf16(n + shift, 1e-2, seed, DEV)
    elif kind == "f16":
        t = synth.normal_f16(n + shift, 1e-1, seed, DEV)
    else:
        t = synth.normal_fp8(n + shift, 2.0, seed, kind, DEV)
    return t[shift:]


def _cmp(got, want, kind, what):
    assert_bitwise(synth.as_numpy_bits(got), want, what, f16=(kind == "f16"),
                   fp8=(kind if kind in ("e4m3", "e5m2") else ""))


def _random_knobs(rng):
    hfr.hfr_set_tuning(hfr.HFR_TUNE_GRID_CAP, int(rng.choice([0, 0, 1, 3, 64, 300])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_UNROLL, int(rng.choice([0, 0, 1, 2, 4])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, int(rng.choice([0, 1, 2, 5, 17, 256])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, int(rng.choice([0, -1, 1, 1, 4096])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, int(rng.choice([0, -1, 1, 2, 3])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_BLOCK, int(rng.choice([0, 0, 64, 160, 256, 384])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_PACE, int(rng.choice([0, 0, -1, 3, 16])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_WIDE_WGS_PER_CU, int(rng.choice([0, 0, -1, 1, 3])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_FOLD, int(rng.choice([0, 0, 0, 1, -1])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_SEGMENT_MIB, int(rng.choice([0, 0, 0, 1])))
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_LIST, int(rng.choice([0, 0, -1, 1, 1])))


def _random_n(rng):
    pick = rng.integers(0, 6)
    if pick == 0:
        return int(rng.integers(0, 40))
    if pick == 1:
        return int(rng.integers(40, 5000))
    if pick == 2:                                   # whole tiles of some unroll, plus or minus a little
        return max(0, int(256 * 16 * rng.integers(1, 40) + rng.integers(-3, 4)))
    return int(rng.integers(5000, 400000))


def _one_case(rng, case):
    kind = str(rng.choice(list(KINDS)))
    tdt, hdt, odt, es = KINDS[kind]
    op = str(rng.choice(["sum", "sum", "avg", "combine", "fused", "slice", "buckets", "batched", "table", "broadcast"]))
    K = int(rng.integers(1, 17))
    n = _random_n(rng)
    shifts = [int(rng.choice([0, 0, 0, 1, 3, 8])) for _ in range(K + 2)]
    if rng.random() < 0.5:
        shifts = [0] * (K + 2)                      # fully 16-byte aligned: the fast paths
    seed = 7000 + 37 * case
    scale = float(rng.choice([1.0, 0.5, 1.0 / 3.0, 1.0 / 128, 0.1]))
    what = "case %d: %s %s K=%d n=%d shifts=%s scale=%r" % (case, op, kind, K, n, shifts[:4], scale)
    _random_knobs(rng)

    if op == "combine":
        a, b = _buffer(kind, n, seed, shifts[0]), _buffer(kind, n, seed + 1, shifts[1])
        ha, hb = synth.as_numpy_bits(a), synth.as_numpy_bits(b)
        want = oracle.combine_avg(ha, hb, scale, odt)
        out = a if rng.random() < 0.4 else _buffer(kind, n, seed + 2, shifts[2])
        hfr.hfr_combine_avg(a, b, out, n, scale, hdt)
        torch.cuda.synchronize()
        return _cmp(out, want, kind, what)

    if op == "broadcast":
        src = _buffer(kind, n, seed, shifts[0])
        dsts = [_buffer(kind, n, seed + 1 + j, shifts[1 + (j % 2)]) for j in range(K)]
        hfr.hfr_broadcast(src, dsts, K, n, hdt)
        torch.cuda.synchronize()
        want = synth.as_numpy_bits(src)
        for j, d in enumerate(dsts):
            assert np.array_equal(synth.as_numpy_bits(d), want), what + " dst %d" % j
        return None

    ins = [_buffer(kind, n, seed + j, shifts[j]) for j in range(K)]
    host = [synth.as_numpy_bits(t) for t in ins]
    fresh = _buffer(kind, n, seed + 99, shifts[K])
    alias = int(rng.integers(0, K)) if rng.random() < 0.35 else None
    out = ins[alias] if alias is not None else fresh

    if op == "sum":
        want = oracle.reduce_sum(host, odt)
        hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    elif op == "avg":
        want = oracle.reduce_avg(host, scale, odt)
        hfr.hfr_reduce_avg(ins, K, out, n, scale, hdt)
    elif op == "fused":
        if K == 16:
            K, ins, host = 15, ins[:15], host[:15]
            if alias == 15:
                out = fresh
        remote = _buffer(kind, n, seed + 50, shifts[K + 1])
        partial = oracle.reduce_sum(host, odt)
        want = oracle.combine_avg(partial, synth.as_numpy_bits(remote), scale, odt)
        hfr.hfr_reduce_combine_avg(ins, K, remote, out, n, scale, hdt)
    elif op == "slice":
        world = int(rng.integers(1, 9))
        rank = int(rng.integers(0, world))
        want = synth.as_numpy_bits(out).copy()          # elements outside the slice keep their bytes
        oracle.reduce_scatter_slice(host, rank, world, odt, want)
        hfr.hfr_reduce_scatter_slice(ins, K, out, n, rank, world, hdt)
    else:
        # cut [0, n) into buckets at 16-byte multiples (views stay as aligned as their buffers)
        step = 16 // es
        # half of the bucket lists leave 16 bytes between buckets: adjacent buckets are merged by
        # hfr_reduce_buckets, buckets that lie apart take its folding and ring paths
        apart = op == "buckets" and rng.random() < 0.5
        cuts, off, covered = [], 0, np.zeros(n, dtype=bool)
        while off < n:
            ln = min(n - off, int(rng.integers(1, 6000)) * step)
            cuts.append((off, ln))
            covered[off:off + ln] = True
            off += ln + (step if apart else 0)
        if not cuts:
            cuts = [(0, 0)]
        want = oracle.reduce_sum(host, odt)
        if apart:
            before = synth.as_numpy_bits(out)
            want = np.where(covered, want, before)      # the gaps keep their bytes
        buckets = [([t[o:o + l] for t in ins], out[o:o + l], l) for o, l in cuts]
        if op == "buckets":
            chunk = int(rng.choice([1, 7, 1000, 4096, 1 << 30]))
            if chunk < 64 and n > 20000:
                chunk = 1000                            # keep the launch count of a case bounded
            hfr.hfr_reduce_buckets(buckets, len(buckets), K, hdt, chunk, int(rng.integers(1, 9)))
        elif op == "table":
            table = hfr.make_chunk_table(buckets, DEV)
            hfr.hfr_reduce_chunk_table(table, len(buckets), int(rng.choice([1, 777, 8192, 1 << 20])), K, hdt)
        else:
            hfr.hfr_reduce_buckets_batched(buckets, len(buckets), K, hdt)
    torch.cuda.synchronize()
    return _cmp(out, want, kind, what)


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6, 7, 8])
def test_random_cases_match_the_oracle(seed):
    rng = np.random.default_rng(seed)
    for case in range(100):
        _one_case(rng, seed * 1000 + case)
