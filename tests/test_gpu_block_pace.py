"""GPU parity of the bulk K-way sum for every workgroup size and pause the host
may choose (request pacing: a tile is as many vectors as the workgroup has
lanes, and a workgroup may pause after each trip). Neither changes which
operands are added in which order, so every combination must give the oracle's
bits: every element type, input counts on both sides of the kernels' launch
bounds, epilogues, skewed variants, in place, ragged sizes."""
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import assert_bitwise

pytestmark = pytest.mark.gpu
DEV = "cuda"

KNOBS = (hfr.HFR_TUNE_BULK_GRID, hfr.HFR_TUNE_BULK_MIN_BYTES, hfr.HFR_TUNE_BULK_SKEW, hfr.HFR_TUNE_PLACEMENT_ONLINE,
         hfr.HFR_TUNE_BULK_BLOCK, hfr.HFR_TUNE_BULK_PACE, hfr.HFR_TUNE_SEGMENT_MIB, hfr.HFR_TUNE_WIDE_WGS_PER_CU,
         hfr.HFR_TUNE_UNROLL, hfr.HFR_TUNE_GRID_CAP)


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    for knob in KNOBS:
        hfr.hfr_set_tuning(knob, 0)
    hfr.hfr_shutdown()


def _peers(kind, K, n, seed):
    if kind == "f32":
        return synth.peer_buffers_uniform_f32(K, n, seed, DEV), hfr.HFR_F32, oracle.F32
    if kind == "bf16":
        return synth.peer_buffers_normal_bf16(K, n, 1e-3, seed, DEV), hfr.HFR_BF16, oracle.BF16
    if kind == "f16":
        return synth.peer_buffers_normal_f16(K, n, 1e-2, seed, DEV), hfr.HFR_F16, oracle.F16
    return synth.peer_buffers_normal_fp8(K, n, 1.0, seed, kind, DEV), \
        (hfr.HFR_FP8_E4M3 if kind == "e4m3" else hfr.HFR_FP8_E5M2), \
        (oracle.FP8_E4M3 if kind == "e4m3" else oracle.FP8_E5M2)


VEC = {"f32": 4, "bf16": 8, "f16": 8, "e4m3": 16, "e5m2": 16}


def _fmt(kind):
    return dict(f16=(kind == "f16"), fp8=(kind if kind in ("e4m3", "e5m2") else ""))


def _force(block, pace, grid, skew=0):
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)      # the bulk shape whatever the size
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, grid)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_BLOCK, block)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_PACE, pace)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, skew)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)


@pytest.mark.parametrize("block", [64, 96, 160, 224, 256, 288, 352, 384])
@pytest.mark.parametrize("K", [1, 3, 5, 7, 8, 12, 16])
@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_every_workgroup_size_gives_the_oracles_sum(kind, K, block):
    """Three workgroups, 40 trips each whatever the tile size works out to
    (sizes above what a kernel was built for are clamped, so the tile is not
    always `block` vectors: the element count is chosen for 96-lane tiles and
    leaves whole tiles, a partial tile and a scalar tail for every other size)."""
    _force(block, 3 if block % 64 else 0, 3)
    n = 96 * VEC[kind] * (3 * 40 - 1) + 96 * VEC[kind] // 2 + 3
    ins, hdt, odt = _peers(kind, K, n, 1200 + K)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    assert_bitwise(synth.as_numpy_bits(out), want, "block %d %s K=%d" % (block, kind, K), **_fmt(kind))


@pytest.mark.parametrize("block,pace", [(64, 1), (192, 8), (320, 0), (384, 64)])
@pytest.mark.parametrize("K", [5, 9, 13])
@pytest.mark.parametrize("kind", ["f16", "e4m3", "e5m2"])
def test_workgroup_sizes_and_pauses_for_the_narrow_types(kind, K, block, pace):
    _force(block, pace, 5)
    n = 64 * VEC[kind] * (5 * 33 + 2) + 17
    ins, hdt, odt = _peers(kind, K, n, 1300 + K)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    assert_bitwise(synth.as_numpy_bits(out), want, "block %d pace %d %s K=%d" % (block, pace, kind, K), **_fmt(kind))


@pytest.mark.parametrize("block,pace", [(128, 2), (224, 0), (352, 5)])
@pytest.mark.parametrize("K", [6, 7, 8, 11])
@pytest.mark.parametrize("kind", ["bf16", "f32", "f16", "e4m3"])
def test_epilogues_and_in_place_under_block_and_pace(kind, K, block, pace):
    """The fused average, the fused combine (K peers + remote partial) and the
    plain sum written over input 0, all in the bulk shape with the chosen
    workgroup size and pause."""
    _force(block, pace, 7)
    n = 32 * VEC[kind] * (7 * 29 + 3) + 5
    ins, hdt, odt = _peers(kind, K + 1, n, 1400 + K)
    peers, remote = ins[:K], ins[K]
    host = [synth.as_numpy_bits(t) for t in peers]
    scale = 0.3
    out = torch.empty_like(peers[0])
    hfr.hfr_reduce_avg(peers, K, out, n, scale, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, scale, odt), "avg %s K=%d b%d" % (kind, K, block),
                   **_fmt(kind))
    hfr.hfr_reduce_combine_avg(peers, K, remote, out, n, scale, hdt)
    torch.cuda.synchronize()
    partial = oracle.reduce_sum(host, odt)
    want = oracle.combine_avg(partial, synth.as_numpy_bits(remote), scale, odt)
    assert_bitwise(synth.as_numpy_bits(out), want, "fused combine %s K=%d b%d" % (kind, K, block), **_fmt(kind))
    want = oracle.reduce_sum(host, odt)
    hfr.hfr_reduce_sum(peers, K, peers[0], n, hdt)          # in place on input 0
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(peers[0]), want, "in place %s K=%d b%d" % (kind, K, block), **_fmt(kind))


@pytest.mark.parametrize("skew", [1, 2, 3])
@pytest.mark.parametrize("block,pace", [(64, 0), (160, 4), (256, 1)])
@pytest.mark.parametrize("K", [8, 9])
def test_skewed_variants_under_block_and_pace(K, block, pace, skew):
    _force(block, pace, 3, skew)
    for kind in ("bf16", "f32"):
        n = 32 * VEC[kind] * (3 * 45 - 1) + 16 * VEC[kind] + 3
        ins, hdt, odt = _peers(kind, K, n, 1500 + K)
        out = torch.empty_like(ins[0])
        hfr.hfr_reduce_sum(ins, K, out, n, hdt)
        torch.cuda.synchronize()
        want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
        assert_bitwise(synth.as_numpy_bits(out), want, "skew %d block %d %s K=%d" % (skew, block, kind, K), **_fmt(kind))


@pytest.mark.parametrize("block,pace", [(64, 0), (224, 4), (384, 1)])
@pytest.mark.parametrize("K", [5, 7, 10, 16])
def test_pattern_three_of_the_other_input_counts_under_block_and_pace(K, block, pace):
    _force(block, pace, 3, 3)
    for kind in ("bf16", "e4m3"):
        n = 32 * VEC[kind] * (3 * 45 - 1) + 16 * VEC[kind] + 3
        ins, hdt, odt = _peers(kind, K, n, 1550 + K)
        out = torch.empty_like(ins[0])
        hfr.hfr_reduce_sum(ins, K, out, n, hdt)
        torch.cuda.synchronize()
        want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
        assert_bitwise(synth.as_numpy_bits(out), want, "pattern 3 block %d %s K=%d" % (block, kind, K), **_fmt(kind))


@pytest.mark.parametrize("kind", ["bf16", "f32", "f16", "e4m3", "e5m2"])
@pytest.mark.parametrize("K", list(range(5, 17)))
def test_the_tables_own_choice_for_every_type_and_k(kind, K):
    """The workgroup size and pause the library picks by itself (knobs at 0),
    at a size that takes the bulk shape without being forced to: whole chip,
    two bursts per workgroup, a ragged end."""
    for knob in KNOBS:
        hfr.hfr_set_tuning(knob, 0)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
    n = (24 << 20) // (16 // VEC[kind]) + 1237               # a little over 24 MiB per buffer
    ins, hdt, odt = _peers(kind, K, n, 1600 + K)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    assert_bitwise(synth.as_numpy_bits(out), want, "table %s K=%d" % (kind, K), **_fmt(kind))


@pytest.mark.parametrize("wgs", [-1, 1, 2, 3, 16])
@pytest.mark.parametrize("K", [1, 2, 3, 4, 7])
@pytest.mark.parametrize("kind", ["bf16", "f32", "e5m2"])
def test_wide_shape_with_a_bound_on_resident_workgroups(kind, K, wgs):
    """The wide shape with LDS reserved so that at most `wgs` workgroups share a
    compute unit (the reservation changes where workgroups run, never what they
    compute): plain sum, fused average, in place."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, -1)      # wide shape only
    hfr.hfr_set_tuning(hfr.HFR_TUNE_WIDE_WGS_PER_CU, wgs)
    n = 256 * VEC[kind] * 4 * 300 + 256 * VEC[kind] + 7       # a few hundred tiles, a partial one, a tail
    ins, hdt, odt = _peers(kind, K, n, 1700 + K)
    host = [synth.as_numpy_bits(t) for t in ins]
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum(host, odt), "wgs %d %s K=%d" % (wgs, kind, K), **_fmt(kind))
    hfr.hfr_reduce_avg(ins, K, out, n, 0.7, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, 0.7, odt), "wgs %d avg %s K=%d" % (wgs, kind, K),
                   **_fmt(kind))
    want = oracle.reduce_sum(host, odt)
    hfr.hfr_reduce_sum(ins, K, ins[K - 1], n, hdt)           # in place on the last input
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(ins[K - 1]), want, "wgs %d in place %s K=%d" % (wgs, kind, K), **_fmt(kind))


@pytest.mark.parametrize("K", [1, 3, 4])
def test_the_default_bound_at_a_size_that_takes_it(K):
    """48 MiB per buffer and more: the library bounds the resident workgroups of
    one-, three- and four-operand launches by itself."""
    n = (48 << 20) // 2 + 4099
    ins, hdt, odt = _peers("bf16", K, n, 1800 + K)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt), "default bound K=%d" % K)
