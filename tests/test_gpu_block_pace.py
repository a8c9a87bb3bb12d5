"""GPU parity of the bulk K-way sum for every workgroup size and pause the host
may choose (request pacing: a tile is as many vectors as the workgroup has
lanes, and a workgroup may pause after each trip). Neither changes which
operands are added in which order, so every combination must give the oracle's
bits: every element type, input counts on both sides of the kernels' launch
bounds, epilogues, skewed variants, in place, ragged sizes."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import assert_bitwise

pytestmark = pytest.mark.gpu
DEV = "cuda"

KNOBS = (hfr.HFR_TUNE_BULK_GRID, hfr.HFR_TUNE_BULK_MIN_BYTES, hfr.HFR_TUNE_BULK_SKEW, hfr.HFR_TUNE_PLACEMENT_ONLINE,
         hfr.HFR_TUNE_BULK_BLOCK, hfr.HFR_TUNE_BULK_PACE, hfr.HFR_TUNE_SEGMENT_MIB, hfr.HFR_TUNE_WIDE_WGS_PER_CU,
         hfr.HFR_TUNE_UNROLL, hfr.HFR_TUNE_GRID_CAP, hfr.HFR_TUNE_BUCKET_LIST)


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


@pytest.mark.parametrize("skew", [0, 3, 2])
@pytest.mark.parametrize("grid,block", [(3, 64), (7, 0), (256, 256)])
@pytest.mark.parametrize("K", [8, 16])
@pytest.mark.parametrize("kind", ["bf16", "f32", "f16", "e4m3", "e5m2"])
def test_chunks_that_lie_apart_run_as_bulk_launches_over_a_list(kind, K, grid, block, skew):
    """hfr_reduce_buckets with every aligned chunk sent to the list kernel (the
    knob forces it whatever the size): more chunks than one kernel-argument
    table holds, ragged sizes down to less than a vector, an element-shifted
    chunk in between (not listable), an empty one, one summed in place. Every
    chunk lies 64 bytes from the next, so nothing is merged. The list kernels
    exist plain and with skew pattern 3 (a forced pattern 2 runs plain)."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, skew)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, grid)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_BLOCK, block)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_LIST, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
    try:
        v = VEC[kind]
        sizes = [64 * v * (grid * 5 + 2) + 3, 5, 0, 256 * v * 9, 1, 100 * v + 7, 64 * v * grid * 40 + 11] + [64 * v * 3 + j for j in range(40)]
        gap = 64 // (16 // v)                                   # 64 bytes in elements
        shifted = 4                                             # bucket 4 starts one element off 16-byte alignment
        offs, off = [], 0
        for i, sz in enumerate(sizes):
            if i == shifted:
                off += 1
            offs.append(off)
            off = (off + sz + gap + v - 1) // v * v             # the next chunk is 16-byte aligned again
        total = off + v
        ins, hdt, odt = _peers(kind, K, total, 2700 + K)
        host = [synth.as_numpy_bits(t).copy() for t in ins]
        out = torch.zeros_like(ins[0])
        buckets, want = [], []
        for i, (o, sz) in enumerate(zip(offs, sizes)):
            dst = ins[2][o:o + sz] if i == 3 else out[o:o + sz]  # bucket 3 in place on input 2
            buckets.append(([t[o:o + sz] for t in ins], dst, sz))
            want.append(oracle.reduce_sum([h[o:o + sz] for h in host], odt))
        hfr.hfr_reduce_buckets(buckets, len(buckets), K, hdt, 1 << 30, 4)
        torch.cuda.synchronize()
        for i, (b, w) in enumerate(zip(buckets, want)):
            assert_bitwise(synth.as_numpy_bits(b[1]), w, "list %s K=%d skew %d chunk %d (n=%d)" % (kind, K, skew, i, sizes[i]), **_fmt(kind))
        o_bits = synth.as_numpy_bits(out)
        covered = np.zeros(total, dtype=bool)
        for i, (o, sz) in enumerate(zip(offs, sizes)):
            if i != 3:
                covered[o:o + sz] = True
        assert not o_bits[~covered].any(), "bytes between the chunks were written"
    finally:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_LIST, 0)


@pytest.mark.parametrize("kind,K,mib_per_chunk,count", [("bf16", 8, 12, 5), ("f32", 16, 6, 4), ("e4m3", 8, 11, 13)])
def test_mid_size_chunks_that_lie_apart_take_the_list_launch_by_default(kind, K, mib_per_chunk, count):
    """Library defaults: chunks of a size the rule sends to the list kernel (and
    for thirteen chunks of 11 MiB more than one launch's 128 MiB), 4 KiB apart,
    the last one ragged; with the knob off the same call must give the same
    bits by the other schedules."""
    es = {"bf16": 2, "f32": 4, "e4m3": 1}[kind]
    n = mib_per_chunk * (1 << 20) // es
    pitch = n + 4096 // es
    ins, hdt, odt = _peers(kind, K, count * pitch, 2800 + K)
    sizes = [n] * (count - 1) + [n - 12345]
    want = [oracle.reduce_sum([synth.as_numpy_bits(t[c * pitch: c * pitch + sz]) for t in ins], odt) for c, sz in enumerate(sizes)]
    for knob in (0, -1):
        out = torch.zeros_like(ins[0])
        buckets = [([t[c * pitch: c * pitch + sz] for t in ins], out[c * pitch: c * pitch + sz], sz) for c, sz in enumerate(sizes)]
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BUCKET_LIST, knob)
        hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
        hfr.hfr_reduce_buckets(buckets, count, K, hdt, 1 << 40, 4)
        torch.cuda.synchronize()
        for c, (b, w) in enumerate(zip(buckets, want)):
            assert_bitwise(synth.as_numpy_bits(b[1]), w, "knob %d %s K=%d chunk %d" % (knob, kind, K, c), **_fmt(kind))
        o_bits = synth.as_numpy_bits(out)
        for c, sz in enumerate(sizes):
            assert not o_bits[c * pitch + sz: (c + 1) * pitch].any(), "bytes behind chunk %d were written" % c
