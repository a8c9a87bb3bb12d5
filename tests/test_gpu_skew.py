"""GPU parity of the skewed bulk kernels (some input streams run a few trips
ahead of the trip being summed) and of placement tuning: every pattern must
give the oracle's bits, for every element type, epilogue and burst layout."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import assert_bitwise, gpu_reduce_sum, oracle_reduce_sum

pytestmark = pytest.mark.gpu
DEV = "cuda"

KNOBS = (hfr.HFR_TUNE_GRID_CAP, hfr.HFR_TUNE_UNROLL, hfr.HFR_TUNE_BULK_GRID, hfr.HFR_TUNE_BULK_MIN_BYTES,
         hfr.HFR_TUNE_BULK_SKEW, hfr.HFR_TUNE_PLACEMENT_ONLINE)


@pytest.fixture(autouse=True)
def _default_tuning():
    yield
    for knob in KNOBS:
        hfr.hfr_set_tuning(knob, 0)
    hfr.hfr_shutdown()                      # also empties the placement table


def _force(skew, grid):
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)    # bulk shape whatever the size
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, grid)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, skew)


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


def _vec_elems(kind):
    return {"f32": 4, "bf16": 8, "f16": 8, "e4m3": 16, "e5m2": 16}[kind]


@pytest.mark.parametrize("skew", [1, 2, 3])
@pytest.mark.parametrize("K", [8, 9])
@pytest.mark.parametrize("kind", ["bf16", "f32", "f16", "e4m3", "e5m2"])
def test_every_skew_pattern_gives_the_oracles_sum(kind, K, skew):
    """Three workgroups, 45 trips each (bursts of 23 and 22 trips), a last
    workgroup one trip short, a partial tile and a scalar tail."""
    _force(skew, 3)
    n = 256 * _vec_elems(kind) * (3 * 45 - 1) + 256 * _vec_elems(kind) // 2 + 3
    ins, hdt, odt = _peers(kind, K, n, 900 + K)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    assert_bitwise(synth.as_numpy_bits(out), want, "skew %d %s K=%d" % (skew, kind, K),
                   f16=(kind == "f16"), fp8=(kind if kind in ("e4m3", "e5m2") else ""))


OTHER_K = [5, 6, 7, 10, 11, 12, 13, 14, 15, 16]


@pytest.mark.parametrize("K", OTHER_K)
@pytest.mark.parametrize("kind", ["bf16", "f32", "f16", "e4m3", "e5m2"])
def test_pattern_three_for_the_other_input_counts(kind, K):
    """Input counts other than eight and nine have pattern 3 for the plain sum
    (streams lead by 3 - (j mod 4) trips): four workgroups of the size the
    library picks for this type and K, some forty trips each, a partial tile and
    a scalar tail; then the same in place on the last input."""
    _force(3, 4)
    n = 256 * _vec_elems(kind) * (4 * 41 - 1) + 128 * _vec_elems(kind) + 7
    ins, hdt, odt = _peers(kind, K, n, 2000 + K)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    f16, fp8 = kind == "f16", kind if kind in ("e4m3", "e5m2") else ""
    assert_bitwise(synth.as_numpy_bits(out), want, "pattern 3 %s K=%d" % (kind, K), f16=f16, fp8=fp8)
    hfr.hfr_reduce_sum(ins, K, ins[K - 1], n, hdt)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(ins[K - 1]), want, "pattern 3 in place %s K=%d" % (kind, K), f16=f16, fp8=fp8)


@pytest.mark.parametrize("K", [5, 7, 12, 16])
@pytest.mark.parametrize("grid,trips", [(1, 1), (1, 2), (1, 3), (1, 4), (2, 5), (256, 1), (5, 70)])
def test_pattern_three_with_few_trips_and_many_bursts(K, grid, trips):
    """Fewer trips than the longest lead, one trip per workgroup, several full
    bursts, with 64-lane workgroups so that the trip counts are exact."""
    _force(3, grid)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_BLOCK, 64)
    try:
        n = 64 * 8 * (grid * trips) + 11
        ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 2100 + K, DEV)
        out = torch.empty_like(ins[0])
        hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "K=%d grid %d trips %d" % (K, grid, trips))
    finally:
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_BLOCK, 0)


@pytest.mark.parametrize("skew", [1, 2, 3])
@pytest.mark.parametrize("grid,trips", [(1, 1), (1, 2), (1, 3), (1, 4), (2, 5), (7, 33), (256, 1), (5, 70)])
def test_skew_with_few_trips_and_many_bursts(skew, grid, trips):
    """Fewer trips than the longest lead (the early loads run past the end),
    one trip per workgroup, several full bursts."""
    _force(skew, grid)
    K = 8
    n = 256 * 8 * (grid * trips) + 11
    ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 950, DEV)
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "skew %d grid %d trips %d" % (skew, grid, trips))


@pytest.mark.parametrize("skew", [1, 2, 3])
def test_skewed_fused_average_and_fused_combine(skew):
    _force(skew, 4)
    K, n = 8, 256 * 8 * (4 * 37) + 1234
    ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 960, DEV)
    remote = synth.normal_bf16(n, 1e-3, 969, DEV)
    host = [synth.as_numpy_bits(t) for t in ins]
    out = torch.empty_like(ins[0])
    hfr.hfr_reduce_avg(ins, K, out, n, 0.1, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, 0.1, oracle.BF16), "skewed average")
    # K peers + the remote partial ride as nine inputs of one launch
    hfr.hfr_reduce_combine_avg(ins, K, remote, out, n, 1.0 / 128, hfr.HFR_BF16)
    torch.cuda.synchronize()
    partial = oracle.reduce_sum(host, oracle.BF16)
    want = oracle.combine_avg(partial, synth.as_numpy_bits(remote), 1.0 / 128, oracle.BF16)
    assert_bitwise(synth.as_numpy_bits(out), want, "skewed fused combine")


@pytest.mark.parametrize("skew", [1, 2, 3])
@pytest.mark.parametrize("alias", [0, 3, 7])
def test_skewed_in_place(skew, alias):
    """out == in[alias]: a stream that runs ahead reads tiles of the output
    buffer before they are written, never after."""
    _force(skew, 3)
    K, n = 8, 256 * 8 * (3 * 40) + 77
    ins = synth.peer_buffers_uniform_f32(K, n, 970, DEV)
    want = oracle_reduce_sum(ins)
    hfr.hfr_reduce_sum(ins, K, ins[alias], n, hfr.HFR_F32)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(ins[alias]), want, "skew %d in place on %d" % (skew, alias))


def test_skew_knob_is_ignored_where_no_variant_exists():
    """Patterns 1 and 2 exist for eight and nine inputs only, pattern 3 for the
    other input counts only with the plain sum, and nothing below five inputs:
    a forced pattern that a launch does not have leaves it the plain kernel."""
    for skew in (1, 2):
        _force(skew, 3)
        for K in (3, 5, 7, 10, 16):
            n = 256 * 8 * 90 + 5
            ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 980 + K, DEV)
            out = gpu_reduce_sum(ins)
            torch.cuda.synchronize()
            assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "pattern %d K=%d" % (skew, K))
    _force(3, 3)
    for K in (4, 6, 13):
        n = 256 * 8 * 90 + 5
        ins = synth.peer_buffers_normal_bf16(K + 1, n, 1e-3, 985 + K, DEV)
        peers, remote = ins[:K], ins[K]
        host = [synth.as_numpy_bits(t) for t in peers]
        out = torch.empty_like(peers[0])
        hfr.hfr_reduce_avg(peers, K, out, n, 0.25, hfr.HFR_BF16)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), oracle.reduce_avg(host, 0.25, oracle.BF16), "average K=%d" % K)
        hfr.hfr_reduce_combine_avg(peers, K, remote, out, n, 0.5, hfr.HFR_BF16)
        torch.cuda.synchronize()
        want = oracle.combine_avg(oracle.reduce_sum(host, oracle.BF16), synth.as_numpy_bits(remote), 0.5, oracle.BF16)
        assert_bitwise(synth.as_numpy_bits(out), want, "fused combine K=%d" % K)
    _force(2, 3)
    # element-aligned views: wide shape, no skew
    K, n = 8, 256 * 8 * 90 + 5
    base = synth.peer_buffers_normal_bf16(K, n + 1, 1e-3, 990, DEV)
    views = [t[1:] for t in base]
    out = torch.empty(n + 1, dtype=torch.bfloat16, device=DEV)[1:]
    hfr.hfr_reduce_sum(views, K, out, n, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(views), "unaligned")


def test_tune_placement_records_a_pattern_and_keeps_the_bits():
    """32 MiB per buffer takes the bulk shape by default. Whatever pattern wins
    on this machine, `out` holds the oracle's sum, later calls on the same buffers
    and on chunks of them give the same bits, and shutdown forgets the choice."""
    K, n = 8, 1 << 24
    ins = synth.peer_buffers_normal_bf16(K, n, 1e-3, 1000, DEV)
    out = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    want = oracle_reduce_sum(ins)
    st, chosen = hfr.hfr_tune_placement(ins, K, out, n, hfr.HFR_BF16)
    assert st == hfr.HFR_OK and 0 <= chosen <= 3
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "tuning run")
    out.zero_()
    hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "after tuning")
    # chunks of the same buffers share the placement key
    out.zero_()
    hfr.hfr_reduce_buckets([(ins, out, n)], 1, K, hfr.HFR_BF16, 12 << 20, 2)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "chunks after tuning")
    # every pattern forced on the tuned buffers: still the same bits
    for skew in (-1, 1, 2, 3):
        hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, skew)
        out.zero_()
        hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16)
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), want, "forced %d" % skew)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_SKEW, 0)
    assert hfr.hfr_shutdown() == hfr.HFR_OK
    out.zero_()
    hfr.hfr_reduce_sum(ins, K, out, n, hfr.HFR_BF16)
    torch.cuda.synchronize()
    assert_bitwise(synth.as_numpy_bits(out), want, "after shutdown")


def _page_spaced(tensors, extra=1):
    """Copies of the tensors (plus `extra` spare buffers) carved from one
    allocation at a spacing that is a multiple of 4 KiB: the placement table
    keys on distances in 4 KiB units, and small torch allocations are only
    512-byte aligned."""
    t0 = tensors[0]
    nbytes = t0.numel() * t0.element_size()
    pitch = (nbytes + 4095) // 4096 * 4096 // t0.element_size()
    slab = torch.zeros(pitch * (len(tensors) + extra) * t0.element_size(), dtype=torch.uint8, device=DEV).view(t0.dtype)
    views = [slab[j * pitch: j * pitch + t0.numel()] for j in range(len(tensors) + extra)]
    for v, t in zip(views, tensors):
        v.copy_(t)
    return views[:len(tensors)], views[len(tensors):]


@pytest.mark.parametrize("kind,K", [("bf16", 8), ("f32", 9), ("e4m3", 8), ("f16", 12), ("bf16", 5), ("e5m2", 16)])
def test_placement_is_measured_on_the_fly_without_blocking(kind, K):
    """An unseen placement: the first bulk launches are the trials (three per
    variant that exists for K inputs: the plain kernel and the three skewed ones
    for eight and nine inputs, the plain kernel and pattern 3 otherwise; same
    bits), a launch after they have finished records a pattern, and every result
    on the way is the oracle's. In place (out = an input) is a placement of its
    own. With the knob off nothing is measured."""
    patterns = (0, 1, 2, 3) if K in (8, 9) else (0, 3)
    trials = 3 * len(patterns)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)        # bulk shape whatever the size
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 7)
    n = 256 * _vec_elems(kind) * (7 * 40 - 2) + 5
    ins, hdt, odt = _peers(kind, K, n, 1200 + K)
    ins, (out,) = _page_spaced(ins)
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    f16, fp8 = kind == "f16", kind if kind in ("e4m3", "e5m2") else ""
    assert hfr.hfr_placement_query(ins, K, out, hdt) == (hfr.HFR_OK, 0, 0)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, -1)
    hfr.hfr_reduce_sum(ins, K, out, n, hdt)
    assert hfr.hfr_placement_query(ins, K, out, hdt)[1] == 0   # knob off: the table stays empty
    hfr.hfr_set_tuning(hfr.HFR_TUNE_PLACEMENT_ONLINE, 0)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    for it in range(trials):
        out.zero_()
        torch.cuda.synchronize()
        hfr.hfr_reduce_sum(ins, K, out, n, hdt, s)
        assert hfr.hfr_placement_query(ins, K, out, hdt)[1] == 1, "launch %d is a trial" % it
        s.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), want, "trial %d" % it, f16=f16, fp8=fp8)
    # every trial has finished: the next launch concludes the measurement
    hfr.hfr_reduce_sum(ins, K, out, n, hdt, s)
    st, state, pattern = hfr.hfr_placement_query(ins, K, out, hdt)
    assert (st, state) == (hfr.HFR_OK, 2) and pattern in patterns
    for it in range(3):
        out.zero_()
        torch.cuda.synchronize()                 # the fill ran on the default stream
        hfr.hfr_reduce_sum(ins, K, out, n, hdt, s)
        s.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), want, "recorded pattern %d" % pattern, f16=f16, fp8=fp8)
    # in place on input 2: another placement, measured on its own, still the oracle's bits
    saved = ins[2].clone()
    for it in range(trials + 2):
        ins[2].copy_(saved)
        torch.cuda.synchronize()                 # the copy ran on the default stream
        hfr.hfr_reduce_sum(ins, K, ins[2], n, hdt, s)
        s.synchronize()
        assert_bitwise(synth.as_numpy_bits(ins[2]), want, "in place %d" % it, f16=f16, fp8=fp8)
    assert hfr.hfr_placement_query(ins, K, ins[2], hdt)[1] == 2
    ins[2].copy_(saved)
    torch.cuda.synchronize()
    # the explicit form overrides what was measured
    st, chosen = hfr.hfr_tune_placement(ins, K, out, n, hdt, s)
    assert chosen in patterns
    assert hfr.hfr_placement_query(ins, K, out, hdt) == (hfr.HFR_OK, 2, chosen)
    hfr.hfr_shutdown()
    assert hfr.hfr_placement_query(ins, K, out, hdt) == (hfr.HFR_OK, 0, 0)


def test_no_placement_trials_under_graph_capture():
    """Launches on a capturing stream take no trials (their events would be
    replayed with the graph): the table keeps saying "being measured" with
    nothing issued, and every replay gives the oracle's bits."""
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_MIN_BYTES, 1)
    hfr.hfr_set_tuning(hfr.HFR_TUNE_BULK_GRID, 5)
    K, n = 8, 256 * 8 * (5 * 35) + 123
    ins, hdt, odt = _peers("bf16", K, n, 1300)
    ins, (out,) = _page_spaced(ins)
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        for _ in range(3):
            hfr.hfr_reduce_sum(ins, K, out, n, hdt, s)
    for rep in range(3):
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert_bitwise(synth.as_numpy_bits(out), want, "replay %d" % rep)
    del g
    # eager launches afterwards run their twelve trials as usual
    for it in range(13):
        hfr.hfr_reduce_sum(ins, K, out, n, hdt, s)
        s.synchronize()
    assert hfr.hfr_placement_query(ins, K, out, hdt)[1] == 2
    assert_bitwise(synth.as_numpy_bits(out), want, "after the trials")


@pytest.mark.parametrize("kind,K,size_mib,spare_mib", [("bf16", 8, 24, 16), ("f32", 5, 32, 0), ("e4m3", 16, 20, 6)])
def test_tune_peer_stride_returns_a_candidate_and_the_sum_there_is_the_oracles(kind, K, size_mib, spare_mib):
    """The measured stride is one of the candidates that fit the arena (with no
    spare room: none above the rule's value), at least the buffer size, a
    multiple of 2 MiB; buffers carved at it sum to the oracle's bits."""
    mib = 1 << 20
    es = {"bf16": 2, "f32": 4, "e4m3": 1}[kind]
    n = size_mib * mib // es - 3
    nbytes = n * es
    rule = hfr.hfr_peer_stride(nbytes)
    arena_bytes = K * (rule + spare_mib * mib) + nbytes
    ins, hdt, odt = _peers(kind, K, n, 2500 + K)
    arena = torch.zeros(arena_bytes, dtype=torch.uint8, device=DEV)
    st, stride = hfr.hfr_tune_peer_stride(arena, arena_bytes, K, n, hdt)
    torch.cuda.synchronize()
    assert st == hfr.HFR_OK
    up2 = (nbytes + 2 * mib - 1) // (2 * mib) * (2 * mib)
    assert stride in [rule] + [up2 + d * 2 * mib for d in range(8)]
    assert stride >= nbytes and K * stride + nbytes <= arena_bytes
    views = [arena[j * stride: j * stride + nbytes].view(ins[0].dtype) for j in range(K + 1)]
    for v, t in zip(views, ins):
        v.copy_(t)
    torch.cuda.synchronize()
    hfr.hfr_reduce_sum(views[:K], K, views[K], n, hdt)
    torch.cuda.synchronize()
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
    assert_bitwise(synth.as_numpy_bits(views[K]), want, "sum at the measured stride %s K=%d" % (kind, K),
                   f16=False, fp8=(kind if kind in ("e4m3", "e5m2") else ""))
    for v, t in zip(views, ins):                       # the inputs were only read
        assert torch.equal(v.view(torch.uint8), t.view(torch.uint8))


def test_tune_placement_small_or_unsupported_inputs_are_summed_once():
    for K, n in ((8, 100003), (4, 1 << 22), (1, 5)):
        ins = synth.peer_buffers_uniform_f32(K, n, 1010 + K, DEV)
        out = torch.zeros(n, dtype=torch.float32, device=DEV)
        st, chosen = hfr.hfr_tune_placement(ins, K, out, n, hfr.HFR_F32)
        torch.cuda.synchronize()
        assert st == hfr.HFR_OK and chosen == 0
        assert_bitwise(synth.as_numpy_bits(out), oracle_reduce_sum(ins), "K=%d n=%d" % (K, n))
    # empty input: nothing to do
    st, chosen = hfr.hfr_tune_placement(ins, 1, out, 0, hfr.HFR_F32)
    assert st == hfr.HFR_OK and chosen == 0


def test_tune_placement_rejects_an_output_that_is_an_input():
    K, n = 8, 4096
    ins = synth.peer_buffers_uniform_f32(K, n, 1020, DEV)
    st, _ = hfr.hfr_tune_placement(ins, K, ins[2], n, hfr.HFR_F32, check=False)
    assert st == hfr.HFR_ERR_INVALID_ARG


def test_entry_points_from_several_host_threads_at_once():
    """Four host threads, a stream each, call the sum, the bucket scheduler
    (whose worker ring is shared: calls take turns), placement tuning and the
    knobs at the same time; every result must still be the oracle's."""
    import threading
    K, n_small, n_big = 8, 300007, 1 << 24
    work = []
    for t in range(4):
        small = synth.peer_buffers_normal_bf16(K, n_small, 1e-3, 1100 + 10 * t, DEV)
        big = synth.peer_buffers_normal_bf16(K, n_big, 1e-3, 1150 + 10 * t, DEV) if t < 2 else None
        work.append({"small": small, "big": big, "stream": torch.cuda.Stream(),
                     "want_small": oracle_reduce_sum(small), "want_big": oracle_reduce_sum(big) if big else None,
                     "outs": [], "error": None})
    torch.cuda.synchronize()

    def body(w, t):
        try:
            s = w["stream"]
            torch.cuda.set_stream(s)        # this thread's fills run on its stream too, ahead of the library's launches
            for it in range(12):
                out = torch.zeros(n_small, dtype=torch.bfloat16, device=DEV)
                if it % 3 == 0:
                    hfr.hfr_reduce_sum(w["small"], K, out, n_small, hfr.HFR_BF16, s)
                elif it % 3 == 1:
                    hfr.hfr_reduce_buckets([(w["small"], out, n_small)], 1, K, hfr.HFR_BF16, 20000, 4, s)
                else:
                    cuts = synth.bucket_cuts(n_small, 8 * 5000)
                    hfr.hfr_reduce_buckets_batched([([x[o:o + l] for x in w["small"]], out[o:o + l], l) for o, l in cuts],
                                                   len(cuts), K, hfr.HFR_BF16, s)
                w["outs"].append(("small", out))
                if t == 3:
                    hfr.hfr_set_tuning(hfr.HFR_TUNE_UNROLL, (0, 1, 2, 4)[it % 4])   # knobs never change results
                if w["big"] is not None and it % 4 == 0:
                    big_out = torch.zeros(n_big, dtype=torch.bfloat16, device=DEV)
                    st, chosen = hfr.hfr_tune_placement(w["big"], K, big_out, n_big, hfr.HFR_BF16, s)
                    assert st == hfr.HFR_OK and 0 <= chosen <= 3
                    again = torch.zeros(n_big, dtype=torch.bfloat16, device=DEV)
                    hfr.hfr_reduce_sum(w["big"], K, again, n_big, hfr.HFR_BF16, s)
                    w["outs"].append(("big", big_out))
                    w["outs"].append(("big", again))
            s.synchronize()
        except Exception as exc:            # reported by the main thread
            w["error"] = exc

    threads = [threading.Thread(target=body, args=(w, t)) for t, w in enumerate(work)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=120)
        assert not th.is_alive(), "a worker thread did not finish"
    torch.cuda.synchronize()
    for t, w in enumerate(work):
        assert w["error"] is None, (t, w["error"])
        for i, (which, out) in enumerate(w["outs"]):
            assert_bitwise(synth.as_numpy_bits(out), w["want_" + which], "thread %d result %d (%s)" % (t, i, which))
