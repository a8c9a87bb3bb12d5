"""The entry point that allocates nothing (hfr_reduce_chunks_noalloc) against
the entry point it is a variant of (hfr_reduce_chunk_table, table in a device
buffer of the caller's) and against the oracle, bit for bit, on two calls in a
row - the second with a smaller input, so that stale entries of the first call
sit behind the second call's table."""
import numpy as np
import pytest
import torch

import oracle
from paper_2408_14158_amd import hfr, synth
from tests.parity_util import assert_bitwise

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _chunks(flats, out, sizes, pad):
    lst, off = [], 0
    for i, sz in enumerate(sizes):
        sh = (0, 1, 0, 3)[i % 4]                    # mixed alignment classes
        lst.append(([f[off + sh: off + sh + sz] for f in flats], out[off + sh: off + sh + sz], sz))
        off += sz + pad
    return lst


@pytest.mark.parametrize("K,dtype", [(8, torch.bfloat16), (3, torch.float32), (16, torch.float8_e4m3fn)])
def test_noalloc_matches_the_chunk_table_entry_point_twice_in_a_row(K, dtype):
    hdt, odt = {torch.bfloat16: (hfr.HFR_BF16, oracle.BF16), torch.float32: (hfr.HFR_F32, oracle.F32),
                torch.float8_e4m3fn: (hfr.HFR_FP8_E4M3, oracle.FP8_E4M3)}[dtype]
    fp8 = "e4m3" if dtype == torch.float8_e4m3fn else ""
    rng = np.random.default_rng(70 + K)
    first = [int(x) for x in rng.integers(1, 30000, size=300)] + [0, 1, 7, 70001, (2 << 20) + 5]
    second = [int(x) for x in rng.integers(1, 9000, size=40)] + [0, 3]       # fewer and shorter chunks
    pad = 16
    s = torch.cuda.Stream()
    for call, sizes in enumerate((first, second)):
        total = sum(sz + pad for sz in sizes)
        if dtype == torch.float32:
            flats = synth.peer_buffers_uniform_f32(K, total, 7100 + call, DEV)
        elif dtype == torch.bfloat16:
            flats = synth.peer_buffers_normal_bf16(K, total, 1.0, 7100 + call, DEV)
        else:
            flats = synth.peer_buffers_normal_fp8(K, total, 1.0, 7100 + call, "e4m3", DEV)
        out_a = torch.zeros(total, dtype=torch.uint8 if fp8 else dtype, device=DEV).view(dtype) if fp8 else \
            torch.zeros(total, dtype=dtype, device=DEV)
        out_b = torch.zeros_like(out_a)
        hint = 8192
        # existing entry point: the table in a device buffer the caller allocated
        ch_b = _chunks(flats, out_b, sizes, pad)
        table = hfr.make_chunk_table(ch_b, DEV)
        torch.cuda.synchronize()
        hfr.hfr_reduce_chunk_table(table, len(ch_b), hint, K, hdt, s)
        # the new one: host chunk list, static device table
        ch_a = _chunks(flats, out_a, sizes, pad)
        host = hfr.make_host_chunk_array(ch_a)
        hfr.hfr_reduce_chunks_noalloc(host, len(ch_a), hint, K, hdt, s)
        del host                                     # read during the call only
        s.synchronize()
        assert torch.equal(out_a.view(torch.uint8), out_b.view(torch.uint8)), "call %d differs from hfr_reduce_chunk_table" % call
        for i, (ins, o, sz) in enumerate(ch_a):
            if sz == 0:
                continue
            want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], odt)
            assert_bitwise(synth.as_numpy_bits(o), want, "call %d chunk %d (n=%d)" % (call, i, sz), fp8=fp8)


def test_noalloc_limits_and_argument_errors():
    K, per = 2, 8
    n = hfr.HFR_NOALLOC_MAX_CHUNKS * per
    ins = synth.peer_buffers_uniform_f32(K, n, 7200, DEV)
    out = torch.zeros(n, dtype=torch.float32, device=DEV)
    tiny = [([t[c * per:(c + 1) * per] for t in ins], out[c * per:(c + 1) * per], per)
            for c in range(hfr.HFR_NOALLOC_MAX_CHUNKS)]
    host = hfr.make_host_chunk_array(tiny + tiny[:1])
    st = hfr.hfr_reduce_chunks_noalloc(host, hfr.HFR_NOALLOC_MAX_CHUNKS + 1, per, K, hfr.HFR_F32, check=False)
    assert st == hfr.HFR_ERR_INVALID_ARG and str(hfr.HFR_NOALLOC_MAX_CHUNKS) in hfr.hfr_last_error()
    torch.cuda.synchronize()
    assert not out.any(), "a rejected call enqueues nothing"
    # exactly the maximum is accepted
    st = hfr.hfr_reduce_chunks_noalloc(host, hfr.HFR_NOALLOC_MAX_CHUNKS, per, K, hfr.HFR_F32, check=False)
    torch.cuda.synchronize()
    assert st == hfr.HFR_OK
    want = oracle.reduce_sum([synth.as_numpy_bits(t) for t in ins], oracle.F32)
    assert_bitwise(synth.as_numpy_bits(out), want, "max table")
    n = 1000
    bad = hfr.make_host_chunk_array([([t[:n] for t in ins], out[:n], n), ([t[n:2 * n] for t in ins], out[n:2 * n], n)])
    bad[1, 1] += 2                                   # a misaligned input in the second chunk
    assert hfr.hfr_reduce_chunks_noalloc(bad, 2, n, K, hfr.HFR_F32, check=False) == hfr.HFR_ERR_MISALIGNED
    assert hfr.hfr_reduce_chunks_noalloc(None, 0, n, K, hfr.HFR_F32, check=False) == hfr.HFR_OK
    assert hfr.hfr_reduce_chunks_noalloc(None, 1, n, K, hfr.HFR_F32, check=False) == hfr.HFR_ERR_INVALID_ARG
    assert hfr.hfr_reduce_chunks_noalloc(host, 1, 0, K, hfr.HFR_F32, check=False) == hfr.HFR_ERR_INVALID_ARG
    assert hfr.hfr_reduce_chunks_noalloc(host, 1, n, 17, hfr.HFR_F32, check=False) == hfr.HFR_ERR_INVALID_ARG
    assert hfr.hfr_reduce_chunks_noalloc(host, 1, n, K, 9, check=False) == hfr.HFR_ERR_UNSUPPORTED_DTYPE
