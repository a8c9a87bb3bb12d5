"""The benchmark's streaming probes really read and write what they claim:
the output of a pass is the XOR of its read streams in every write stream, in
both launch shapes, so a measured rate is the rate of that traffic."""
import pytest
import torch

from paper_2408_14158_amd import probe

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("shape", [probe.HFR_PROBE_WIDE, probe.HFR_PROBE_BULK])
@pytest.mark.parametrize("R,W", [(0, 1), (1, 1), (2, 1), (8, 1), (16, 1), (1, 8), (8, 0), (0, 3)])
def test_probe_pass_moves_the_bytes_it_counts(R, W, shape):
    nbytes = 32768 * 37                     # ragged against the grid, a multiple of the tile
    g = torch.Generator(device=DEV)
    g.manual_seed(50 + R)
    rd = [torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g) for _ in range(R)]
    wr = [torch.full((nbytes + 64,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sink = torch.zeros(64, dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()
    probe.hfr_probe_stream(rd, [w[:nbytes] for w in wr], sink, nbytes, shape)
    torch.cuda.synchronize()
    want = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    for t in rd:
        want ^= t
    for w in wr:
        assert torch.equal(w[:nbytes], want)
        assert bool((w[nbytes:] == 0xAA).all()), "nothing is written past nbytes"
    assert not sink.any()


@pytest.mark.parametrize("lanes,pace", [(64, 0), (96, 3), (160, 0), (256, 1), (352, 0), (384, 64)])
@pytest.mark.parametrize("R,W", [(0, 1), (1, 1), (2, 1), (8, 1), (16, 1), (1, 8), (8, 0)])
def test_paced_probe_moves_the_whole_tiles_it_counts(R, W, lanes, pace):
    """The bulk shape with a run-time workgroup size and pause: every whole tile
    holds the XOR of the read streams, nothing beyond the last whole tile is
    touched."""
    nbytes = 32768 * 37
    U = 8 if max(R, W) <= 1 else (4 if max(R, W) == 2 else (2 if max(R, W) <= 4 else 1))
    tile = lanes * U * 16
    whole = nbytes // tile * tile
    g = torch.Generator(device=DEV)
    g.manual_seed(60 + R)
    rd = [torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device=DEV, generator=g) for _ in range(R)]
    wr = [torch.full((nbytes + 64,), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(W)]
    sink = torch.zeros(64, dtype=torch.uint8, device=DEV)
    torch.cuda.synchronize()
    probe.hfr_probe_stream_paced(rd, [w[:nbytes] for w in wr], sink, nbytes, lanes, pace)
    torch.cuda.synchronize()
    want = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
    for t in rd:
        want ^= t
    for w in wr:
        assert torch.equal(w[:whole], want[:whole])
        assert bool((w[whole:] == 0xAA).all()), "nothing is written past the last whole tile"
    assert not sink.any()
