"""The calibration kernels (plain copy, plain read, hash arithmetic alone) do
what they say: the bandwidth and integer-rate ceilings bench.py quotes next to
the path's own kernels rest on them."""
import numpy as np
import pytest
import torch

from paper_2202_07848_amd import binding as ck

pytestmark = pytest.mark.gpu

M = (1 << 64) - 1
P1, P2 = 0x9E3779B185EBCA87, 0xC2B2AE3D27D4EB4F


def test_bw_copy_copies_and_bw_read_reads_every_byte():
    n = (8 << 20) + 4096
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")
    ck.bw_copy(dst, src, n)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and int(dst[n:].sum()) == 0
    sink = torch.zeros(4096, dtype=torch.int64, device="cuda")
    ck.bw_read(src, n, sink)
    torch.cuda.synchronize()
    words = src.cpu().numpy().view(np.uint64)
    want = np.bitwise_xor.reduce(words[0::2]) ^ np.bitwise_xor.reduce(words[1::2])
    got = np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint64))
    # the kernel folds the four 32-bit columns of every 16-byte unit into one 64-bit word
    w32 = src.cpu().numpy().view(np.uint32).reshape(-1, 4)
    fold = (np.bitwise_xor.reduce(w32[:, 0] ^ w32[:, 2]).astype(np.uint64) << np.uint64(32)) | \
        np.bitwise_xor.reduce(w32[:, 1] ^ w32[:, 3]).astype(np.uint64)
    assert got == fold
    src[12345] ^= 1                        # one flipped bit must show
    ck.bw_read(src, n, sink)
    torch.cuda.synchronize()
    assert np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint64)) != got
    del want


def test_alu_probe_runs_the_xxh64_accumulator_step():
    sink = torch.zeros(4096, dtype=torch.int64, device="cuda")
    rounds = 8
    stood_for = ck.alu_xxh64(rounds, sink)
    torch.cuda.synchronize()
    groups = stood_for // (8 * rounds * 256)
    assert groups * 8 * rounds * 256 == stood_for and 0 < groups <= 4096
    got = sink.cpu().numpy().view(np.uint64)

    def rotl(x, r):
        return ((x << r) | (x >> (64 - r))) & M

    init = [(P1 + P2) & M, P2, 0, (-P1) & M]
    for block in (0, 1, groups - 1):
        x = 0
        for tid in range(256):
            acc = (init[tid & 3] + block) & M
            w = block * 256 + tid
            for _ in range(rounds):
                acc = (rotl((acc + w * P2) & M, 31) * P1) & M
                w = (w + 0x9E3779B97F4A7C15) & M
            x ^= acc
        assert int(got[block]) == x, block
    assert ck.alu_xxh64(9, sink) == 8 * 16 * 256 * groups      # rounded up to a multiple of 8
    with pytest.raises(ck.CkptError):
        ck.alu_xxh64(8, None)
    torch.cuda.synchronize()


@pytest.mark.parametrize("tile", [256, 1024])
@pytest.mark.parametrize("nstreams,stream_bytes", [(16, 2048), (48, 4096), (32, 1 << 20)])
def test_bw_streams_copies_every_stream_and_nothing_else(nstreams, stream_bytes, tile):
    n = nstreams * stream_bytes
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.full((n + 4096,), 0x6B, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4096, dtype=torch.int64, device="cuda")
    ck.bw_streams(dst, src, nstreams, stream_bytes, sink, tile_bytes=tile)
    torch.cuda.synchronize()
    assert torch.equal(dst[:n], src) and bool((dst[n:] == 0x6B).all())
    ck.bw_streams(None, src, nstreams, stream_bytes, sink, tile_bytes=tile)        # read only
    torch.cuda.synchronize()
    for bad in ((15, stream_bytes), (nstreams, stream_bytes + tile), (nstreams, 0)):
        with pytest.raises(ck.CkptError) as e:
            ck.bw_streams(dst, src, bad[0], bad[1], sink, tile_bytes=tile)
        assert e.value.status == -1
    if tile == 256:
        ck.bw_streams(dst[:16 * 512], src, 16, 512, sink)            # the smallest stream: two tiles
        torch.cuda.synchronize()
        assert torch.equal(dst[:16 * 512], src[:16 * 512])
    with pytest.raises(ck.CkptError) as e:
        ck.bw_streams(dst, src, nstreams, stream_bytes, sink, tile_bytes=512)
    assert e.value.status == -1
