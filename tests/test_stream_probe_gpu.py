"""The calibration kernel behind bench.py --calibrate-stream (include/kvev_test_hooks.h): every access form (plain,
non-temporal, writes held back and issued in chip-wide bursts) leaves the same bytes, and those are the per-lane
sums of the tile it read.  It exists to measure the memory system, so a wrong index would falsify the ceilings that
the pooling and attention kernels are read against."""
import pytest
import torch

from paper_2509_21354_amd import binding as kb

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tiles,tile_bytes,write_bytes", [
    (3001, 32768, 4096),        # more tiles than persistent workgroups, not a multiple of their number
    (7, 32768, 8192),           # fewer tiles than compute units
    (1025, 65536, 16),          # one 16-byte word per tile
])
def test_every_access_form_writes_the_same_bytes(tiles, tile_bytes, write_bytes):
    g = torch.Generator(device="cuda").manual_seed(5)
    src = torch.randint(0, 2 ** 31 - 1, (tiles * tile_bytes // 4,), dtype=torch.int32, device="cuda", generator=g)
    outs = []
    for hints in (0, 1, 2, 3, 4, 7):
        dst = torch.full((tiles * write_bytes // 4 + 4,), -1, dtype=torch.int32, device="cuda")
        kb.kvev_debug_stream_probe(src, tile_bytes, dst, write_bytes, hints)
        torch.cuda.synchronize()
        assert (dst[tiles * write_bytes // 4:] == -1).all()          # nothing past the last tile's slot
        outs.append(dst[:tiles * write_bytes // 4].clone())
    for o in outs[1:]:
        assert torch.equal(o, outs[0])
    # lane t of a tile sums the 16-byte words t, t + 256, ... of the tile (mod 2^32 per component) and writes the sum to
    # words t, t + 256, ... of the tile's slot
    words = src.view(tiles, tile_bytes // 16, 4).to(torch.int64)
    lane_sum = words.view(tiles, tile_bytes // 16 // 256, 256, 4).sum(1) % (1 << 32)
    w16 = write_bytes // 16
    want = lane_sum[:, torch.arange(w16, device="cuda") % 256, :]
    got = outs[0].view(tiles, w16, 4).to(torch.int64) % (1 << 32)
    assert torch.equal(got, want)


def test_probe_without_writes_leaves_the_destination_alone():
    src = torch.ones(8 * 32768 // 4, dtype=torch.int32, device="cuda")
    dst = torch.full((16,), 7, dtype=torch.int32, device="cuda")
    for hints in (0, 1, 7):
        kb.kvev_debug_stream_probe(src, 32768, dst, 0, hints)
    torch.cuda.synchronize()
    assert (dst == 7).all()
