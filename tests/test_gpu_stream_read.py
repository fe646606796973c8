"""The streaming-read kernel behind bench.py's measured bandwidth ceiling reads every 16-byte item
of its buffer: a marker planted anywhere (inside a wave's private run, in the remainder behind the
runs, in the last item) reaches the sink, and an all-zero buffer leaves the sink alone."""
import pytest
import torch

from paper_2410_20488_amd import binding

pytestmark = pytest.mark.gpu
MAGIC = 0x9E3779B9


def _run(buf, sink):
    lib = binding.load_library()
    stream = torch.cuda.current_stream(buf.device)
    rc = lib.firp_debug_stream_read(buf.data_ptr(), buf.numel() * 4, sink.data_ptr(), stream.cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    return int(sink.cpu()[0]) & 0xFFFFFFFF


@pytest.mark.parametrize("items", [1, 5, 64 * 4 * 8192 + 0, 64 * 4 * 8192 * 3 + 12345, (1 << 24) + 77])
def test_every_item_is_read(items, progress):
    dev = torch.device("cuda:0")
    buf = torch.zeros(items * 4, dtype=torch.int32, device=dev)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    assert _run(buf, sink) == 0
    g = torch.Generator().manual_seed(items)
    where = {0, items - 1, items // 2, items // 3} | {int(x) for x in torch.randint(0, items, (6,), generator=g)}
    for w in sorted(where):
        buf.zero_()
        sink.zero_()
        buf[4 * w] = MAGIC - (1 << 32)     # as a signed 32-bit value, in the item's first word
        assert _run(buf, sink) == MAGIC, (items, w)   # the sink takes the reader's running xor
    progress(f"stream read: {items} items, {len(where)} marker positions")


def test_rate_is_reported(progress):
    gbps = binding.stream_read_gbps(nbytes=1 << 30, repeats=2)
    progress(f"stream read: {gbps:.0f} GB/s over 1 GiB")
    assert 500.0 < gbps < 8000.0
