"""The streaming-read probe (a measurement aid) runs, reads inside its buffer and writes nothing."""
import pytest
import torch

from paper_2602_09323_amd import probe

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes,wgs", [(16, 1), (4096 * 16 + 48, 1), (1 << 24, 64), ((1 << 24) + 16 * 12345, 2048)])
def test_probe_reads_and_leaves_memory_alone(nbytes, wgs):
    # guard words on both sides of the buffer and of the sink stay as they were
    whole = torch.zeros(nbytes + 512, dtype=torch.uint8, device="cuda")
    whole[:256] = 0x5A
    whole[-256:] = 0x5A
    sink = torch.full((8,), 77, dtype=torch.int32, device="cuda")
    probe.stream_read_probe(whole[256:-256], wgs, sink[4:5])
    torch.cuda.synchronize()
    assert bool((whole[:256] == 0x5A).all()) and bool((whole[-256:] == 0x5A).all())
    assert bool((whole[256:-256] == 0).all())
    assert sink.tolist() == [77] * 8          # zeros never XOR to the constant: no write at all
