"""The streaming kernel that bench.py sets beside the scan's bandwidth (rodimus_hbm_stream_probe) does what its header says:
every written unit is the constant plus the sum of the matching units of the input streams (needs an MI355X)."""
import pytest
import torch

from paper_2410_06577_amd import rodimus

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("reads", [0, 1, 2, 4])
@pytest.mark.parametrize("units,workgroups", [(1, 1), (1000, 3), (1 << 16, 256)])
def test_sums_of_the_streams(reads, units, workgroups):
    print(f"stream probe reads {reads} units {units} workgroups {workgroups}", flush=True)
    dev = "cuda:0"
    src = torch.arange(4 * max(reads, 1) * units, dtype=torch.float32, device=dev) % 1024      # exact in fp32
    dst = torch.full((4 * units + 4,), -1.0, dtype=torch.float32, device=dev)
    rodimus.rodimus_hbm_stream_probe(src, dst[:4 * units], reads, workgroups)
    torch.cuda.synchronize()
    want = torch.tensor([1.0, 2.0, 3.0, 4.0], device=dev).repeat(units)
    if reads:
        want = want + src.view(reads, -1).sum(0)
    assert torch.equal(dst[:4 * units], want) and torch.all(dst[4 * units:] == -1.0)
