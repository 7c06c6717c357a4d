"""The measurement aid tsm_mfma_probe: runs, reports the operation count of its launch, leaves its sink alone."""
import pytest
import torch

from paper_1910_00932_amd import binding as B

pytestmark = pytest.mark.gpu


def test_mfma_probe_runs_and_counts():
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    flops = B.tsm_mfma_probe(100, sink)
    torch.cuda.synchronize()
    # blocks (2 per CU) x 4 wavefronts x iters x 4 chains x one 32x32x16 MFMA
    assert flops == cus * 2 * 4 * 100 * 4 * 2.0 * 32 * 32 * 16
    assert float(sink.item()) == 0.0
