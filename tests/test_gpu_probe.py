"""The MFMA-only probe (measurement aid of bench.py) runs the count of instructions it reports."""
import math

import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import to_device
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("data", ["ones", "small_ints", "normal_like"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_mfma_probe_does_its_work(dtype, data):
    from paper_2505_14687_amd.probe import probe_wave_sum
    sink = grat.grat_probe_mfma(dtype, data, 512, 64)
    torch.cuda.synchronize()
    assert sink.shape == (512 * 256,)
    assert torch.all(sink.view(-1, 64).sum(1) == probe_wave_sum(data, 64))
