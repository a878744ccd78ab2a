"""The library enqueues on the stream the caller names, ordered with what that stream already holds."""
import math

import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import to_device
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


def test_side_stream_is_the_launch_stream():
    """Work is enqueued on the stream the caller names and ordered with what that stream already
    holds: inputs written by copies on a side stream (default priority) are what the kernels read,
    and the result equals a run on the default stream bit for bit."""
    grid, group = (64, 64), (16, 16)
    scale = 1.0 / math.sqrt(128)
    host = [to_device(x) for x in synth.make_qkv(1, 4, 4096, 128, "bf16", 410)]
    count, index = grat.grat_build_block_lists(grid, group, "cross", (0, 0))
    want = grat.grat_attention_fwd(*host, scale, grid, group, count, index)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    Q, K, V = (torch.zeros_like(t) for t in host)
    O = torch.zeros_like(Q)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for dst, src in zip((Q, K, V), host):
            dst.copy_(src, non_blocking=True)
        c2, i2 = grat.grat_build_block_lists(grid, group, "cross", (0, 0), stream=side)
        grat.grat_attention_fwd(Q, K, V, scale, grid, group, c2, i2, out=O, stream=side)
    side.synchronize()
    assert torch.equal(O, want)
