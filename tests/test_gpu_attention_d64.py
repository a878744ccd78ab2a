"""head_dim 64 on the MFMA path (bf16 and half) vs the oracle."""
import math

import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import assert_close, to_device, to_f64
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("grid,group,pattern,radius", [
    ((64, 64), (16, 16), "block", (1, 1)),
    ((64, 64), (16, 16), "cross", (0, 0)),
    ((32, 48), (8, 16), "block", (1, 1)),             # 4-wave workgroups
    ((32, 48), (8, 8), "cross", (0, 0)),              # 2-wave workgroups
    ((4, 16, 24), (2, 8, 8), "block", (1, 1, 1)),
    ((40, 56), (16, 16), "block", (1, 1)),            # clipped border groups
])
def test_small_grouped(dtype, grid, group, pattern, radius):
    N = int(np.prod(grid))
    host = synth.make_qkv(2, 3, N, 64, dtype, 601, q_gain=2.0)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(64)
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    O = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    torch.cuda.synchronize()
    want = orc.grat_attention(*host, grid, group, pattern, radius, scale)
    assert_close(to_f64(O), want, dtype, f"d64 {dtype} {grid} {group} {pattern}")


@pytest.mark.parametrize("N", [1, 65, 1000])
def test_dense(N):
    host = synth.make_qkv(2, 2, N, 64, "bf16", 602, q_gain=2.0)
    dev = [to_device(x) for x in host]
    O = grat.grat_dense_attention_fwd(*dev, 0.125)
    torch.cuda.synchronize()
    assert_close(to_f64(O), orc.dense_attention(*host, 0.125), "bf16", f"d64 dense N={N}")


def test_joint_and_packed():
    grid, group, n_global = (32, 32), (16, 16), 100
    host = synth.make_qkv(1, 3, n_global + 1024, 64, "bf16", 603, q_gain=2.0)
    dev = [to_device(x) for x in host]
    count, index = grat.grat_build_block_lists(grid, group, "cross", (0, 0))
    want = orc.joint_attention(*host, n_global, False, grid, group, "cross", (0, 0), 0.125)
    O = grat.grat_attention_global_fwd(*dev, 0.125, n_global, False, grid, group, count, index)
    QKV = torch.stack([t.permute(0, 2, 1, 3) for t in dev], dim=2).contiguous()
    Op = grat.grat_attention_packed_fwd(QKV, 0.125, grid, group, count, index, n_global=n_global, global_first=False)
    torch.cuda.synchronize()
    assert_close(to_f64(O), want, "bf16", "d64 joint")
    assert torch.equal(O, Op.permute(0, 2, 1, 3))


def test_token_major_layout_with_wider_stride():
    """[B][N][H][64] storage (token stride H*64 elements) passed as a [B][H][N][64] view."""
    grid, group = (32, 32), (16, 16)
    host = synth.make_qkv(1, 4, 1024, 64, "bf16", 604)
    want = orc.grat_attention(*host, grid, group, "block", (1, 1), 0.125)
    dev = [to_device(np.ascontiguousarray(x.transpose(0, 2, 1, 3))).permute(0, 2, 1, 3) for x in host]
    out = torch.zeros_like(dev[0].permute(0, 2, 1, 3).contiguous()).permute(0, 2, 1, 3)
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    grat.grat_attention_fwd(*dev, 0.125, grid, group, count, index, out=out)
    torch.cuda.synchronize()
    assert_close(to_f64(out), want, "bf16", "d64 token-major")
