"""grat_attention_packed_fwd: Q, K, V read in place from one [B, L, 3, H, d] buffer, O written as
[B, L, H, d] with its own strides; checked against the oracle on the unpacked tensors."""
import math

import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import assert_close, to_device, to_f64
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


def pack(dev):
    """[B, H, L, d] x 3 -> contiguous [B, L, 3, H, d]."""
    return torch.stack([t.permute(0, 2, 1, 3) for t in dev], dim=2).contiguous()


@pytest.mark.parametrize("dtype,d,grid,group,pattern,radius,n_global", [
    ("bf16", 128, (32, 32), (16, 16), "block", (1, 1), 0),
    ("bf16", 128, (32, 48), (8, 16), "cross", (0, 0), 0),          # 4-wave workgroups
    ("bf16", 128, (32, 48), (8, 8), "block", (1, 1), 0),           # 2-wave workgroups
    ("bf16", 128, (4, 16, 16), (4, 8, 8), "cross_planes", (0, 0, 0), 0),
    ("bf16", 128, (32, 32), (16, 16), "block", (1, 1), 100),       # prompt tokens ahead of the grid
    ("bf16", 128, (40, 56), (16, 16), "block", (1, 1), 0),         # clipped border groups, O with its own pitch
    ("f16", 64, (33, 47), (8, 8), "cross", (0, 0), 0),             # half, head_dim 64, clipped, 2-wave workgroups
    ("f32", 64, (30, 44), (8, 8), "block", (1, 1), 0),             # fp32 path, clipped
    ("f32", 64, (32, 32), (8, 8), "block", (1, 1), 0),
    ("f32", 128, (24, 40), (4, 8), "cross", (0, 0), 0),
])
def test_packed_small_all_rows(dtype, d, grid, group, pattern, radius, n_global):
    B, H = 2, 3
    L = n_global + int(np.prod(grid))
    host = synth.make_qkv(B, H, L, d, dtype, 311, q_gain=2.0)
    QKV = pack([to_device(x) for x in host])
    scale = 1.0 / math.sqrt(d)
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    O = grat.grat_attention_packed_fwd(QKV, scale, grid, group, count, index, n_global=n_global)
    torch.cuda.synchronize()
    assert O.shape == (B, L, H, d)
    if n_global:
        want = orc.joint_attention(*host, n_global, True, grid, group, pattern, radius, scale)
    else:
        want = orc.grat_attention(*host, grid, group, pattern, radius, scale)
    assert_close(to_f64(O.permute(0, 2, 1, 3)), want, dtype, f"packed {dtype} {grid} {pattern}")


def test_packed_equals_split_call_bitwise():
    grid, group = (64, 64), (16, 16)
    host = synth.make_qkv(1, 4, 4096, 128, "bf16", 312)
    dev = [to_device(x) for x in host]
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    a = grat.grat_attention_fwd(*dev, 0.09, grid, group, count, index)
    b = grat.grat_attention_packed_fwd(pack(dev), 0.09, grid, group, count, index)
    torch.cuda.synchronize()
    assert torch.equal(a, b.permute(0, 2, 1, 3))


def test_packed_buffer_beyond_4gib_sampled_rows():
    """512x512 tokens, 24 heads: the packed buffer is 4.8 GB, so row addresses need 64 bits."""
    w = synth.WORKLOADS["img8192"]
    pattern, radius = w.patterns["B3"]
    host = synth.make_workload_qkv(w, threads=16)
    QKV = pack([to_device(x) for x in host])
    assert QKV.numel() * QKV.element_size() > 1 << 32
    count, index = grat.grat_build_block_lists(w.grid, w.group, pattern, radius)
    O = grat.grat_attention_packed_fwd(QKV, w.scale, w.grid, w.group, count, index)
    torch.cuda.synchronize()
    samples = synth.sample_rows(2011, 768, w.batch, w.heads, w.n_tokens)
    samples[:4, 2] = [0, w.n_tokens - 1, w.n_tokens - 513, 233017]   # incl. rows past 2^31 elements
    want = orc.grat_attention_rows(*host, samples, w.grid, w.group, pattern, radius, w.scale)
    s = torch.from_numpy(samples).cuda()
    got = to_f64(O[s[:, 0], s[:, 2], s[:, 1]])
    print(assert_close(got, want, "bf16", "packed img8192 B3"))
