"""Joint sequences (prompt tokens + grid tokens) on the bf16 path vs the oracle."""
import math

import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import assert_all_written, assert_close, gather_rows, nan_like, to_device, to_f64
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


def run_joint(host, n_global, global_first, grid, group, pattern, radius, scale):
    dev = [to_device(x) for x in host]
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    O = nan_like(dev[0])
    grat.grat_attention_global_fwd(*dev, scale, n_global, global_first, grid, group, count, index, out=O)
    torch.cuda.synchronize()
    assert_all_written(O, f"joint {n_global} {grid} {pattern}")
    return O


@pytest.mark.parametrize("n_global,global_first,grid,group,pattern,radius", [
    (64, True, (32, 32), (16, 16), "block", (1, 1)),
    (64, False, (32, 32), (16, 16), "block", (1, 1)),
    (100, True, (32, 48), (8, 16), "cross", (0, 0)),          # ragged prompt tile, 4-wave workgroups
    (1, False, (32, 48), (8, 8), "block", (1, 1)),            # one prompt token, 2-wave workgroups
    (300, True, (48, 48), (16, 16), "cross", (0, 0)),         # more prompt rows than one dense tile
    (77, False, (4, 16, 24), (2, 8, 8), "block", (1, 1, 1)),
    (200, True, (4, 16, 16), (4, 8, 8), "cross_planes", (0, 0, 0)),
])
def test_joint_small_all_rows(n_global, global_first, grid, group, pattern, radius):
    L = n_global + int(np.prod(grid))
    host = synth.make_qkv(2, 3, L, 128, "bf16", 97, q_gain=2.0)
    scale = 1.0 / math.sqrt(128)
    O = run_joint(host, n_global, global_first, grid, group, pattern, radius, scale)
    want = orc.joint_attention(*host, n_global, global_first, grid, group, pattern, radius, scale)
    assert_close(to_f64(O), want, "bf16", f"joint {n_global} {global_first} {grid} {pattern}")


def test_joint_with_zero_prompt_tokens_equals_plain_call():
    grid, group = (32, 32), (16, 16)
    host = synth.make_qkv(1, 2, 1024, 128, "bf16", 98)
    dev = [to_device(x) for x in host]
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    a = grat.grat_attention_global_fwd(*dev, 0.09, 0, True, grid, group, count, index)
    b = grat.grat_attention_fwd(*dev, 0.09, grid, group, count, index)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("label,global_first", [("B3", True), ("X", False)])
def test_joint_image_scale_sampled_rows(label, global_first):
    """128x128 tokens + 512 prompt tokens, 24 heads: sampled rows incl. prompt rows."""
    w = synth.WORKLOADS["img2048"]
    pattern, radius = w.patterns[label]
    n_global = 512
    L = n_global + w.n_tokens
    host = synth.make_qkv(w.batch, w.heads, L, w.head_dim, "bf16", 1010, threads=16)
    O = run_joint(host, n_global, global_first, w.grid, w.group, pattern, radius, w.scale)
    samples = synth.sample_rows(2007, 1024, w.batch, w.heads, L)
    g0 = 0 if global_first else w.n_tokens
    samples[:64, 2] = g0 + np.arange(64) * 8          # prompt rows
    samples[64:68, 2] = [0, L - 1, g0 + n_global - 1, (n_global if global_first else 0) + 5]
    want = orc.joint_attention_rows(*host, samples, n_global, global_first, w.grid, w.group, pattern,
                                    radius, w.scale)
    print(label, assert_close(gather_rows(O, samples), want, "bf16", f"joint img2048 {label}"))


@pytest.mark.parametrize("label,global_first", [("B3", True), ("X", True)])
def test_joint_paper_scale_sampled_rows(label, global_first):
    """512x512 tokens + 512 prompt tokens, 24 heads (the sequence Tab. 1 / Tab. 6 were measured on,
    by their printed GRAT-X sparsities): sampled rows incl. prompt rows and the grid's corners."""
    w = synth.WORKLOADS["img8192"]
    pattern, radius = w.patterns[label]
    n_global = 512
    L = n_global + w.n_tokens
    host = synth.make_qkv(w.batch, w.heads, L, w.head_dim, "bf16", 1011, threads=16)
    O = run_joint(host, n_global, global_first, w.grid, w.group, pattern, radius, w.scale)
    samples = synth.sample_rows(2008, 512, w.batch, w.heads, L)
    samples[:32, 2] = np.arange(32) * 16              # prompt rows
    samples[32:36, 2] = [n_global, L - 1, n_global + 511, n_global + 511 * 512]
    want = orc.joint_attention_rows(*host, samples, n_global, global_first, w.grid, w.group, pattern,
                                    radius, w.scale)
    del host
    print(label, assert_close(gather_rows(O, samples), want, "bf16", f"joint img8192 {label}"))
