"""fp32 attention path vs the oracle: max-abs and relative L2 within 1e-4."""
import math

import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import assert_close, to_device, to_f64
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


def run_grouped(Q, K, V, grid, group, pattern, radius, scale):
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    O = grat.grat_attention_fwd(to_device(Q), to_device(K), to_device(V), scale, grid, group, count, index)
    torch.cuda.synchronize()
    return to_f64(O)


@pytest.mark.parametrize("label", ["B3", "X"])
def test_tiny2d_workload(label):
    w = synth.WORKLOADS["tiny2d"]
    pattern, radius = w.patterns[label]
    Q, K, V = synth.make_workload_qkv(w)
    want = orc.grat_attention(Q, K, V, w.grid, w.group, pattern, radius, w.scale)
    got = run_grouped(Q, K, V, w.grid, w.group, pattern, radius, w.scale)
    assert_close(got, want, "f32", f"tiny2d {label}")


@pytest.mark.parametrize("grid,group,pattern,radius,heads,d", [
    ((24, 40), (8, 8), "block", (1, 2), 3, 64),
    ((24, 40), (4, 10), "cross", (0, 0), 2, 128),     # 40-token groups: ragged 32-key tiles
    ((9, 11), (1, 1), "cross", (0, 0), 2, 64),        # per-token criss-cross
    ((9, 11), (1, 1), "block", (2, 2), 2, 64),        # per-token square window
    ((6, 16, 20), (2, 8, 5), "block", (1, 1, 1), 2, 64),   # 80-token groups
    ((6, 16, 20), (2, 8, 5), "cross", (0, 0, 0), 2, 64),
    ((6, 16, 20), (2, 8, 5), "cross_planes", (0, 0, 0), 2, 64),
    ((6, 16, 20), (3, 16, 20), "dense", (0, 0, 0), 1, 64),  # 960-token groups: 15 query tiles
])
def test_small_shapes(grid, group, pattern, radius, heads, d):
    N = int(np.prod(grid))
    Q, K, V = synth.make_qkv(2, heads, N, d, "f32", 77, q_gain=2.0)
    scale = 1.0 / math.sqrt(d)
    want = orc.grat_attention(Q, K, V, grid, group, pattern, radius, scale)
    got = run_grouped(Q, K, V, grid, group, pattern, radius, scale)
    assert_close(got, want, "f32", f"{grid} {group} {pattern}")


@pytest.mark.parametrize("grid,group,pattern,radius,d", [
    ((30, 44), (8, 8), "block", (1, 1), 64),              # last groups 6 rows / 4 columns deep
    ((30, 44), (8, 8), "cross", (0, 0), 64),
    ((5, 7), (2, 3), "block", (1, 1), 64),                # the oracle's own ragged pin shape
    ((70,), (16,), "block", (1,), 128),                   # 1D, last group of 6 tokens
    ((5, 18, 20), (2, 8, 8), "block", (1, 1, 1), 64),     # ragged on all three axes
    ((5, 18, 20), (2, 8, 8), "cross_planes", (0, 0, 0), 64),
    ((100, 9), (40, 4), "cross", (0, 0), 64),             # 160-token boxes: border groups with fewer query tiles
])
def test_group_dims_not_dividing_the_grid(grid, group, pattern, radius, d):
    """Eq. 2-4 are floor divisions: border groups are the part of their box inside the grid."""
    N = int(np.prod(grid))
    Q, K, V = synth.make_qkv(2, 2, N, d, "f32", 79, q_gain=2.0)
    scale = 1.0 / math.sqrt(d)
    want = orc.grat_attention(Q, K, V, grid, group, pattern, radius, scale)
    got = run_grouped(Q, K, V, grid, group, pattern, radius, scale)
    assert_close(got, want, "f32", f"ragged {grid} {group} {pattern}")


@pytest.mark.parametrize("N", [1, 31, 64, 1000])
def test_dense(N):
    Q, K, V = synth.make_qkv(1, 3, N, 64, "f32", 78, q_gain=3.0)
    want = orc.dense_attention(Q, K, V, 0.125)
    O = grat.grat_dense_attention_fwd(to_device(Q), to_device(K), to_device(V), 0.125)
    torch.cuda.synchronize()
    assert_close(to_f64(O), want, "f32", f"dense N={N}")


def test_token_major_strides():
    """[B][N][H][d] storage passed as a [B][H][N][d] view."""
    w = synth.WORKLOADS["tiny2d"]
    Q, K, V = synth.make_workload_qkv(w)
    want = orc.grat_attention(Q, K, V, w.grid, w.group, "block", (1, 1), w.scale)
    count, index = grat.grat_build_block_lists(w.grid, w.group, "block", (1, 1))
    dev = [to_device(np.ascontiguousarray(x.transpose(0, 2, 1, 3))).permute(0, 2, 1, 3) for x in (Q, K, V)]
    out = torch.zeros_like(dev[0].permute(0, 2, 1, 3).contiguous()).permute(0, 2, 1, 3)
    grat.grat_attention_fwd(*dev, w.scale, w.grid, w.group, count, index, out=out)
    torch.cuda.synchronize()
    assert not out.is_contiguous()
    assert_close(to_f64(out), want, "f32", "token-major")
