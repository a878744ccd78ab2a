"""IEEE half inputs on the MFMA path vs the oracle (which reads the same float16 values exactly).
Tolerance: an eighth of the bf16 bar (three more significand bits, same arithmetic around them)."""
import math

import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import assert_close, to_device, to_f64
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu


def small_case(B, H, grid, group, pattern, radius, q_gain=1.0, seed=501):
    N = int(np.prod(grid))
    host = synth.make_qkv(B, H, N, 128, "f16", seed, q_gain=q_gain)
    dev = [to_device(x) for x in host]
    assert dev[0].dtype == torch.float16
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    O = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    torch.cuda.synchronize()
    return to_f64(O), orc.grat_attention(*host, grid, group, pattern, radius, scale)


@pytest.mark.parametrize("grid,group,pattern,radius", [
    ((64, 64), (16, 16), "block", (1, 1)),
    ((64, 64), (16, 16), "cross", (0, 0)),
    ((32, 48), (8, 16), "block", (1, 1)),             # 4-wave workgroups
    ((32, 48), (8, 8), "cross", (0, 0)),              # 2-wave workgroups
    ((4, 16, 24), (2, 8, 8), "cross_planes", (0, 0, 0)),
    ((40, 56), (16, 16), "block", (1, 1)),            # clipped border groups
])
def test_small_grouped(grid, group, pattern, radius):
    got, want = small_case(2, 3, grid, group, pattern, radius, q_gain=2.0)
    print(assert_close(got, want, "f16", f"f16 {grid} {group} {pattern}"))


@pytest.mark.parametrize("q_gain", [4.0, 16.0, 40.0])
def test_peaked_softmax_stays_in_half_range(q_gain):
    """Scores spread over hundreds of units: weights taken against a stale reference maximum must be
    refreshed before they leave the range of a half (65504)."""
    got, want = small_case(1, 2, (64, 64), (16, 16), "cross", (0, 0), q_gain=q_gain, seed=502)
    print(assert_close(got, want, "f16", f"f16 peaked x{q_gain}"))


def test_rising_scores_force_refreshes():
    """Keys ordered so that every KV tile beats the previous one by far more than 2^15."""
    grid, group = (64, 64), (16, 16)
    N = 4096
    Q, K, V = synth.make_qkv(1, 2, N, 128, "f16", 503)
    ramp = (np.arange(N, dtype=np.float32) / N * 6.0)[None, None, :, None]      # key magnitude grows along the sequence
    K = (K.astype(np.float32) * 0.05 + ramp * np.sign(Q.astype(np.float32).mean(axis=2, keepdims=True) + 1e-3)).astype(np.float16)
    Q = (Q.astype(np.float32) * 0.05 + 3.0 * np.sign(Q.astype(np.float32).mean(axis=2, keepdims=True) + 1e-3)).astype(np.float16)
    dev = [to_device(x) for x in (Q, K, V)]
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, "cross", (0, 0))
    O = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    torch.cuda.synchronize()
    want = orc.grat_attention(Q, K, V, grid, group, "cross", (0, 0), scale)
    print(assert_close(to_f64(O), want, "f16", "f16 rising scores"))


@pytest.mark.parametrize("N", [1, 65, 1000])
def test_dense(N):
    host = synth.make_qkv(2, 2, N, 128, "f16", 504, q_gain=2.0)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    O = grat.grat_dense_attention_fwd(*dev, scale)
    torch.cuda.synchronize()
    print(assert_close(to_f64(O), orc.dense_attention(*host, scale), "f16", f"f16 dense N={N}"))


def test_joint_and_packed():
    grid, group, n_global = (32, 32), (16, 16), 100
    L = n_global + 1024
    host = synth.make_qkv(1, 3, L, 128, "f16", 505, q_gain=2.0)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    want = orc.joint_attention(*host, n_global, True, grid, group, "block", (1, 1), scale)
    O = grat.grat_attention_global_fwd(*dev, scale, n_global, True, grid, group, count, index)
    QKV = torch.stack([t.permute(0, 2, 1, 3) for t in dev], dim=2).contiguous()
    Op = grat.grat_attention_packed_fwd(QKV, scale, grid, group, count, index, n_global=n_global)
    torch.cuda.synchronize()
    assert_close(to_f64(O), want, "f16", "f16 joint")
    assert torch.equal(O, Op.permute(0, 2, 1, 3))
