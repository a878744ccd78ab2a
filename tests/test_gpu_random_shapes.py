"""Seeded sweep of small random configurations through the 16-bit MFMA path, every output row against
the oracle: grids of 1 to 3 axes that the group does or does not divide, groups of 64 to 512 tokens,
all patterns and radii, head_dim 64 / 128, bf16 / half, with and without prompt tokens.  The cases
are drawn once from a fixed seed, so every run sees the same ones; sizes stay below 4 608 tokens so
that the oracle takes a second or two per case.
"""
import math

import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from gpu_util import assert_all_written, assert_close, gather_rows, nan_like, to_device, to_f64
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu

GROUPS = {
    1: [(64,), (128,), (256,)],
    2: [(8, 8), (8, 16), (16, 8), (16, 16), (4, 16), (16, 32), (2, 32)],
    3: [(2, 8, 8), (4, 4, 4), (4, 8, 8), (1, 8, 8), (2, 4, 16), (4, 4, 8)],
}


def draw_cases(seed: int, count: int):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        ndim = int(rng.integers(1, 4))
        group = GROUPS[ndim][int(rng.integers(len(GROUPS[ndim])))]
        ragged = bool(rng.integers(0, 3) == 0)
        grid = []
        for g in group:
            n_groups = int(rng.integers(1, 7 if ndim < 3 else 4))
            t = n_groups * g
            if ragged and g > 1 and n_groups > 1:
                t -= int(rng.integers(0, g))          # the last group of this axis is cut
            grid.append(t)
        n = int(np.prod(grid))
        if n < 64 or n > 4608:
            continue
        pattern = ("block", "cross", "cross_planes")[int(rng.integers(3))]
        radius = tuple(int(rng.integers(0, 3)) for _ in range(ndim)) if pattern == "block" else (0,) * ndim
        n_global = 0 if ragged or rng.integers(0, 3) else int(rng.integers(1, 200))
        cases.append(dict(
            grid=tuple(grid), group=group, pattern=pattern, radius=radius, n_global=n_global,
            global_first=bool(rng.integers(2)), head_dim=(64, 128)[int(rng.integers(2))],
            dtype=("bf16", "f16")[int(rng.integers(0, 4) == 0)], batch=int(rng.integers(1, 3)),
            heads=int(rng.integers(1, 4)), q_gain=float((1.0, 2.0, 4.0)[int(rng.integers(3))]),
            seed=7000 + len(cases)))
    return cases


CASES = draw_cases(20250514, 40)


def case_id(c):
    g = "x".join(map(str, c["grid"])) + "/" + "x".join(map(str, c["group"]))
    return f"{g}-{c['pattern']}{''.join(map(str, c['radius']))}-p{c['n_global']}-d{c['head_dim']}-{c['dtype']}"


@pytest.mark.parametrize("c", CASES, ids=case_id)
def test_random_shape(c):
    grid, group, pattern, radius = c["grid"], c["group"], c["pattern"], c["radius"]
    seq = c["n_global"] + int(np.prod(grid))
    host = synth.make_qkv(c["batch"], c["heads"], seq, c["head_dim"], c["dtype"], c["seed"], q_gain=c["q_gain"])
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(c["head_dim"])
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    want_count, want_index = orc.block_lists(grid, group, pattern, radius)
    assert np.array_equal(count.cpu().numpy(), want_count) and np.array_equal(index.cpu().numpy(), want_index)
    O = nan_like(dev[0])
    if c["n_global"]:
        grat.grat_attention_global_fwd(*dev, scale, c["n_global"], c["global_first"], grid, group, count, index, out=O)
        want = orc.joint_attention(*host, c["n_global"], c["global_first"], grid, group, pattern, radius, scale)
    else:
        grat.grat_attention_fwd(*dev, scale, grid, group, count, index, out=O)
        want = orc.grat_attention(*host, grid, group, pattern, radius, scale)
    torch.cuda.synchronize()
    assert_all_written(O, case_id(c))
    print(case_id(c), assert_close(to_f64(O), want, c["dtype"], case_id(c)))


# ---- the same, at sizes with more than 64 groups (the tile order of large launches), on sampled rows ----
def draw_mid_cases(seed: int, count: int):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        ndim = int(rng.integers(2, 4))
        group = GROUPS[ndim][int(rng.integers(len(GROUPS[ndim])))]
        ragged = bool(rng.integers(0, 3) == 0)
        grid = []
        for g in group:
            n_groups = int(rng.integers(3, 14 if ndim == 2 else 8))
            t = n_groups * g
            if ragged and g > 1:
                t -= int(rng.integers(0, g))
            grid.append(t)
        n = int(np.prod(grid))
        n_groups = int(np.prod([-(-t // g) for t, g in zip(grid, group)]))
        if n_groups <= 64 or n > 40000:
            continue
        pattern = ("block", "cross", "cross_planes")[int(rng.integers(3))]
        radius = tuple(int(rng.integers(0, 3)) for _ in range(ndim)) if pattern == "block" else (0,) * ndim
        n_global = 0 if ragged or rng.integers(0, 2) else int(rng.integers(1, 300))
        cases.append(dict(
            grid=tuple(grid), group=group, pattern=pattern, radius=radius, n_global=n_global,
            global_first=bool(rng.integers(2)), head_dim=(64, 128)[int(rng.integers(2))],
            dtype=("bf16", "f16")[int(rng.integers(0, 4) == 0)], batch=int(rng.integers(1, 3)),
            heads=int(rng.integers(2, 7)), q_gain=float((1.0, 2.0)[int(rng.integers(2))]),
            seed=7500 + len(cases)))
    return cases


MID_CASES = draw_mid_cases(20250515, 12)


@pytest.mark.parametrize("c", MID_CASES, ids=case_id)
def test_random_mid_shape_sampled_rows(c):
    grid, group, pattern, radius = c["grid"], c["group"], c["pattern"], c["radius"]
    seq = c["n_global"] + int(np.prod(grid))
    host = synth.make_qkv(c["batch"], c["heads"], seq, c["head_dim"], c["dtype"], c["seed"], q_gain=c["q_gain"], threads=16)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(c["head_dim"])
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    want_count, want_index = orc.block_lists(grid, group, pattern, radius)
    assert np.array_equal(count.cpu().numpy(), want_count) and np.array_equal(index.cpu().numpy(), want_index)
    samples = synth.sample_rows(c["seed"], 768, c["batch"], c["heads"], seq)
    O = nan_like(dev[0])
    if c["n_global"]:
        grat.grat_attention_global_fwd(*dev, scale, c["n_global"], c["global_first"], grid, group, count, index, out=O)
        want = orc.joint_attention_rows(*host, samples, c["n_global"], c["global_first"], grid, group, pattern, radius, scale)
    else:
        grat.grat_attention_fwd(*dev, scale, grid, group, count, index, out=O)
        want = orc.grat_attention_rows(*host, samples, grid, group, pattern, radius, scale)
    torch.cuda.synchronize()
    assert_all_written(O, case_id(c))
    print(case_id(c), assert_close(gather_rows(O, samples), want, c["dtype"], case_id(c)))
