"""Pins for the oracle's grouping, attendable-set predicate, block lists and mask.

None of these re-use the oracle to check itself: the expected values are hand-enumerated
lists, closed-form counts, figures printed in the paper's tables, or nested loops written
directly from the set definitions of Sec. 3.2.
"""
import itertools
import math

import numpy as np
import pytest

from conftest import read_golden_figures, read_golden_lists
from oracle import grat_oracle as orc


def lists_as_dict(count, index):
    return {g: [int(x) for x in index[g, :count[g]]] for g in range(len(count))}


# -- hand-enumerated lists on a 4x4 group grid (Eq. 5-8) ----------------------------------
@pytest.mark.parametrize("grid,group", [((32, 32), (8, 8)), ((64, 64), (16, 16)), ((4, 4), (1, 1))])
def test_block_lists_match_hand_enumeration_4x4(grid, group):
    want = read_golden_lists("lists_4x4_block_b1.txt")
    count, index = orc.block_lists(grid, group, "block", (1, 1))
    assert lists_as_dict(count, index) == want
    assert index.shape == (16, 9) and (index[count[:, None] <= np.arange(9)] == -1).all()
    assert int(count.sum()) == 100


@pytest.mark.parametrize("pattern", ["cross", "cross_planes"])
def test_cross_lists_match_hand_enumeration_4x4(pattern):
    want = read_golden_lists("lists_4x4_cross.txt")
    count, index = orc.block_lists((32, 32), (8, 8), pattern, (0, 0))
    assert lists_as_dict(count, index) == want
    assert index.shape == (16, 7) and int(count.sum()) == 112


# -- brute force straight from the set definitions, any dimension -------------------------
def brute_lists(gg, pattern, radius):
    ndim = len(gg)
    ids = list(itertools.product(*[range(n) for n in gg]))
    lin = {p: i for i, p in enumerate(ids)}  # itertools.product is row-major, last fastest
    out = {}
    for p in ids:
        keep = []
        for m in ids:
            if pattern == "block":
                ok = all(abs(m[k] - p[k]) <= radius[k] for k in range(ndim))
            elif pattern == "cross":          # on a common axis line through p
                ok = sum(m[k] != p[k] for k in range(ndim)) <= 1
            elif pattern == "cross_planes":   # Eq. 14-15 as printed
                ok = any(m[k] == p[k] for k in range(ndim))
            else:
                ok = True
            if ok:
                keep.append(lin[m])
        out[lin[p]] = sorted(keep)
    return out


@pytest.mark.parametrize("grid,group,pattern,radius", [
    ((12, 20), (4, 4), "block", (1, 1)),
    ((12, 20), (4, 4), "block", (0, 2)),
    ((12, 20), (4, 4), "block", (5, 5)),
    ((12, 20), (4, 4), "cross", (0, 0)),
    ((10, 21), (4, 4), "block", (1, 1)),          # ragged last groups: 3 x 6 group grid
    ((10, 21), (4, 4), "cross", (0, 0)),
    ((6, 8, 10), (2, 4, 2), "block", (1, 1, 1)),
    ((6, 8, 10), (2, 4, 2), "block", (1, 0, 2)),
    ((6, 8, 10), (2, 4, 2), "cross", (0, 0, 0)),
    ((6, 8, 10), (2, 4, 2), "cross_planes", (0, 0, 0)),
    ((6, 8, 10), (2, 4, 2), "dense", (0, 0, 0)),
    ((24,), (4,), "block", (1,)),
])
def test_lists_match_brute_force(grid, group, pattern, radius):
    gg = orc.group_grid(grid, group)
    count, index = orc.block_lists(grid, group, pattern, radius)
    assert lists_as_dict(count, index) == brute_lists(gg, pattern, radius)


# -- closed-form totals at the five benchmark shapes --------------------------------------
def block_total_closed_form(gg, radius):
    tot = 1
    for G, b in zip(gg, radius):
        tot *= sum(min(G - 1, p + b) - max(0, p - b) + 1 for p in range(G))
    return tot


@pytest.mark.parametrize("grid,group,radius,total,max_kv", [
    ((32, 32), (8, 8), (1, 1), 100, 9),
    ((64, 64), (16, 16), (1, 1), 100, 9),
    ((128, 128), (16, 16), (1, 1), 484, 9),
    ((128, 128), (16, 16), (2, 2), 1156, 25),
    ((512, 512), (16, 16), (1, 1), 8836, 9),
    ((30, 48, 80), (2, 8, 8), (1, 1, 1), 19264, 27),
])
def test_block_totals(grid, group, radius, total, max_kv):
    count, index = orc.block_lists(grid, group, "block", radius)
    assert int(count.sum()) == total == block_total_closed_form(orc.group_grid(grid, group), radius)
    assert index.shape[1] == max_kv


@pytest.mark.parametrize("grid,group,pattern,per_group", [
    ((32, 32), (8, 8), "cross", 7),
    ((128, 128), (16, 16), "cross", 15),
    ((512, 512), (16, 16), "cross", 63),
    ((30, 48, 80), (2, 8, 8), "cross", 29),            # 15 + 6 + 10 - 2
    ((30, 48, 80), (2, 8, 8), "cross_planes", 270),    # inclusion-exclusion over 3 planes
])
def test_cross_counts(grid, group, pattern, per_group):
    count, index = orc.block_lists(grid, group, pattern, (0,) * len(grid))
    assert (count == per_group).all() and index.shape[1] == per_group
    assert (index >= 0).all()


def test_lists_symmetric_and_self_inclusive():
    for grid, group, pattern, radius in [((128, 128), (16, 16), "block", (2, 1)),
                                         ((30, 48, 80), (2, 8, 8), "cross", (0, 0, 0)),
                                         ((12, 12, 12), (4, 4, 4), "cross_planes", (0, 0, 0))]:
        count, index = orc.block_lists(grid, group, pattern, radius)
        G = len(count)
        A = np.zeros((G, G), dtype=bool)
        for g in range(G):
            A[g, index[g, :count[g]]] = True
            assert (np.diff(index[g, :count[g]]) > 0).all()
        assert (A == A.T).all() and A.diagonal().all()


# -- figures printed in the paper ----------------------------------------------------------
def farthest(rows, grid, group, pattern, radius):
    """max over attended (query, key) pairs of || |delta_k| + 1 ||_2, floored."""
    mask = orc.mask_rows(np.asarray(rows), grid, group, pattern, radius)
    xq = np.stack(np.unravel_index(np.asarray(rows), grid), -1)
    xk = np.stack(np.unravel_index(np.arange(int(np.prod(grid))), grid), -1)
    best = 0.0
    for r in range(len(rows)):
        ext = np.abs(xk[mask[r]] - xq[r]) + 1
        best = max(best, float(np.sqrt((ext.astype(np.float64) ** 2).sum(-1)).max()))
    return math.floor(best)


def corner_rows(grid, group, gcoord):
    """Token rows of the corners of group gcoord."""
    lo = [p * g for p, g in zip(gcoord, group)]
    hi = [min(t, l + g) - 1 for t, l, g in zip(grid, lo, group)]
    pts = itertools.product(*[(l, h) for l, h in zip(lo, hi)])
    return [int(np.ravel_multi_index(p, grid)) for p in pts]


def test_farthest_token_figures():
    fig = read_golden_figures()
    img, vid = (512, 512), (32, 48, 80)
    rows = corner_rows(img, (16, 16), (5, 7)) + corner_rows(img, (16, 16), (0, 0))
    assert farthest(rows, img, (16, 16), "block", (1, 1)) == fig["farthest_image_gratb_16_b1"]
    assert farthest(rows, img, (16, 16), "cross", (0, 0)) == fig["farthest_image_gratx_16"]
    assert farthest(rows, img, (16, 16), "dense", (0, 0)) == fig["farthest_image_full"]
    vrows = corner_rows(vid, (4, 8, 8), (3, 2, 4)) + corner_rows(vid, (4, 8, 8), (0, 0, 0))
    assert farthest(vrows, vid, (4, 8, 8), "block", (1, 1, 1)) == fig["farthest_video_gratb_4x8x8_b1"]
    assert farthest(vrows, vid, (4, 8, 8), "dense", (0, 0, 0)) == fig["farthest_video_full"]


@pytest.mark.parametrize("g", [8, 16, 32])
def test_gratx_sparsity_figures(g):
    fig = read_golden_figures()
    n_img, n_txt = 512 * 512, 512
    # every image query attends its criss-cross image tokens plus the prompt tokens
    count, _ = orc.block_lists((512, 512), (g, g), "cross", (0, 0))
    assert len(set(count.tolist())) == 1
    per_query = int(count[0]) * g * g
    assert per_query == int(orc.mask_rows(np.array([777]), (512, 512), (g, g), "cross", (0, 0)).sum())
    sparsity = 100.0 * (1.0 - (per_query + n_txt) / (n_img + n_txt))
    assert abs(sparsity - fig[f"sparsity_gratx_{g}"]) < 0.0075


def test_video_gratx_plane_counts():
    fig = read_golden_figures()
    gg = (8, 6, 10)
    count, index = orc.block_lists((32, 48, 80), (4, 8, 8), "cross_planes", (0, 0, 0))
    plane_sum = gg[1] * gg[2] + gg[0] * gg[2] + gg[0] * gg[1]
    assert plane_sum == fig["video_gratx_plane_sum"]
    union = plane_sum - (gg[0] + gg[1] + gg[2]) + 1
    assert (count == union).all()
    lines, _ = orc.block_lists((32, 48, 80), (4, 8, 8), "cross", (0, 0, 0))
    assert (lines == sum(gg) - 2).all()


# -- the mask comes from token coordinates and must agree with the lists -------------------
@pytest.mark.parametrize("grid,group,pattern,radius", [
    ((32, 32), (8, 8), "block", (1, 1)),
    ((32, 32), (8, 8), "cross", (0, 0)),
    ((10, 21), (4, 4), "block", (1, 1)),
    ((6, 8, 10), (2, 4, 2), "cross", (0, 0, 0)),
    ((6, 8, 10), (2, 4, 2), "cross_planes", (0, 0, 0)),
    ((6, 8, 10), (2, 4, 2), "block", (1, 0, 1)),
])
def test_mask_equals_lists_expanded(grid, group, pattern, radius):
    N = int(np.prod(grid))
    gg = orc.group_grid(grid, group)
    mask = orc.mask_rows(np.arange(N), grid, group, pattern, radius)
    count, index = orc.block_lists(grid, group, pattern, radius)
    # token -> linear group id, typed out here from Eq. 2-4 / 9-11
    gid = np.empty(N, dtype=np.int64)
    for r, x in enumerate(itertools.product(*[range(t) for t in grid])):
        lin = 0
        for k in range(len(grid)):
            lin = lin * gg[k] + x[k] // group[k]
        gid[r] = lin
    want = np.zeros((N, N), dtype=bool)
    for r in range(N):
        want[r] = np.isin(gid, index[gid[r], :count[gid[r]]])
    assert (mask == want).all()
    assert orc.attended_pairs(grid, group, pattern, radius) == int(mask.sum())


def test_attended_pairs_benchmark_shapes():
    assert orc.attended_pairs((32, 32), (8, 8), "block", (1, 1)) == 409_600
    assert orc.attended_pairs((32, 32), (8, 8), "cross", (0, 0)) == 458_752
    assert orc.attended_pairs((512, 512), (16, 16), "block", (1, 1)) == 8836 * 65536
    assert orc.attended_pairs((512, 512), (16, 16), "cross", (0, 0)) == 64512 * 65536
    assert orc.attended_pairs((30, 48, 80), (2, 8, 8), "block", (1, 1, 1)) == 19264 * 16384
