"""GPU block lists vs the oracle: bit-exact (counts, ascending ids, -1 padding)."""
import numpy as np
import pytest
import torch

import paper_2505_14687_amd as grat
from oracle import grat_oracle as orc
from paper_2505_14687_amd import synth

pytestmark = pytest.mark.gpu

CASES = [(w.grid, w.group, pat, rad) for w in synth.WORKLOADS.values() for pat, rad in w.patterns.values()]
CASES += [
    ((128, 128), (16, 16), "block", (8, 8)),         # radius covers the grid
    ((128, 128), (16, 16), "block", (0, 3)),
    ((130, 70), (16, 16), "block", (1, 1)),          # ragged last groups
    ((130, 70), (16, 16), "cross", (0, 0)),
    ((512, 512), (8, 8), "cross", (0, 0)),           # 4096 groups
    ((512, 512), (32, 32), "block", (1, 1)),
    ((32, 48, 80), (4, 8, 8), "cross_planes", (0, 0, 0)),
    ((32, 48, 80), (4, 8, 8), "block", (1, 1, 1)),
    ((7, 5, 3), (1, 1, 1), "cross", (0, 0, 0)),
    ((4096,), (64,), "block", (2,)),
    ((4096,), (64,), "cross_planes", (0,)),
    ((64, 64), (64, 64), "block", (1, 1)),           # a single group
]


@pytest.mark.parametrize("grid,group,pattern,radius", CASES)
def test_block_lists_bit_exact(grid, group, pattern, radius):
    want_count, want_index = orc.block_lists(grid, group, pattern, radius)
    G, max_kv = grat.grat_block_list_shape(grid, group, pattern, radius)
    assert G == len(want_count) and max_kv == want_index.shape[1]
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    torch.cuda.synchronize()
    assert count.dtype == torch.int32 and index.dtype == torch.int32
    assert np.array_equal(count.cpu().numpy(), want_count)
    assert np.array_equal(index.cpu().numpy(), want_index)


def test_wider_pitch_is_padded_with_minus_one():
    grid, group = (128, 128), (16, 16)
    want_count, want_index = orc.block_lists(grid, group, "block", (1, 1))
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1), max_kv=13)
    torch.cuda.synchronize()
    got = index.cpu().numpy()
    assert got.shape == (64, 13)
    assert np.array_equal(got[:, :9], want_index) and (got[:, 9:] == -1).all()
    assert np.array_equal(count.cpu().numpy(), want_count)


def test_rebuild_is_deterministic():
    a = grat.grat_build_block_lists((30, 48, 80), (2, 8, 8), "cross_planes")
    b = grat.grat_build_block_lists((30, 48, 80), (2, 8, 8), "cross_planes")
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_validate_block_lists_flags():
    """grat_validate_block_lists through the C ABI: 0 for the builder's own lists (also with a wider
    row pitch), and the flag of every kind of damage planted in a copy of them."""
    from paper_2505_14687_amd.grat import LIST_BAD_COUNT, LIST_BAD_ENTRY, LIST_BAD_PADDING
    for grid, group, pattern, radius in [((128, 128), (16, 16), "block", (1, 1)), ((30, 48, 80), (2, 8, 8), "cross", None),
                                         ((70, 50), (16, 16), "cross_planes", None)]:
        G, need = grat.grat_block_list_shape(grid, group, pattern, radius)
        for max_kv in (need, need + 5):
            count, index = grat.grat_build_block_lists(grid, group, pattern, radius, max_kv=max_kv)
            assert grat.grat_validate_block_lists(grid, group, count, index).item() == 0
            def damaged(edit):
                c, i = count.clone(), index.clone()
                edit(c, i)
                return grat.grat_validate_block_lists(grid, group, c, i).item()
            def zero_count(c, i): c[G // 2] = 0
            def long_count(c, i): c[G - 1] = max_kv + 1
            def entry_past_end(c, i): i[3, 0] = G
            def negative_entry(c, i): i[0, 1] = -1
            def dirty_padding(c, i): i[0, max_kv - 1] = 0        # (a corner group: its list is shorter than the row)
            assert damaged(zero_count) & LIST_BAD_COUNT
            assert damaged(long_count) & LIST_BAD_COUNT
            assert damaged(entry_past_end) == LIST_BAD_ENTRY
            assert damaged(negative_entry) == LIST_BAD_ENTRY
            if int(count[0]) < max_kv:
                assert damaged(dirty_padding) == LIST_BAD_PADDING
