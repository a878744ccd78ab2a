"""bf16 MFMA attention path vs the oracle on the benchmark workloads and on edge shapes.

Tolerance (bf16 inputs): max-abs error <= 3e-2 and relative L2 error <= 1e-2 against the
float64 oracle evaluated on the same bf16 input bits.
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

_cache = {}


def workload_on_device(name, q_gain=1.0):
    """Host bits + device tensors of a workload, kept for the tests that share it."""
    key = (name, q_gain)
    if key not in _cache:
        _cache.clear()
        torch.cuda.empty_cache()
        w = synth.WORKLOADS[name]
        host = synth.make_workload_qkv(w, q_gain=q_gain, threads=16)
        _cache[key] = (w, host, [to_device(x) for x in host])
    return _cache[key]


def run_pattern(w, dev, pattern, radius):
    """Runs into a NaN-filled output and checks that every element was stored (the sampled-row
    tests below would not see a query tile that no workgroup took)."""
    O = nan_like(dev[0])
    if pattern == "dense":
        grat.grat_dense_attention_fwd(*dev, w.scale, out=O)
    else:
        count, index = grat.grat_build_block_lists(w.grid, w.group, pattern, radius)
        grat.grat_attention_fwd(*dev, w.scale, w.grid, w.group, count, index, out=O)
    torch.cuda.synchronize()
    assert_all_written(O, f"{pattern} {w.grid}")
    return O


# ---- the benchmark workloads ------------------------------------------------------------------
@pytest.mark.parametrize("label", ["B3", "X"])
def test_img1024_all_rows(label):
    w, host, dev = workload_on_device("img1024")
    pattern, radius = w.patterns[label]
    O = run_pattern(w, dev, pattern, radius)
    want = orc.grat_attention(*host, w.grid, w.group, pattern, radius, w.scale)
    print(label, assert_close(to_f64(O), want, "bf16", f"img1024 {label}"))


@pytest.mark.parametrize("label", ["B3", "B5", "X", "dense"])
def test_img2048(label):
    w, host, dev = workload_on_device("img2048")
    pattern, radius = w.patterns[label]
    O = run_pattern(w, dev, pattern, radius)
    samples = synth.sample_rows(2003, 4096, w.batch, w.heads, w.n_tokens)
    if pattern == "dense":
        samples = samples[np.lexsort((samples[:, 2], samples[:, 1], samples[:, 0]))]
        want = orc.dense_attention_rows(*host, samples, w.scale)
    else:
        want = orc.grat_attention_rows(*host, samples, w.grid, w.group, pattern, radius, w.scale)
    print(label, assert_close(gather_rows(O, samples), want, "bf16", f"img2048 {label} sampled"))
    # every row of one head
    h = 5
    one = [x[:, h:h + 1] for x in host]
    if pattern == "dense":
        full = orc.dense_attention(*one, w.scale)
    else:
        full = orc.grat_attention(*one, w.grid, w.group, pattern, radius, w.scale)
    assert_close(to_f64(O[:, h:h + 1]), full, "bf16", f"img2048 {label} head {h}")


@pytest.mark.parametrize("label", ["B3", "X"])
def test_img8192_sampled_rows(label):
    w, host, dev = workload_on_device("img8192")
    pattern, radius = w.patterns[label]
    O = run_pattern(w, dev, pattern, radius)
    samples = synth.sample_rows(2004, 4096, w.batch, w.heads, w.n_tokens)
    # make sure border groups (short lists) and every head are among the samples
    corners = np.array([[0, h, r] for h in range(w.heads)
                        for r in (0, 511, 511 * 512, 512 * 512 - 1, 255 * 512 + 256)], dtype=np.int64)
    samples = np.concatenate([samples[:-len(corners)], corners])
    want = orc.grat_attention_rows(*host, samples, w.grid, w.group, pattern, radius, w.scale)
    print(label, assert_close(gather_rows(O, samples), want, "bf16", f"img8192 {label}"))


@pytest.mark.parametrize("label", ["B3", "X", "Xplanes"])
def test_video_sampled_rows(label):
    w, host, dev = workload_on_device("video")
    pattern, radius = w.patterns[label]
    O = run_pattern(w, dev, pattern, radius)
    samples = synth.sample_rows(2005, 2048, w.batch, w.heads, w.n_tokens)
    samples[:4, 2] = [0, w.n_tokens - 1, 79, 48 * 80 * 29]
    want = orc.grat_attention_rows(*host, samples, w.grid, w.group, pattern, radius, w.scale)
    print(label, assert_close(gather_rows(O, samples), want, "bf16", f"video {label}"))


# ---- beyond the five configs: the paper's video shape and its group-size / radius ablation ------
@pytest.mark.parametrize("name,label", [
    ("video_paper", "B3"), ("video_paper", "X"), ("video_paper", "Xplanes"),
    ("img8192_g8", "B3"), ("img8192_g8", "B5"), ("img8192_g8", "B7"), ("img8192_g8", "X"),
    ("img8192_g32", "B3"), ("img8192_g32", "X"),
    ("img8192_b2", "B5"),
])
def test_paper_shapes_sampled_rows(name, label):
    w, host, dev = workload_on_device(name)
    pattern, radius = w.patterns[label]
    O = run_pattern(w, dev, pattern, radius)
    samples = synth.sample_rows(2006, 1024, w.batch, w.heads, w.n_tokens)
    samples[:3, 2] = [0, w.n_tokens - 1, w.n_tokens // 2 + 17]
    want = orc.grat_attention_rows(*host, samples, w.grid, w.group, pattern, radius, w.scale)
    print(name, label, assert_close(gather_rows(O, samples), want, "bf16", f"{name} {label}"))


# ---- edge shapes ----------------------------------------------------------------------------
def small_case(B, H, grid, group, pattern, radius, q_gain=1.0, seed=91):
    N = int(np.prod(grid))
    host = synth.make_qkv(B, H, N, 128, "bf16", seed, q_gain=q_gain)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, pattern, radius)
    O = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    torch.cuda.synchronize()
    want = orc.grat_attention(*host, grid, group, pattern, radius, scale)
    return to_f64(O), want


@pytest.mark.parametrize("grid,group,pattern,radius", [
    ((32, 48), (8, 8), "block", (1, 1)),              # 64-token groups: 2-wave workgroups
    ((32, 48), (8, 8), "cross", (0, 0)),
    ((32, 48), (8, 16), "block", (1, 1)),             # 128-token groups: 4-wave workgroups
    ((48, 48), (16, 16), "block", (1, 0)),            # 256-token groups, asymmetric radius
    ((48, 48), (24, 8), "cross", (0, 0)),             # 192-token groups -> 64-row query tiles
    ((64, 64), (32, 32), "block", (1, 1)),            # 1024-token groups: 4 query tiles each
    ((4, 16, 24), (2, 8, 8), "block", (1, 1, 1)),
    ((4, 16, 24), (2, 8, 8), "cross", (0, 0, 0)),
    ((4, 16, 24), (2, 8, 8), "cross_planes", (0, 0, 0)),
    ((6, 16, 16), (3, 4, 16), "block", (0, 1, 1)),    # 192-token 3D groups
    ((16, 16), (16, 16), "block", (1, 1)),            # a single group
    ((2048,), (128,), "block", (1,)),                 # 1D sequence, sliding blocks
])
def test_small_grouped(grid, group, pattern, radius):
    got, want = small_case(2, 3, grid, group, pattern, radius)
    assert_close(got, want, "bf16", f"{grid} {group} {pattern}")


@pytest.mark.parametrize("grid,group,pattern,radius", [
    ((40, 56), (16, 16), "block", (1, 1)),            # last groups 8 x 8 of 16 x 16: whole KV tiles outside
    ((40, 56), (16, 16), "cross", (0, 0)),
    ((33, 47), (8, 8), "block", (1, 1)),              # 2-wave workgroups; one row / seven columns left over
    ((36, 40), (8, 16), "cross", (0, 0)),             # 4-wave workgroups
    ((70, 90), (32, 32), "block", (1, 1)),            # 1024-token boxes: border query tiles wholly outside
    ((5, 20, 28), (2, 8, 8), "block", (1, 1, 1)),     # ragged on all three axes
    ((5, 20, 28), (2, 8, 8), "cross_planes", (0, 0, 0)),
    ((1000,), (128,), "block", (1,)),                 # 1D, last group of 104 tokens
    ((17, 16), (16, 16), "block", (1, 1)),            # the last group is a single grid row
])
def test_group_dims_not_dividing_the_grid(grid, group, pattern, radius):
    """Eq. 2-4 are floor divisions: border groups are the part of their box inside the grid."""
    got, want = small_case(2, 2, grid, group, pattern, radius, q_gain=2.0, seed=94)
    assert_close(got, want, "bf16", f"ragged {grid} {group} {pattern}")


def test_last_token_of_the_tensor_is_the_clamp_target():
    """A ragged grid whose K/V end exactly at the end of their allocation: rows of border boxes past
    the last token must be fetched from inside the tensor."""
    grid, group = (24, 40), (16, 16)
    host = synth.make_qkv(1, 1, 24 * 40, 128, "bf16", 95)
    dev = [to_device(x).clone() for x in host]        # exact-size allocations
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    O = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    torch.cuda.synchronize()
    assert_close(to_f64(O), orc.grat_attention(*host, grid, group, "block", (1, 1), scale), "bf16", "ragged tail")


@pytest.mark.parametrize("pattern,radius", [("block", (1, 1)), ("cross", (0, 0))])
def test_peaked_softmax(pattern, radius):
    """Q scaled by 4: near one-hot weights, the running max keeps moving."""
    got, want = small_case(1, 4, (64, 64), (16, 16), pattern, radius, q_gain=4.0)
    assert_close(got, want, "bf16", f"peaked {pattern}")
    got, want = small_case(1, 2, (64, 64), (16, 16), pattern, radius, q_gain=16.0)
    assert_close(got, want, "bf16", f"very peaked {pattern}")


@pytest.mark.parametrize("N", [1, 63, 64, 65, 256, 1000, 4097])
def test_dense_ragged_lengths(N):
    host = synth.make_qkv(2, 2, N, 128, "bf16", 92, q_gain=2.0)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    O = grat.grat_dense_attention_fwd(*dev, scale)
    torch.cuda.synchronize()
    assert_close(to_f64(O), orc.dense_attention(*host, scale), "bf16", f"dense N={N}")


def test_full_coverage_matches_dense_kernel_and_oracle():
    grid, group = (64, 64), (16, 16)
    host = synth.make_qkv(1, 2, 4096, 128, "bf16", 93)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, "block", (3, 3))
    Og = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    Od = grat.grat_dense_attention_fwd(*dev, scale)
    torch.cuda.synchronize()
    want = orc.dense_attention(*host, scale)
    assert_close(to_f64(Og), want, "bf16", "grouped, full coverage")
    assert_close(to_f64(Od), want, "bf16", "dense kernel")


def test_constant_v_passes_through():
    grid, group = (64, 64), (16, 16)
    Q, K, _ = synth.make_qkv(1, 2, 4096, 128, "bf16", 94, q_gain=3.0)
    row = synth.f32_to_bf16_bits(np.linspace(-2, 3, 128, dtype=np.float32))
    V = np.broadcast_to(row, Q.shape).copy()
    dev = [to_device(x) for x in (Q, K, V)]
    count, index = grat.grat_build_block_lists(grid, group, "cross")
    O = grat.grat_attention_fwd(*dev, 0.1, grid, group, count, index)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_f64(O), orc.decode_bf16(V), rtol=2 ** -7, atol=1e-6)


def test_token_major_strides_and_rerun_is_bit_identical():
    grid, group = (32, 48), (8, 16)
    host = synth.make_qkv(2, 3, 32 * 48, 128, "bf16", 95)
    scale = 1.0 / math.sqrt(128)
    want = orc.grat_attention(*host, grid, group, "block", (1, 1), scale)
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    dev = [to_device(np.ascontiguousarray(x.transpose(0, 2, 1, 3))).permute(0, 2, 1, 3) for x in host]
    out1 = torch.zeros((2, 32 * 48, 3, 128), dtype=torch.bfloat16, device="cuda").permute(0, 2, 1, 3)
    out2 = torch.zeros_like(out1)
    grat.grat_attention_fwd(*dev, scale, grid, group, count, index, out=out1)
    grat.grat_attention_fwd(*dev, scale, grid, group, count, index, out=out2)
    torch.cuda.synchronize()
    assert_close(to_f64(out1), want, "bf16", "token-major")
    assert torch.equal(out1, out2)


def test_caller_supplied_lists():
    """Lists are data: a hand-made list (every group attends group 0 and itself) is honoured."""
    grid, group = (32, 32), (8, 8)
    G = 16
    index = np.full((G, 3), -1, dtype=np.int32)
    count = np.empty(G, dtype=np.int32)
    for g in range(G):
        ids = sorted({0, g})
        count[g] = len(ids)
        index[g, :len(ids)] = ids
    host = synth.make_qkv(1, 2, 1024, 128, "bf16", 96)
    dev = [to_device(x) for x in host]
    O = grat.grat_attention_fwd(*dev, 0.09, grid, group, torch.from_numpy(count).cuda(),
                                torch.from_numpy(index).cuda())
    torch.cuda.synchronize()
    # expected: oracle attention under the mask those lists expand to
    gid = (np.arange(1024) // 32 // 8) * 4 + (np.arange(1024) % 32) // 8
    mask = (gid[None, :] == gid[:, None]) | (gid[None, :] == 0)
    want = np.stack([orc.masked_attention(host[0][0, h], host[1][0, h], host[2][0, h], mask, 0.09)
                     for h in range(2)])[None]
    assert_close(to_f64(O), want, "bf16", "hand-made lists")


# ---- the largest sizes the entry points accept --------------------------------------------------
def test_longest_list_8192_groups():
    """max_kv = 8192 (the limit): a 1D sequence of 8192 groups of 64 tokens, every group listed."""
    grid, group = (8192 * 64,), (64,)
    host = synth.make_qkv(1, 1, grid[0], 128, "bf16", 96, threads=8)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, "dense")
    assert index.shape == (8192, 8192) and int(count.min()) == 8192
    O = grat.grat_attention_fwd(*dev, scale, grid, group, count, index)
    torch.cuda.synchronize()
    samples = synth.sample_rows(2012, 48, 1, 1, grid[0])
    samples[:2, 2] = [0, grid[0] - 1]
    want = orc.dense_attention_rows(*host, samples, scale)
    print(assert_close(gather_rows(O, samples), want, "bf16", "8192-entry lists"))


def test_largest_group_4096_tokens():
    """4096 tokens per group (the limit of the in-LDS offset table): 16 query tiles per group."""
    got, want = small_case(1, 2, (128, 64), (64, 64), "block", (1, 0), seed=97)
    assert_close(got, want, "bf16", "4096-token groups")


def test_out_of_range_list_entries_are_forced_into_range():
    """A caller-made list that breaks the contract (count beyond the row, entries outside [0, G)) is
    read as the list with its count and entries forced into range: every access stays inside the
    tensors and the result is that of the repaired list."""
    grid, group = (64, 64), (16, 16)
    host = synth.make_qkv(1, 2, 4096, 128, "bf16", 93)
    dev = [to_device(x) for x in host]
    scale = 1.0 / math.sqrt(128)
    count, index = grat.grat_build_block_lists(grid, group, "block", (1, 1))
    G, max_kv = index.shape
    bad_c, bad_i = count.clone(), index.clone()
    bad_c[5] = max_kv + 7                 # interior group: its row is full, so the forced count reads the same 9 entries
    bad_i[0, 1] = G + 100                 # -> G - 1
    bad_i[3, 0] = -12                     # -> 0
    fix_c, fix_i = count.clone(), index.clone()
    fix_i[0, 1] = G - 1
    fix_i[3, 0] = 0
    assert grat.grat_validate_block_lists(grid, group, bad_c, bad_i).item() == 3
    assert grat.grat_validate_block_lists(grid, group, fix_c, fix_i).item() == 0
    a = grat.grat_attention_fwd(*dev, scale, grid, group, bad_c, bad_i)
    b = grat.grat_attention_fwd(*dev, scale, grid, group, fix_c, fix_i)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
