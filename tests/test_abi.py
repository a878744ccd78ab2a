"""The C-ABI library loads, exports every symbol the header declares, and validates its
arguments on the host (no launch happens on these paths, so no GPU is needed)."""
import ctypes
import glob
import os
import re

import pytest

import paper_2505_14687_amd as grat
from paper_2505_14687_amd import grat as binding
from paper_2505_14687_amd.build import LIB_PATH, ROOT


def declared_symbols():
    names = set()
    for header in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
        names |= set(re.findall(r"\b(grat_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    L = ctypes.CDLL(LIB_PATH)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings():
    L = grat.lib()
    seen = {L.grat_status_string(i) for i in range(8)}
    assert len(seen) == 8 and all(s for s in seen)
    assert L.grat_status_string(0) == b"ok"


def test_block_list_shape_closed_forms():
    f = grat.grat_block_list_shape
    assert f((32, 32), (8, 8), "block", (1, 1)) == (16, 9)
    assert f((128, 128), (16, 16), "block", (2, 2)) == (64, 25)
    assert f((128, 128), (16, 16), "block", (20, 0)) == (64, 8)
    assert f((512, 512), (16, 16), "cross") == (1024, 63)
    assert f((30, 48, 80), (2, 8, 8), "block", (1, 1, 1)) == (900, 27)
    assert f((30, 48, 80), (2, 8, 8), "cross") == (900, 29)
    assert f((30, 48, 80), (2, 8, 8), "cross_planes") == (900, 270)
    assert f((30, 48, 80), (2, 8, 8), "dense") == (900, 900)
    assert f((130, 70), (16, 16), "cross") == (9 * 5, 13)      # ragged last groups count
    assert f((100,), (10,), "cross_planes") == (10, 1)


def status_of(fn):
    with pytest.raises(grat.GratError) as e:
        fn()
    return e.value.status


def test_shape_argument_errors():
    f = grat.grat_block_list_shape
    assert status_of(lambda: f((32, 32, 32, 32), (8, 8, 8, 8), "cross")) == 2
    assert status_of(lambda: f((32, 0), (8, 8), "cross")) == 2
    assert status_of(lambda: f((32, 32), (8, -8), "cross")) == 2
    assert status_of(lambda: f((32, 32), (8, 8), "block", (1, -1))) == 2
    assert status_of(lambda: f((32, 32), (8, 8), "block", None)) == 1
    assert status_of(lambda: f((32, 32), (8, 8), 9)) == 4


def test_attention_argument_errors_return_before_any_launch():
    L = grat.lib()
    i32x2 = ctypes.c_int32 * 2
    fake = 0x1000   # never dereferenced: every call below fails validation first
    def call(Q=fake, K=fake, V=fake, O=fake, dtype=0, batch=1, heads=2, d=128, sb=0, sh=4096 * 128,
             sn=128, scale=0.1, grid=(64, 64), group=(16, 16), cnt=fake, idx=fake, max_kv=9):
        return L.grat_attention_fwd(Q, K, V, O, dtype, batch, heads, d, sb, sh, sn, scale, 2,
                                    i32x2(*grid), i32x2(*group), cnt, idx, max_kv, None)
    assert call(Q=None) == 1 and call(O=None) == 1 and call(cnt=None) == 1
    assert call(batch=0) == 2 and call(scale=0.0) == 2 and call(scale=float("nan")) == 2
    assert call(sn=64) == 2
    assert call(grid=(2100, 64), group=(2048, 2)) == 6   # clipped border groups: box coordinates beyond the packing
    assert call(d=96) == 6                       # the 16-bit path has head_dim 128 or 64
    assert call(dtype=1, d=96) == 6
    assert call(dtype=2, d=32) == 6
    assert call(dtype=5) == 6
    assert call(group=(4, 4)) == 6               # 16-token groups on the bf16 path
    assert call(sn=132) == 6                     # rows not 16-byte aligned
    assert call(Q=fake + 2) == 6
    assert call(max_kv=0) == 5
    assert call(max_kv=100000) == 6
    assert call(sn=1 << 24) == 6                 # token stride beyond 2^24 elements
    assert call(sn=1 << 23) == 6                 # bf16: one group's rows span 4 GiB or more
    assert call(grid=(1 << 16, 1 << 16), group=(16, 16)) == 2   # 2^32 tokens
    d = L.grat_dense_attention_fwd
    assert d(fake, fake, fake, None, 0, 1, 1, 100, 128, 0, 0, 128, 0.1, None) == 1
    assert d(fake, fake, fake, fake, 0, 1, 1, 0, 128, 0, 0, 128, 0.1, None) == 2
    assert d(fake, fake, fake, fake, 0, 1, 1, 100, 32, 0, 0, 128, 0.1, None) == 6
    b = L.grat_build_block_lists
    assert b(2, i32x2(64, 64), i32x2(16, 16), 0, i32x2(1, 1), fake, fake, 8, None) == 5
    assert b(2, i32x2(64, 64), i32x2(16, 16), 0, i32x2(1, 1), None, fake, 9, None) == 1
    assert b(2, i32x2(64, 64), i32x2(16, 16), 7, i32x2(1, 1), fake, fake, 9, None) == 4


def test_binding_rejects_host_tensors():
    import torch
    x = torch.zeros(1, 1, 64, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        grat.grat_dense_attention_fwd(x, x, x, 0.1, out=torch.zeros_like(x))


def test_binding_checks_sequence_length_and_lists():
    """The binding refuses what would make the kernels read past a tensor or misread a list: a
    sequence that is not prod(grid) (+ n_global) rows long, lists that are not int32 / contiguous /
    [G] and [G, max_kv].  (Host tensors: every one of these checks comes before the device check.)"""
    import torch
    grid, group = (64, 64), (16, 16)
    x = torch.zeros(1, 2, 4096, 128, dtype=torch.bfloat16)
    cnt = torch.zeros(16, dtype=torch.int32)
    idx = torch.zeros(16, 9, dtype=torch.int32)
    def plain(q=x, c=cnt, i=idx, g=grid):
        return grat.grat_attention_fwd(q, q, q, 0.1, g, group, c, i, out=torch.zeros_like(q))
    with pytest.raises(ValueError, match="sequence length"):
        plain(g=(64, 128))                                   # grid larger than the tensor
    with pytest.raises(ValueError, match="sequence length"):
        plain(q=torch.zeros(1, 2, 4100, 128, dtype=torch.bfloat16))
    with pytest.raises(ValueError, match="int32"):
        plain(c=cnt.to(torch.int64))
    with pytest.raises(ValueError, match="int32"):
        plain(i=idx.to(torch.int64))
    with pytest.raises(ValueError, match="contiguous"):
        plain(i=torch.zeros(9, 16, dtype=torch.int32).t())
    with pytest.raises(ValueError, match="kv_count"):
        plain(c=torch.zeros(15, dtype=torch.int32))
    with pytest.raises(ValueError, match="kv_index"):
        plain(i=torch.zeros(15, 9, dtype=torch.int32))
    with pytest.raises(ValueError, match="kv_index"):
        plain(i=torch.zeros(16 * 9, dtype=torch.int32))
    with pytest.raises(ValueError, match="device memory"):
        plain()                                              # all shapes right: the host tensors themselves
    # joint and packed entry points: n_global counts
    xj = torch.zeros(1, 2, 4096 + 100, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="sequence length"):
        grat.grat_attention_global_fwd(xj, xj, xj, 0.1, 99, True, grid, group, cnt, idx, out=torch.zeros_like(xj))
    with pytest.raises(ValueError, match="device memory"):
        grat.grat_attention_global_fwd(xj, xj, xj, 0.1, 100, True, grid, group, cnt, idx, out=torch.zeros_like(xj))
    qkv = torch.zeros(1, 4096, 3, 2, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="sequence length"):
        grat.grat_attention_packed_fwd(qkv, 0.1, (64, 60), group, cnt, idx)
    with pytest.raises(ValueError, match="int32"):
        grat.grat_attention_packed_fwd(qkv, 0.1, grid, group, cnt.to(torch.int16), idx)
    with pytest.raises(ValueError, match="device memory"):
        grat.grat_attention_packed_fwd(qkv, 0.1, grid, group, cnt, idx)


def test_validate_block_lists_argument_errors():
    L = grat.lib()
    i32x2 = ctypes.c_int32 * 2
    fake = 0x1000
    def call(cnt=fake, idx=fake, status=fake, max_kv=9, grid=(64, 64), group=(16, 16), ndim=2):
        return L.grat_validate_block_lists(ndim, i32x2(*grid), i32x2(*group), cnt, idx, max_kv, status, None)
    assert call(cnt=None) == 1 and call(idx=None) == 1 and call(status=None) == 1
    assert call(ndim=4) == 2
    assert call(grid=(64, 0)) == 2
    assert call(max_kv=0) == 5


def test_joint_sequence_argument_errors():
    L = grat.lib()
    i32x2 = ctypes.c_int32 * 2
    fake = 0x1000
    def call(dtype=0, n_global=512, sn=128, grid=(64, 64)):
        return L.grat_attention_global_fwd(fake, fake, fake, fake, dtype, 1, 2, 128, 0, (4096 + 512) * 128, sn,
                                           0.1, n_global, 1, 2, i32x2(*grid), i32x2(16, 16), fake, fake, 9, None)
    assert call(n_global=-1) == 2
    assert call(dtype=1) == 6                      # prompt tokens on the fp32 path
    assert call(grid=(64, 60)) == 3
    assert call(sn=1 << 24) == 6


def test_packed_entry_argument_errors():
    L = grat.lib()
    i32x2 = ctypes.c_int32 * 2
    fake = 0x1000
    def call(QKV=fake, O=fake, dtype=0, batch=1, heads=2, d=128, n_global=0, grid=(64, 64), group=(16, 16),
             cnt=fake, max_kv=9):
        return L.grat_attention_packed_fwd(QKV, O, dtype, batch, heads, d, 0.1, n_global, 1, 2, i32x2(*grid),
                                           i32x2(*group), cnt, fake, max_kv, None)
    assert call(QKV=None) == 1 and call(O=None) == 1 and call(cnt=None) == 1
    assert call(heads=0) == 2 and call(n_global=-1) == 2
    assert call(dtype=3) == 6 and call(d=96) == 6
    assert call(dtype=1, n_global=8) == 6
    assert call(grid=(64, 60), n_global=8) == 3    # prompt tokens: whole groups only
    assert call(QKV=fake + 4) == 6                 # not 16-byte aligned
    assert call(max_kv=0) == 5


def test_probe_argument_errors():
    L = grat.lib()
    fake = 0x1000
    assert L.grat_probe_mfma(0, 2, None, 256, 16, None) == 1
    assert L.grat_probe_mfma(0, 2, fake, 0, 16, None) == 2 and L.grat_probe_mfma(0, 2, fake, 65537, 16, None) == 2
    assert L.grat_probe_mfma(0, 2, fake, 256, 0, None) == 2 and L.grat_probe_mfma(2, 2, fake, 256, 4097, None) == 2
    assert L.grat_probe_mfma(0, 3, fake, 256, 16, None) == 2 and L.grat_probe_mfma(0, -1, fake, 256, 16, None) == 2
    assert L.grat_probe_mfma(1, 0, fake, 256, 16, None) == 6


def test_bench_names_the_launched_instantiation():
    """bench.py restates the library's launch rules to name the kernel in its roofline block (host only)."""
    import numpy as np
    import bench
    from paper_2505_14687_amd import synth
    names = {}
    for wl, label in (("img8192", "B3"), ("img1024", "X"), ("video", "B3"), ("img8192_g8", "B3"), ("img8192_g8", "X")):
        w = synth.WORKLOADS[wl]
        pattern, radius = w.patterns[label]
        names[(wl, label)] = bench.kernel_name(w, int(np.prod(w.group)), 0, pattern, radius)
    assert names[("img8192", "B3")] == "grat::attn_mfma_kernel<8, 64, 0, false, 128>"
    assert names[("img1024", "X")] == "grat::attn_mfma_kernel<4, 64, 0, false, 128>"
    assert names[("video", "B3")] == "grat::attn_mfma_kernel<4, 64, 0, false, 128>"
    assert names[("img8192_g8", "B3")] == "grat::attn_mfma_kernel<2, 32, 0, false, 128>"
    assert names[("img8192_g8", "X")] == "grat::attn_mfma_kernel<2, 64, 0, false, 128>"
