"""The MFMA-only probe of libgrat (grat_probe.h): binding and the checksum its sink must show.
A measurement aid for benchmarks, not part of the attention path."""
from __future__ import annotations

import numpy as np
import torch

from .grat import DTYPES, GRAT_OK, GratError, _stream_ptr, lib

PROBE_DATA = {"ones": 0, "small_ints": 1, "normal_like": 2}


def grat_probe_mfma(dtype, data, blocks: int, iters: int, sink=None, stream=None):
    """One launch of the MFMA-only loop (grat_probe.h) on operands of kind `data` ("ones",
    "small_ints", "normal_like" or 0..2); returns the sink tensor [blocks * 256] int64."""
    if sink is None:
        sink = torch.empty(int(blocks) * 256, dtype=torch.int64, device="cuda")
    if sink.dtype != torch.int64 or not sink.is_contiguous() or sink.numel() < int(blocks) * 256:
        raise ValueError("sink: contiguous int64, at least blocks * 256 elements")
    kind = PROBE_DATA[data] if isinstance(data, str) else int(data)
    st = lib().grat_probe_mfma(DTYPES[dtype], kind, sink.data_ptr(), int(blocks), int(iters), _stream_ptr(stream))
    if st != GRAT_OK:
        raise GratError(st, "grat_probe_mfma")
    return sink


def probe_wave_sum(data, iters: int) -> int:
    """What the 64 sink values of one wave add up to (grat_probe.h)."""
    kind = PROBE_DATA[data] if isinstance(data, str) else int(data)
    if kind == 0:
        return 4 * 2 * 32 * 32 * 16 * int(iters)
    l = np.arange(64)[:, None]
    e = np.arange(8)[None, :]

    def matrix(values):   # [lane, e] -> M[l % 32][8 (l // 32) + e]
        M = np.zeros((32, 16), dtype=np.int64)
        for lane in range(64):
            M[lane % 32, 8 * (lane // 32):8 * (lane // 32) + 8] = values[lane]
        return M

    total = 0
    for v in ((0, 1, 2, 3) if kind == 1 else (3,)):
        A = matrix(((37 + 2 * v) * l + 11 * e + 5 + 3 * v) % 9 - 4)
        B = matrix(((53 + 2 * v) * l + 17 * e + 2 + 3 * v) % 9 - 4).T
        total += 2 * int((A @ B).sum())
    return total * int(iters)
