"""Helpers for the GPU parity tests: host<->device marshalling and error norms."""
import numpy as np
import torch

from oracle import grat_oracle as orc

BF16_MAX_ABS, BF16_REL_L2 = 3e-2, 1e-2     # tolerance stated for bf16 inputs
F32_TOL = 1e-4                             # fp32: both max-abs and relative L2
# fp16 has 3 more significand bits than bf16 and the same arithmetic around it (fp32 scores and
# accumulators, weights and output rounded once to the element type): an eighth of the bf16 bar
F16_MAX_ABS, F16_REL_L2 = BF16_MAX_ABS / 8, BF16_REL_L2 / 8


def to_device(x: np.ndarray) -> torch.Tensor:
    """float32 / float16 array -> tensor of that type; uint16 bf16 bit patterns -> bf16 tensor (same bits)."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(x).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def errors(got: np.ndarray, want: np.ndarray):
    diff = got.astype(np.float64) - want
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / np.linalg.norm(want))


# Every single output row also has to be right on its own: a global norm over 10^5 rows would hide a
# few wrong rows.  Per row the relative L2 error may be twice the bar of the whole tensor for 16-bit
# outputs (a row of 128 roundings scatters around the tensor-wide rms) and equals it for fp32.
ROW_REL_L2 = {"bf16": 2e-2, "f16": 2.5e-3, "f32": 1e-4}


def row_errors(got: np.ndarray, want: np.ndarray):
    """worst relative L2 error of a row (last axis) and its index"""
    g = got.astype(np.float64).reshape(-1, got.shape[-1])
    w = want.reshape(-1, want.shape[-1])
    num = np.linalg.norm(g - w, axis=1)
    den = np.maximum(np.linalg.norm(w, axis=1), 1e-30)
    rel = num / den
    worst = int(np.argmax(rel))
    return float(rel[worst]), worst


def assert_close(got, want, dtype: str, what: str = ""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, rel_l2 = errors(got, want)
    if dtype == "bf16":
        ok = max_abs <= BF16_MAX_ABS and rel_l2 <= BF16_REL_L2
    elif dtype == "f16":
        ok = max_abs <= F16_MAX_ABS and rel_l2 <= F16_REL_L2
    else:
        ok = max_abs <= F32_TOL and rel_l2 <= F32_TOL
    assert ok, f"{what}: max_abs {max_abs:.3e} rel_l2 {rel_l2:.3e} ({dtype})"
    row_rel, row = row_errors(got, want)
    assert row_rel <= ROW_REL_L2[dtype], f"{what}: row {row} (flattened) rel_l2 {row_rel:.3e} ({dtype})"
    return max_abs, rel_l2, row_rel


def nan_like(t: torch.Tensor) -> torch.Tensor:
    """An output buffer in which every element a kernel fails to store stays visible."""
    return torch.full_like(t, float("nan"))


def assert_all_written(O: torch.Tensor, what: str = ""):
    assert bool(torch.isfinite(O).all()), f"{what}: rows of the output were never stored"


def gather_rows(O: torch.Tensor, samples: np.ndarray) -> np.ndarray:
    s = torch.from_numpy(samples).to(O.device)
    return to_f64(O[s[:, 0], s[:, 1], s[:, 2]])
