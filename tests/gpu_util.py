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
    return max_abs, rel_l2


def gather_rows(O: torch.Tensor, samples: np.ndarray) -> np.ndarray:
    s = torch.from_numpy(samples).to(O.device)
    return to_f64(O[s[:, 0], s[:, 1], s[:, 2]])
