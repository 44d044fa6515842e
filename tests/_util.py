"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np
import torch

import synth_inputs as si

# Tolerances of the bf16 path against the float64 oracle: max |diff| and relative L2 error.
BF16_MAX_ABS = 2e-2
BF16_REL_L2 = 5e-3


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def errors(got: np.ndarray, want: np.ndarray):
    diff = got - want
    return float(np.abs(diff).max()), float(np.linalg.norm(diff.ravel()) / max(np.linalg.norm(want.ravel()), 1e-300))


def assert_close_bf16(got: np.ndarray, want: np.ndarray, what: str = ""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, rel_l2 = errors(got, want)
    assert max_abs <= BF16_MAX_ABS and rel_l2 <= BF16_REL_L2, f"{what}: max-abs {max_abs:.3e}, rel-L2 {rel_l2:.3e}"
    return max_abs, rel_l2


def gather_rows(out: torch.Tensor, rows: np.ndarray) -> np.ndarray:
    """out[b, n, head, :] for rows[i] = (b, head, n), as float64."""
    r = torch.from_numpy(rows)
    return to_np64(out[r[:, 0].to(out.device), r[:, 2].to(out.device), r[:, 1].to(out.device)])


def oracle_inputs(q, k, v):
    return tuple(si.as_oracle_array(t) for t in (q, k, v))
