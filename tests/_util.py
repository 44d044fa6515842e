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


# The two stated bounds are pooled over everything compared; at the benchmark shapes outputs are ~0.05, so the absolute bound
# cannot fail there and one bad row would drown in the pooled norm.  Two sharper checks therefore ride along (they tighten,
# never replace, the stated tolerance): every compared row (the last axis: one query's head_dim outputs) on its own, and the
# largest error relative to the largest reference value.  bf16 rounding of the probabilities and of the output gives ~2.5e-3
# per row and ~0.3 % of the largest value; the bounds leave a factor of about 6.
BF16_ROW_REL_L2 = 1.5e-2
BF16_MAX_ABS_OF_MAX = 2e-2


def assert_close_bf16(got: np.ndarray, want: np.ndarray, what: str = ""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    max_abs, rel_l2 = errors(got, want)
    assert max_abs <= BF16_MAX_ABS and rel_l2 <= BF16_REL_L2, f"{what}: max-abs {max_abs:.3e}, rel-L2 {rel_l2:.3e}"
    g2, w2 = got.reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    row_err = np.linalg.norm(g2 - w2, axis=1) / np.maximum(np.linalg.norm(w2, axis=1), 1e-300)
    worst = int(row_err.argmax())
    assert row_err[worst] <= BF16_ROW_REL_L2, f"{what}: row {worst} rel-L2 {row_err[worst]:.3e}"
    peak = float(np.abs(want).max())
    assert max_abs <= BF16_MAX_ABS_OF_MAX * peak, f"{what}: max-abs {max_abs:.3e} is {max_abs / peak:.2%} of max |reference| {peak:.3e}"
    return max_abs, rel_l2


def gather_rows(out: torch.Tensor, rows: np.ndarray) -> np.ndarray:
    """out[b, n, head, :] for rows[i] = (b, head, n), as float64."""
    r = torch.from_numpy(rows)
    return to_np64(out[r[:, 0].to(out.device), r[:, 2].to(out.device), r[:, 1].to(out.device)])


def oracle_inputs(q, k, v):
    return tuple(si.as_oracle_array(t) for t in (q, k, v))
