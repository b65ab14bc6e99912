"""Helpers shared by the GPU parity tests (host <-> device plumbing and the error gate)."""
import numpy as np
import torch

MAX_ABS = 2e-2     # tolerance on fp16 layer outputs stated for this build (max abs error)
MEAN_ABS = 2e-3    # (mean abs error)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def gate(got, want, what="", max_abs=MAX_ABS, mean_abs=MEAN_ABS):
    """got: fp16 array from the GPU; want: float64 from the oracle (same shape, no NaN)."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite GPU output"
    err = np.abs(got - want)
    mx, mn = float(err.max()) if err.size else 0.0, float(err.mean()) if err.size else 0.0
    assert mx <= max_abs and mn <= mean_abs, f"{what}: max abs {mx:.3e} (<= {max_abs}), mean abs {mn:.3e} (<= {mean_abs})"
    return mx, mn
