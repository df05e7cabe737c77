"""Helpers for the GPU parity tests: numpy <-> device tensors and error metrics."""
import numpy as np
import torch

from paper_2503_08640_amd import synth

MAX_ABS_TOL = 2e-2    # bf16 inputs vs the fp64 oracle
MEAN_ABS_TOL = 2e-3


def to_dev(x: np.ndarray) -> torch.Tensor:
    """fp32 array or bf16 bit patterns -> device tensor of the same values."""
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def errors(got: np.ndarray, want: np.ndarray):
    d = np.abs(got - want)
    return float(d.max()), float(d.mean())


def assert_close(got, want, what="", max_tol=MAX_ABS_TOL, mean_tol=MEAN_ABS_TOL):
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    mx, mean = errors(got, want)
    print(f"[parity] {what}: max-abs {mx:.3e} mean-abs {mean:.3e}", flush=True)
    assert mx <= max_tol and mean <= mean_tol, f"{what}: max-abs {mx:.3e} mean-abs {mean:.3e}"


def pool_f64(pc):
    return synth.as_f64(pc.q), synth.as_f64(pc.k), synth.as_f64(pc.v)
