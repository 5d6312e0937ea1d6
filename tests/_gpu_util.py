"""Helpers shared by the GPU parity tests: host bits <-> device tensors, error metrics."""
import numpy as np
import torch

MAX_ABS = 2e-2    # bf16 attention output against the fp64 oracle
MEAN_ABS = 2e-3


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def check_close(got: np.ndarray, want: np.ndarray, what=""):
    err = np.abs(got - want)
    assert np.isfinite(got).all(), "%s: non-finite output" % what
    mx, mean = float(err.max()), float(err.mean())
    assert mx <= MAX_ABS and mean <= MEAN_ABS, "%s: max-abs %.3e (limit %.0e), mean-abs %.3e (limit %.0e)" % (
        what, mx, MAX_ABS, mean, MEAN_ABS)
    return mx, mean
