"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def assert_params_close(got: np.ndarray, want: np.ndarray, d=None, tol=1e-5, what=""):
    """Per worker row: ||got - want||_2 <= tol * ||want||_2 (absolute tol when the row is
    zero) and max |got - want| <= tol * max(1, ||want||_inf)."""
    d = got.shape[1] if d is None else d
    g, w = got[:, :d].astype(np.float64), want[:, :d].astype(np.float64)
    diff = g - w
    l2 = np.linalg.norm(diff, axis=1)
    ref = np.linalg.norm(w, axis=1)
    bound = np.where(ref > 0, tol * ref, tol)
    worst = int(np.argmax(l2 / bound))
    assert np.all(l2 <= bound), f"{what}: row {worst} rel L2 {l2[worst] / max(ref[worst], 1e-300):.3e}"
    amax = np.abs(diff).max(axis=1)
    abound = tol * np.maximum(1.0, np.abs(w).max(axis=1))
    assert np.all(amax <= abound), f"{what}: max abs err {amax.max():.3e}"
