"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# The gradients are discontinuous where a ReLU input is zero or two pooled values tie.  fp32
# accumulation leaves pre-activations of unit scale uncertain by about 1e-6, so a decision
# whose margin (reported by the oracle) is below these bounds may legitimately fall on the
# other side on the GPU; observed flips all had margins below 1.5e-6.  Such a worker is
# compared loosely, every other worker to the full tolerance, and at least three quarters
# of all workers must meet the full tolerance whatever their margins.
AMBIGUOUS_CONV, AMBIGUOUS_FC = 2e-6, 1e-5
AMBIGUOUS_TOL = 1e-3


# Fully connected models with 256-wide layers and inputs of unit scale: pre-activations are
# sums of 256 products of size 0.06, so fp32 leaves them uncertain by a few 1e-7 (observed
# flips: margins 6e-8 and 9e-8; none above).  One flipped unit of one sample moves a row of
# the weight gradient by |delta| |a| / batch, about 1e-5 absolute at batch 1024.
AMBIGUOUS_FC_256 = 5e-7


def ambiguous(margin, fc=AMBIGUOUS_FC):
    margin = np.asarray(margin)
    return (margin[:, 0] < AMBIGUOUS_CONV) | (margin[:, 1] < fc)


def row_tolerances(margin, tol=1e-5, fc=AMBIGUOUS_FC, selection=None):
    """Per-worker tolerance: `tol` where every ReLU / max-pooling decision of the worker's
    gradient is clear, AMBIGUOUS_TOL where the oracle reports a near-tie.  When the local
    step precedes the average (selection = (rowptr, colidx, mask)), a worker also inherits
    the flag of every neighbour it waits for."""
    flag = ambiguous(margin, fc)
    if selection is not None:
        rowptr, colidx, mask = selection
        own = flag.copy()
        for i in range(flag.size):
            row = slice(rowptr[i], rowptr[i + 1])
            flag[i] = own[i] or bool(np.any(own[colidx[row]][mask[row] != 0]))
    return np.where(flag, AMBIGUOUS_TOL, tol)


def assert_mostly_tight(got, want, d, tol=1e-5, frac=0.75, what=""):
    g, w = got[:, :d].astype(np.float64), want[:, :d].astype(np.float64)
    rel = np.linalg.norm(g - w, axis=1) / np.maximum(np.linalg.norm(w, axis=1), 1e-300)
    ok = (rel <= tol).mean()
    assert ok >= frac, f"{what}: only {ok:.0%} of the workers within {tol:g}"
    return rel


def assert_params_close(got: np.ndarray, want: np.ndarray, d=None, tol=1e-5, what=""):
    """Per worker row: ||got - want||_2 <= tol * ||want||_2 (absolute tol when the row is
    zero) and max |got - want| <= tol * max(1, ||want||_inf).  tol may be per row."""
    d = got.shape[1] if d is None else d
    tol = np.broadcast_to(np.asarray(tol, dtype=np.float64), (got.shape[0],))
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
