"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# The gradients are discontinuous where a ReLU input is zero or two pooled values tie: both
# branches are valid subgradients, and fp32 accumulation in another order may land on the other
# side than the oracle's fp64.  The oracle lists every decision of a worker's gradient that lies
# within NEAR_SCALE rounding units of turning (one unit = 2^-24 times the sum of the absolute
# products of the pre-activation; a sequential fp32 sum is off by about half a unit in the root
# mean square) and can evaluate the gradient with any of them
# taken the other way.  A result that misses the oracle's default evaluation must equal, to
# the full tolerance, the oracle's evaluation for SOME assignment of those listed decisions;
# which one is found by least squares over the listed decisions' individual effects and then
# confirmed by an exact re-evaluation.  No tolerance is widened anywhere.
NEAR_SCALE = 8.0


def _row_ok(got, want, tol=1e-5):
    g, w = got.astype(np.float64), want.astype(np.float64)
    diff = g - w
    ref = np.linalg.norm(w)
    return (np.linalg.norm(diff) <= (tol * ref if ref > 0 else tol)
            and np.abs(diff).max(initial=0.0) <= tol * max(1.0, np.abs(w).max(initial=0.0)))


def _choose_flips(residual, columns, what):
    """residual ~ sum_f c_f columns[f] with c_f in {0, 1}: least squares on the support of the
    columns, rounded; a coefficient that is neither 0 nor 1 means the residual is not made of
    decision flips."""
    A = np.stack(columns, axis=1).astype(np.float64)
    support = np.flatnonzero(np.abs(A).sum(axis=1) > 0)
    if support.size == 0:
        return np.zeros(len(columns), dtype=bool)
    c, *_ = np.linalg.lstsq(A[support], residual[support].astype(np.float64), rcond=None)
    chosen = c > 0.5
    # columns without any effect on this row get c = 0 from the minimum-norm solution
    assert np.all(np.abs(c - chosen) < 0.25), f"{what}: flip coefficients {np.round(c, 3)} are not 0/1"
    return chosen


class GradientResolver:
    """Oracle gradients of all workers with their near decisions, and re-evaluation of single
    workers with chosen decisions flipped.  grad holds the current evaluation (default branches
    until a worker has been resolved)."""

    def __init__(self, orc, kind, od, d, params, bx, by, threads=16):
        self.orc, self.kind, self.od, self.d = orc, kind, od, d
        self.params, self.bx, self.by = params, bx, by
        self.threads = threads
        orc.set_threads(threads)
        self.grad, self.loss, self.near = orc.grad_all(kind, od, d, params, bx, by, near_scale=NEAR_SCALE)
        orc.set_threads(1)
        self.base = self.grad.copy()
        self.resolved = {}                    # worker -> list of flipped decisions (maybe empty)

    def flipped(self, j, flips):
        g = np.zeros(self.grad.shape[1], np.float32)
        g[:self.d] = self.orc.grad_one(self.kind, self.od, self.d, self.params[j], self.bx[j], self.by[j], flips=flips)
        return g

    def effects(self, workers):
        """[(worker, decision, gradient change of flipping that decision alone)] for the listed
        decisions of `workers`, evaluated in parallel (the oracle releases the interpreter lock)."""
        from concurrent.futures import ThreadPoolExecutor
        jobs = [(j, f) for j in workers for f in self.near[j]]
        with ThreadPoolExecutor(max_workers=self.threads) as ex:
            grads = list(ex.map(lambda jf: self.flipped(jf[0], [jf[1]]), jobs))
        return [(j, f, g.astype(np.float64) - self.base[j]) for (j, f), g in zip(jobs, grads)]

    def resolve(self, workers, chosen_flips):
        for j in workers:
            fl = chosen_flips.get(j, [])
            self.resolved[j] = fl
            if fl:
                self.grad[j] = self.flipped(j, fl)

    def summary(self):
        n_near = sum(len(v) for v in self.near)
        flips = {j: fl for j, fl in self.resolved.items() if fl}
        return (f"{n_near} decisions within {NEAR_SCALE:g} rounding units over {len(self.near)} workers; "
                f"{sum(len(v) for v in flips.values())} taken the other way on workers {sorted(flips)}"
                + "".join(f" [gap {f.gap:.2f} stage {f.stage}]" for fl in flips.values() for f in fl))


def match_gradients(res, got, tol_fn, d, what=""):
    """got [N, ld]: gradients from the library.  Every worker must agree with the oracle's
    evaluation for some assignment of its own near decisions; tol_fn(got_row, want_row) -> bool
    is the full-tolerance comparison of one worker's d values.  Returns the oracle gradients finally compared against."""
    n = got.shape[0]
    for i in range(n):
        if tol_fn(got[i, :d], res.grad[i, :d]):
            continue
        assert res.near[i], f"{what}: worker {i} misses the oracle and has no decision near turning"
        eff = res.effects([i])
        chosen = _choose_flips(got[i, :d].astype(np.float64) - res.base[i, :d], [e[2][:d] for e in eff],
                               f"{what} worker {i}")
        res.resolve([i], {i: [e[1] for e, c in zip(eff, chosen) if c]})
        assert tol_fn(got[i, :d], res.grad[i, :d]), (f"{what}: worker {i} matches no assignment of its "
                                             f"{len(res.near[i])} near decisions")
    return res.grad


def match_round(res, got, round_fn, involved_fn, d, what="", tol=1e-5):
    """got [N, ld]: parameters after one round from the library.  round_fn(grad) -> the oracle's
    round output for a gradient matrix; involved_fn(i) -> [(worker j, factor)] such that row i
    of the output changes by factor * (change of worker j's gradient).  Every row must meet the
    full tolerance against the oracle's round for one common assignment of near decisions:
    each worker's assignment is fixed the first time a row that depends on it is resolved."""
    want = round_fn(res.grad)
    n = got.shape[0]
    for _ in range(n + 1):
        failing = [i for i in range(n) if not _row_ok(got[i, :d], want[i, :d], tol)]
        if not failing:
            return want
        i = failing[0]
        open_workers = [(j, w) for j, w in involved_fn(i) if j not in res.resolved]
        cands = [j for j, _ in open_workers if res.near[j]]
        assert cands, (f"{what}: row {i} misses the oracle (rel L2 "
                       f"{np.linalg.norm(got[i, :d].astype(np.float64) - want[i, :d]) / max(np.linalg.norm(want[i, :d]), 1e-300):.3e})"
                       f" and no open worker it depends on has a decision near turning")
        factor = dict(open_workers)
        eff = res.effects(cands)
        chosen = _choose_flips(got[i, :d].astype(np.float64) - want[i, :d], [factor[j] * dg[:d] for j, _, dg in eff],
                               f"{what} row {i}")
        picks = {}
        for (j, f, _), c in zip(eff, chosen):
            if c:
                picks.setdefault(j, []).append(f)
        res.resolve([j for j, _ in open_workers], picks)
        want = round_fn(res.grad)
        assert _row_ok(got[i, :d], want[i, :d], tol), (
            f"{what}: row {i} matches no assignment of the near decisions of workers {cands} (rel L2 "
            f"{np.linalg.norm(got[i, :d].astype(np.float64) - want[i, :d]) / max(np.linalg.norm(want[i, :d]), 1e-300):.3e})")
    raise AssertionError(f"{what}: rows still failing after every worker was resolved")


def involved_workers(order, lr, rowptr, colidx, mask, weights_fn):
    """involved_fn for match_round.  Average-then-correct: row i depends on its own gradient with
    factor -lr.  Local step first: on its own and its selected neighbours' gradients with factors
    -lr P_ii and -lr P_ij.  weights_fn() -> (edge weights aligned with colidx, self weights)."""
    lr = np.broadcast_to(np.asarray(lr, dtype=np.float64), (rowptr.size - 1,))
    if order == 0:
        return lambda i: [(i, -lr[i])]
    we, ws = weights_fn()

    def fn(i):
        out = [(i, -lr[i] * ws[i])]
        for e in range(rowptr[i], rowptr[i + 1]):
            if mask[e]:
                out.append((int(colidx[e]), -lr[colidx[e]] * we[e]))
        return out
    return fn


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
