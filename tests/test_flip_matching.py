"""The acceptance rule of the GPU parity tests where gradients are not unique (a ReLU input at
zero, tied pooled values), exercised on the CPU with results fabricated from the oracle: a
result that took the other branch of a listed near decision is accepted at the full tolerance,
the same result with a small error anywhere else is refused."""
import numpy as np
import pytest

from paper_2102_06280_amd import inputs
from gpu_util import GradientResolver, NEAR_SCALE, involved_workers, match_gradients, match_round, _row_ok

DIMS = [12, 10, 5]
N, BATCH = 4, 6
D = sum(DIMS[l + 1] * (DIMS[l] + 1) for l in range(2))
LD = 192


def _setup(orc):
    """Four workers of a small network; workers 1 and 2 each have one hidden unit whose input is
    within fp32 rounding of zero for one sample (the bias is set to cancel the rest)."""
    g = np.random.default_rng(601)
    params = np.zeros((N, LD), np.float32)
    params[:, :D] = g.standard_normal((N, D)) * 0.4
    x = g.standard_normal((N, BATCH, DIMS[0])).astype(np.float32)
    y = g.integers(0, DIMS[-1], (N, BATCH)).astype(np.int32)
    bias0 = DIMS[1] * DIMS[0]
    for worker, sample, unit, sign in ((1, 2, 3, +1), (2, 4, 7, -1)):
        W = params[worker, :bias0].reshape(DIMS[1], DIMS[0]).astype(np.float64)
        params[worker, bias0 + unit] = np.float32(-(W[unit] @ x[worker, sample].astype(np.float64)))
        z = W[unit] @ x[worker, sample].astype(np.float64) + float(params[worker, bias0 + unit])
        if np.sign(z) != sign:           # put the tiny remainder on the wanted side
            params[worker, bias0 + unit] = np.nextafter(params[worker, bias0 + unit], np.float32(sign * np.inf))
    kind, od = orc.model_desc({"kind": "mlp", "dims": DIMS})
    return kind, od, params, x, y


def _noise(a, g, rel=2e-7):
    return (a.astype(np.float64) * (1 + rel * g.standard_normal(a.shape))).astype(np.float32)


def _grad_ok(got, want):
    off = 0
    for l in range(2):
        for n in (DIMS[l + 1] * DIMS[l], DIMS[l + 1]):
            w = want[off:off + n].astype(np.float64)
            if np.linalg.norm(got[off:off + n] - w) > 2e-5 * np.linalg.norm(w):
                return False
            off += n
    return True


def test_near_decisions_are_listed_and_resolved_for_gradients(orc):
    kind, od, params, x, y = _setup(orc)
    res = GradientResolver(orc, kind, od, D, params, x, y, threads=2)
    assert [len(v) for v in res.near] == [0, 1, 1, 0]
    assert res.near[1][0].key() == (16, 2, 3, 0) and res.near[2][0].key() == (16, 4, 7, 1)
    assert all(f.gap < NEAR_SCALE for v in res.near for f in v)
    g = np.random.default_rng(603)
    # worker 1 took the other branch, worker 2 (also near a tie) the oracle's
    got = res.base.copy()
    got[1] = res.flipped(1, res.near[1])
    assert not _grad_ok(got[1, :D], res.base[1, :D])          # the flip is far outside the tolerance
    got = _noise(got, g)
    final = match_gradients(res, got, _grad_ok, D, what="fabricated")
    assert [len(res.resolved.get(j, [])) for j in range(N)] == [0, 1, 0, 0]
    assert np.array_equal(final[2], res.base[2])


def test_error_outside_the_reach_of_a_flip_is_refused(orc):
    kind, od, params, x, y = _setup(orc)
    g = np.random.default_rng(605)
    # worker 1 flipped AND its output-layer bias gradient (which the flip also moves, but in a
    # fixed direction) off by 1e-4 relative; worker 0, with no near decision at all, off as well
    for worker, with_flip in ((1, True), (1, False), (0, False)):
        res = GradientResolver(orc, kind, od, D, params, x, y, threads=2)
        got = res.base.copy()
        if with_flip:
            got[worker] = res.flipped(worker, res.near[worker])
        got = _noise(got, g)
        got[worker, D - DIMS[2]:D] *= np.float32(1 + 1e-4)
        with pytest.raises(AssertionError):
            match_gradients(res, got, _grad_ok, D, what="fabricated")


@pytest.mark.parametrize("order", [0, 1], ids=["cta", "atc"])
def test_round_resolution_uses_one_assignment_for_all_rows(orc, order):
    kind, od, params, x, y = _setup(orc)
    rowptr, colidx = inputs.graph_ring(N)
    t = np.array([0.3, 0.1, 0.05, 0.5], np.float32)    # worker 2 answers first: both neighbours wait for it
    b = np.array([0, 1, 0, 1], np.int32)
    mask, p, _ = orc.select(rowptr, colidx, t, b)
    lr = 0.05
    g = np.random.default_rng(607)

    def fresh():
        res = GradientResolver(orc, kind, od, D, params, x, y, threads=2)
        round_fn = lambda grad: orc.round_(rowptr, colidx, mask, p, params, grad, lr, order, d=D)
        inv = involved_workers(order, lr, rowptr, colidx, mask, lambda: orc.weights(rowptr, colidx, mask, p))
        return res, round_fn, inv

    res, round_fn, inv = fresh()
    grad = res.base.copy()
    grad[2] = res.flipped(2, res.near[2])                      # worker 2 took the other branch
    got = _noise(round_fn(grad), g, rel=1e-7)
    base_rows_off = [i for i in range(N) if not _row_ok(got[i, :D], round_fn(res.base)[i, :D])]
    assert 2 in base_rows_off and (order == 0) == (base_rows_off == [2])   # local step first: neighbours inherit it
    want = match_round(res, got, round_fn, inv, D, what="fabricated")
    assert [len(res.resolved.get(j, [])) for j in range(N)] == [0, 0, 1, 0]
    assert all(_row_ok(got[i, :D], want[i, :D]) for i in range(N))

    # the same result with one more error on a row that no flip explains
    res, round_fn, inv = fresh()
    bad = got.copy()
    bad[0, 5] += 1e-3
    with pytest.raises(AssertionError):
        match_round(res, bad, round_fn, inv, D, what="fabricated")
    # and with an error in a part of worker 2's row that its flip does not reach (output-layer weights
    # move under the flip, so scale them instead of shifting along the flip direction)
    res, round_fn, inv = fresh()
    bad = got.copy()
    bad[2, D - 30:D - 25] += 5e-4
    with pytest.raises(AssertionError):
        match_round(res, bad, round_fn, inv, D, what="fabricated")
