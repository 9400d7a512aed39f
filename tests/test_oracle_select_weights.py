"""Pins for the oracle's selection and Metropolis weights (CPU only).

Each check is something the paper or plain mathematics fixes, computed here without
calling the oracle routine it checks: brute force over subsets, structural invariants of
Assumption 1, degenerate cases of Section 2.2, and a hand-worked example.
"""
import itertools
from fractions import Fraction

import os

import numpy as np
import pytest

from paper_2102_06280_amd import inputs


def small_graphs():
    g = np.random.default_rng(7)
    out = [inputs.graph_ring(5), inputs.graph_ring(8), inputs.graph_complete(5), inputs.graph_complete(7)]
    for n, p in [(6, 0.5), (7, 0.6), (8, 0.5), (8, 0.8)]:
        out.append(inputs.graph_er(n, p, g))
    out.append(inputs.graph_regular(8, 4, g))
    # star: one hub, unequal degrees
    n = 6
    adj = np.zeros((n, n), bool)
    adj[0, 1:] = adj[1:, 0] = True
    out.append(inputs._csr_from_adj(adj))
    return out


def rows(rowptr, colidx):
    for i in range(rowptr.size - 1):
        yield i, range(rowptr[i], rowptr[i + 1])


def key(t, j):
    tt = np.inf if np.isnan(t[j]) else t[j]
    return (tt, j)


@pytest.mark.parametrize("quant", [None, 0.5, 0.1])
def test_selection_brute_force(orc, quant):
    """Section 2.2: S_i is the unique p_i-subset of N_i whose every member precedes every
    non-member in (time, index) order; its max time is the least over all p_i-subsets
    (Section 3.2.2, T_j(k))."""
    g = np.random.default_rng(11)
    for rowptr, colidx in small_graphs():
        n = rowptr.size - 1
        deg = np.diff(rowptr)
        for trial in range(6):
            t = g.standard_exponential(n).astype(np.float32)
            if quant:
                t = (np.round(t / quant) * quant).astype(np.float32)
            b = g.integers(0, deg + 1).astype(np.int32)
            mask, p, wait = orc.select(rowptr, colidx, t, b)
            assert np.array_equal(p, deg - b)
            for i, es in rows(rowptr, colidx):
                nb = [int(colidx[e]) for e in es]
                sel = {int(colidx[e]) for e in es if mask[e]}
                assert len(sel) == p[i]
                good = []
                best_max = None
                for sub in itertools.combinations(nb, int(p[i])):
                    s = set(sub)
                    rest = [j for j in nb if j not in s]
                    if all(key(t, a) < key(t, c) for a in s for c in rest):
                        good.append(s)
                    m = max([t[i]] + [t[j] for j in sub])
                    best_max = m if best_max is None else min(best_max, m)
                assert len(good) == 1 and good[0] == sel
                assert wait[i] == np.float32(best_max)


def test_selection_degenerate(orc):
    rowptr, colidx = inputs.graph_er(8, 0.5, np.random.default_rng(3))
    deg = np.diff(rowptr).astype(np.int32)
    t = np.random.default_rng(4).standard_exponential(8).astype(np.float32)
    mask, p, _ = orc.select(rowptr, colidx, t, np.zeros(8, np.int32))
    assert mask.all() and np.array_equal(p, deg)          # b = 0: everyone participates
    mask, p, wait = orc.select(rowptr, colidx, t, deg)
    assert not mask.any() and not p.any()                  # b = deg: nobody is waited for
    assert np.array_equal(wait, t)
    with pytest.raises(ValueError):
        orc.select(rowptr, colidx, t, deg + 1)
    with pytest.raises(ValueError):
        orc.select(rowptr, colidx, t, -np.ones(8, np.int32))


def test_selection_special_values(orc):
    """+inf is legal and never precedes a finite time; NaN counts as +inf; -0.0 ties +0.0
    and the lower index wins."""
    rowptr, colidx = inputs.graph_complete(5)
    t = np.array([0.0, np.inf, -0.0, np.nan, 1.0], np.float32)
    b = np.array([2, 2, 2, 2, 2], np.int32)
    mask, p, wait = orc.select(rowptr, colidx, t, b)
    sel = [sorted(int(colidx[e]) for e in es if mask[e]) for _, es in rows(rowptr, colidx)]
    assert sel == [[2, 4], [0, 2], [0, 4], [0, 2], [0, 2]]
    assert wait[1] == np.inf and wait[3] == np.inf and wait[0] == 1.0
    # a dead worker is only waited for when p_i exceeds the number of live neighbours
    b = np.array([0, 0, 0, 0, 0], np.int32)
    mask, _, wait = orc.select(rowptr, colidx, t, b)
    assert mask.all() and np.all(wait == np.inf)


def test_round_time_not_longer_than_full(orc):
    """Corollary 4 holds per realisation: a max over a subset is at most the max over all."""
    g = np.random.default_rng(5)
    rowptr, colidx = inputs.graph_regular(16, 4, g)
    deg = np.diff(rowptr)
    for _ in range(20):
        t = g.standard_exponential(16).astype(np.float32)
        b = g.integers(0, deg + 1).astype(np.int32)
        _, _, wait_p = orc.select(rowptr, colidx, t, b)
        _, _, wait_full = orc.select(rowptr, colidx, t, np.zeros(16, np.int32))
        assert np.all(wait_p <= wait_full) and wait_p.max() <= wait_full.max()


def test_weight_invariants(orc):
    """Assumption 1: non-negative; rows sum to one; off-diagonals are 0 or 1/(1+m) with an
    integer m >= p_i (hence <= 1/(1+p_i) and P_ii >= 1/(1+p_i)); zero exactly on backups."""
    g = np.random.default_rng(13)
    for rowptr, colidx in small_graphs():
        n = rowptr.size - 1
        deg = np.diff(rowptr)
        for _ in range(5):
            t = g.standard_exponential(n).astype(np.float32)
            b = g.integers(0, deg + 1).astype(np.int32)
            mask, p, _ = orc.select(rowptr, colidx, t, b)
            P = orc.dense_P(rowptr, colidx, mask, p)
            we, ws = orc.weights(rowptr, colidx, mask, p)
            assert np.all(P >= 0)
            assert np.allclose(P.sum(1), 1.0, atol=1e-15 * n, rtol=0)
            assert np.array_equal(np.diag(P), ws)
            for i, es in rows(rowptr, colidx):
                assert P[i, i] >= 1.0 / (1 + p[i]) - 1e-15
                off = np.delete(P[i], i)
                assert np.count_nonzero(off) == p[i]
                for e in es:
                    j = colidx[e]
                    assert P[i, j] == we[e]
                    if mask[e]:
                        m = 1.0 / P[i, j] - 1.0
                        assert abs(m - round(m)) < 1e-9 and round(m) >= p[i] and round(m) >= p[j]
                        assert round(m) in (p[i], p[j])
                    else:
                        assert P[i, j] == 0.0


def test_weights_symmetric_mask_doubly_stochastic(orc):
    """Assumption 1's doubly-stochastic claim holds when the active edge set is symmetric
    (b = 0 here): then P is symmetric and columns sum to one too."""
    g = np.random.default_rng(17)
    for rowptr, colidx in small_graphs():
        n = rowptr.size - 1
        t = g.standard_exponential(n).astype(np.float32)
        mask, p, _ = orc.select(rowptr, colidx, t, np.zeros(n, np.int32))
        P = orc.dense_P(rowptr, colidx, mask, p)
        assert np.array_equal(P, P.T)
        assert np.allclose(P.sum(0), 1.0, atol=1e-14, rtol=0)


def test_weights_closed_forms(orc):
    """Static Metropolis-Hastings weights on graphs where they are known in closed form:
    k-regular -> all 1/(k+1); complete -> 1/N; star -> every link 1/N (hub degree N-1)."""
    for (rowptr, colidx), w in [(inputs.graph_ring(8), 1 / 3), (inputs.graph_complete(6), 1 / 6),
                                (inputs.graph_regular(10, 4, np.random.default_rng(1)), 1 / 5)]:
        n = rowptr.size - 1
        mask, p, _ = orc.select(rowptr, colidx, np.arange(n, dtype=np.float32), np.zeros(n, np.int32))
        P = orc.dense_P(rowptr, colidx, mask, p)
        assert set(np.unique(P)) <= {0.0, w} or np.allclose(P[P > 0], w, atol=1e-16)
        assert np.allclose(P[P > 0], w, atol=1e-16)
    n = 6
    adj = np.zeros((n, n), bool)
    adj[0, 1:] = adj[1:, 0] = True
    rowptr, colidx = inputs._csr_from_adj(adj)
    mask, p, _ = orc.select(rowptr, colidx, np.arange(n, dtype=np.float32), np.zeros(n, np.int32))
    P = orc.dense_P(rowptr, colidx, mask, p)
    assert np.allclose(P[0], 1 / n) and np.allclose(P[1:, 0], 1 / n)
    assert np.allclose(np.diag(P)[1:], 1 - 1 / n)


def _golden():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "worked_example_assumption1.txt")
    rec = {}
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, *v = line.split()
        rec[k] = v
    return rec


def test_worked_example(orc):
    """tests/golden/worked_example_assumption1.txt: selection, wait times, weights and
    both update orders on a 4-worker graph, worked by hand from Section 2.2 / Assumption 1."""
    r = _golden()
    fr = lambda k: np.array([float(Fraction(v)) for v in r[k]])
    rowptr, colidx = np.array(r["rowptr"], np.int32), np.array(r["colidx"], np.int32)
    t, b = fr("t").astype(np.float32), np.array(r["b"], np.int32)
    mask, p, wait = orc.select(rowptr, colidx, t, b)
    assert np.array_equal(mask, np.array(r["mask"], np.uint8))
    assert np.array_equal(p, np.array(r["p"], np.int32))
    assert np.array_equal(wait, fr("wait").astype(np.float32))
    P = orc.dense_P(rowptr, colidx, mask, p)
    for i in range(4):
        assert np.allclose(P[i], fr(f"P{i}"), atol=1e-15, rtol=0)
    x = np.stack([fr(f"x{i}") for i in range(4)]).astype(np.float32)
    g = np.stack([fr(f"g{i}") for i in range(4)]).astype(np.float32)
    lr = float(Fraction(r["lr"][0]))
    for order, tag in [(0, "cta"), (1, "atc")]:
        out = orc.round_(rowptr, colidx, mask, p, x, g, lr, order)
        want = np.stack([fr(f"{tag}{i}") for i in range(4)])
        assert np.allclose(out, want, rtol=3e-7, atol=0), (tag, out, want)


def test_round_time(orc):
    """Section 3.2.2: T(k) is the max of the per-worker wait times; over all workers, and
    over the set V' of workers that somebody waits for.  Recomputed here from the mask."""
    g = np.random.default_rng(19)
    for rowptr, colidx in small_graphs():
        n = rowptr.size - 1
        deg = np.diff(rowptr)
        for _ in range(5):
            t = g.standard_exponential(n).astype(np.float32)
            b = g.integers(0, deg + 1).astype(np.int32)
            mask, p, wait = orc.select(rowptr, colidx, t, b)
            t_all, t_sel = orc.round_time(rowptr, colidx, mask, wait)
            listed = sorted({int(colidx[e]) for e in range(colidx.size) if mask[e]})
            assert t_all == wait.max()
            assert t_sel == (wait[listed].max() if listed else 0.0)
            # never longer than the full-participation round on the same response times
            m0, _, w0 = orc.select(rowptr, colidx, t, np.zeros(n, np.int32))
            f_all, f_sel = orc.round_time(rowptr, colidx, m0, w0)
            assert t_all <= f_all and f_all == t.max() == f_sel


def test_round_time_worked_example(orc):
    """Hand-worked round duration (tests/golden/worked_example_round_time.txt): the worker with the
    largest wait time is waited for by nobody, so the maximum over the set V' of Section 3.2.2 is
    smaller than the maximum over all workers."""
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "worked_example_round_time.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, *v = line.split()
                vals[k] = v
    rowptr, colidx = np.array(vals["rowptr"], np.int32), np.array(vals["colidx"], np.int32)
    t, b = np.array(vals["t"], np.float32), np.array(vals["b"], np.int32)
    mask, p, wait = orc.select(rowptr, colidx, t, b)
    assert np.array_equal(mask, np.array(vals["mask"], np.uint8))
    assert np.array_equal(p, np.array(vals["p"], np.int32))
    assert np.array_equal(wait, np.array(vals["wait"], np.float32))
    t_all, t_listed = orc.round_time(rowptr, colidx, mask, wait)
    assert t_all == np.float32(vals["T_all_workers"][0]) and t_listed == np.float32(vals["T_over_listed"][0])
    m0, _, w0 = orc.select(rowptr, colidx, t, np.zeros(4, np.int32))
    f_all, f_listed = orc.round_time(rowptr, colidx, m0, w0)
    assert f_all == np.float32(vals["full_T_all_workers"][0]) and f_listed == np.float32(vals["full_T_over_listed"][0])
