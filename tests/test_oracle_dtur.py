"""Pins for the oracle's threshold rule and d-iteration procedure (Section 4.1, Alg. 2)."""
import numpy as np

from paper_2102_06280_amd import inputs


def _connected(n, edges):
    adj = {i: set() for i in range(n)}
    for u, v in edges:
        adj[u].add(v); adj[v].add(u)
    seen, st = {0}, [0]
    while st:
        u = st.pop()
        for v in adj[u]:
            if v not in seen:
                seen.add(v); st.append(v)
    return len(seen) == n


def test_link_set_is_spanning_tree(orc):
    g = np.random.default_rng(61)
    for rowptr, colidx in [inputs.graph_ring(8), inputs.graph_er(20, 0.2, g), inputs.graph_complete(6)]:
        n = rowptr.size - 1
        edges = orc.spanning_tree(rowptr, colidx)
        assert len(edges) == n - 1 and _connected(n, edges.tolist())
        for u, v in edges:
            assert v in colidx[rowptr[u]:rowptr[u + 1]]


def test_dtur_epochs(orc):
    """Every epoch of d rounds activates each link of P once, so the union of the active
    graphs over an epoch is connected (Assumption 2 with B = d); theta is a link
    establishment time, so at least the 2nd-smallest response time; the active edge set is
    symmetric; feeding the resulting b to the fastest-p selection reproduces the threshold
    sets exactly, ties at theta included."""
    g = np.random.default_rng(67)
    for quant in (None, 0.25):
        rowptr, colidx = inputs.graph_er(12, 0.3, g)
        n = 12
        dt = orc.Dtur(rowptr, colidx)
        d = len(dt.edges)
        for epoch in range(3):
            union, established = set(), set()
            for l in range(d):
                t = g.standard_exponential(n).astype(np.float32)
                if quant:
                    t = (np.ceil(t / quant) * quant).astype(np.float32)
                visited_before = dt.visited.copy()
                if visited_before.all():        # P' is emptied when an epoch is complete
                    visited_before[:] = 0
                b, theta = dt.step(t)
                new = np.flatnonzero(dt.visited != visited_before)
                assert new.size == 1
                e = int(new[0])
                u, v = dt.edges[e]
                assert theta == max(t[u], t[v])
                # theta is the minimum over unvisited links, lowest id on ties
                cand = [(max(t[a], t[c]), k) for k, (a, c) in enumerate(dt.edges) if not visited_before[k]]
                assert min(cand) == (theta, e)
                assert theta >= np.sort(t)[1]
                established.add(e)
                mask, p, wait = orc.select(rowptr, colidx, t, b)
                for i in range(n):
                    sel = {int(colidx[k]) for k in range(rowptr[i], rowptr[i + 1]) if mask[k]}
                    want = {int(j) for j in colidx[rowptr[i]:rowptr[i + 1]] if t[j] <= theta} if t[i] <= theta else set()
                    assert sel == want
                    for j in sel:
                        union.add((min(i, j), max(i, j)))
                        assert i in {int(colidx[k]) for k in range(rowptr[j], rowptr[j + 1]) if mask[k]}
                assert (min(u, v), max(u, v)) in union
                assert np.all(wait[t <= theta] <= theta)
            assert established == set(range(d))
            assert _connected(n, list(union))
        assert dt.n_visited.value == d


def test_dtur_dead_worker(orc):
    """A worker that never answers (t = +inf) sits on some link of P; the round that must
    establish that link has theta = +inf and then everyone waits for everyone."""
    rowptr, colidx = inputs.graph_ring(5)
    dt = orc.Dtur(rowptr, colidx)
    t = np.array([0.1, 0.2, np.inf, 0.3, 0.4], np.float32)
    thetas = [dt.step(t) for _ in range(4)]
    assert [th for _, th in thetas[:3]] == [np.float32(0.2), np.float32(0.4), np.float32(0.4)]
    assert np.isinf(thetas[3][1])                           # the one tree link at worker 2
    b, _ = thetas[-1]
    assert not b.any()
