"""GPU parity of several gradient-free rounds collapsed into one pass (dbw_consensus_rounds)
against the oracle's round applied r times, and against the library's own r single rounds."""
import numpy as np
import pytest
import torch

from paper_2102_06280_amd import inputs
from gpu_util import assert_params_close, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2102_06280_amd import binding
    return binding


def _graphs():
    g = np.random.default_rng(501)
    return {"ring8": inputs.graph_ring(8), "er40": inputs.graph_er(40, 0.2, g),
            "reg8x128": inputs.graph_regular(128, 8, g), "complete256": inputs.graph_complete(256),
            "complete130": inputs.graph_complete(130)}


CASES = [
    # graph, d, ld, rounds, mixing path of the context
    ("ring8", 7850, 7850, 5, "csr"),            # rows not 16-byte aligned: scalar application only
    ("ring8", 7850, 7872, 1, "csr"),            # a single round, ragged tail
    ("er40", 5000, 5120, 7, "csr"),
    ("reg8x128", 70001, 70016, 12, "csr"),      # unguarded matrix-core kernel + one tail column
    ("complete130", 777, 832, 4, "dense"),
    ("complete256", 8192, 8192, 6, "dense"),
    ("complete256", 8192 + 70, 8320, 3, "csr"),
]


@pytest.mark.parametrize("gname,d,ld,r,path", CASES, ids=[f"{c[0]}-d{c[1]}-ld{c[2]}-r{c[3]}-{c[4]}" for c in CASES])
def test_collapsed_rounds_match_oracle(B, orc, gname, d, ld, r, path):
    rowptr, colidx = _graphs()[gname]
    n = rowptr.size - 1
    deg = np.diff(rowptr)
    g = np.random.default_rng(503)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, mix_path=B.MIX_DENSE if path == "dense" else B.MIX_CSR)
    try:
        x = g.standard_normal((n, ld)).astype(np.float32)
        t = g.standard_exponential((r, n)).astype(np.float32)
        t[0] = np.round(t[0] * 4) / 4                                   # ties in one round
        b = np.stack([g.integers(0, deg + 1) for _ in range(r)]).astype(np.int32)
        dx, dt, db = dev(x), dev(t), dev(b)
        out = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
        B.dbw_consensus_rounds(h, dx, out, dt, db, r)
        got = out.cpu().numpy()
        # the selection state left behind is the last round's
        mask_d = torch.empty(max(colidx.size, 1), dtype=torch.uint8, device="cuda")
        B.dbw_get_selection(h, None, mask_d, None)
        want = x
        for q in range(r):
            mask, p, _ = orc.select(rowptr, colidx, t[q], b[q])
            want = orc.round_(rowptr, colidx, mask, p, want, None, 0.0, 0, d=d)
        assert np.array_equal(mask_d.cpu().numpy()[:colidx.size], mask)
        assert_params_close(got, want, d=d, what=f"{gname} {r} rounds collapsed")
        assert np.all(got[:, d:] == 7.0)
        # the library's own r single rounds, ping-pong
        a, c = dx.clone(), torch.zeros_like(dx)
        for q in range(r):
            B.dbw_select(h, dt[q], db[q])
            B.dbw_round(h, a, c, 0.0)
            a, c = c, a
        assert_params_close(got, a.cpu().numpy(), d=d, what=f"{gname} collapsed against single rounds")
    finally:
        B.dbw_destroy(h)


def test_collapsed_rounds_reach_the_mean(B):
    """Full participation (b = 0) on a connected graph: many gradient-free rounds drive every
    worker to the average of the initial vectors, which the symmetric weights preserve
    (the corollary on the limit of the truncated recursion)."""
    rowptr, colidx = inputs.graph_regular(32, 4, np.random.default_rng(505))
    n, d, r = 32, 4096, 200
    g = np.random.default_rng(506)
    h = B.dbw_create(rowptr, colidx, n, d)
    try:
        x = g.standard_normal((n, d)).astype(np.float32)
        out = torch.zeros((n, d), device="cuda")
        B.dbw_consensus_rounds(h, dev(x), out, dev(g.standard_exponential((r, n)).astype(np.float32)),
                               dev(np.zeros((r, n), np.int32)), r)
        got = out.cpu().numpy().astype(np.float64)
        mean = x.astype(np.float64).mean(0)
        assert np.abs(got - mean).max() < 1e-4
    finally:
        B.dbw_destroy(h)


def test_collapsed_rounds_argument_checks(B):
    rowptr, colidx = inputs.graph_ring(8)
    h = B.dbw_create(rowptr, colidx, 8, 64)
    try:
        x, y = torch.zeros((8, 64), device="cuda"), torch.zeros((8, 64), device="cuda")
        t, b = torch.ones((2, 8), device="cuda"), torch.zeros((2, 8), dtype=torch.int32, device="cuda")
        with pytest.raises(B.DbwError) as e:
            B.dbw_consensus_rounds(h, x, x, t, b, 2)
        assert e.value.code == B.ERR_ALIAS
        with pytest.raises(B.DbwError) as e:
            B.dbw_consensus_rounds(h, x, y, t, b, 0)
        assert e.value.code == B.ERR_INVALID
        with pytest.raises(B.DbwError) as e:
            B.dbw_consensus_rounds(h, x, y, None, b, 2)
        assert e.value.code == B.ERR_NULL
        bad = torch.full((2, 8), 5, dtype=torch.int32, device="cuda")
        B.dbw_consensus_rounds(h, x, y, t, bad, 2)
        with pytest.raises(B.DbwError) as e:
            B.dbw_check(h)
        assert e.value.code == B.ERR_INVALID
    finally:
        B.dbw_destroy(h)
    big = inputs.graph_ring(300)
    h = B.dbw_create(*big, 300, 64)
    try:
        x, y = torch.zeros((300, 64), device="cuda"), torch.zeros((300, 64), device="cuda")
        with pytest.raises(B.DbwError) as e:
            B.dbw_consensus_rounds(h, x, y, torch.ones((1, 300), device="cuda"),
                                   torch.zeros((1, 300), dtype=torch.int32, device="cuda"), 1)
        assert e.value.code == B.ERR_UNSUPPORTED
    finally:
        B.dbw_destroy(h)
