"""GPU parity of the dense (matrix-core) mixing path against the CPU oracle, and its
agreement with the sparse path, through the C ABI."""
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


def _graph(name):
    g = np.random.default_rng(211)
    return {"complete5": lambda: inputs.graph_complete(5), "complete40": lambda: inputs.graph_complete(40),
            "er100": lambda: inputs.graph_er(100, 0.6, g), "complete256": lambda: inputs.graph_complete(256),
            "complete130": lambda: inputs.graph_complete(130)}[name]()


CASES = [("complete5", 1000, 1024), ("complete40", 4100, 4160), ("er100", 2050, 2112),
         ("complete130", 777, 832), ("complete256", 8192 + 70, 8320), ("complete256", 64, 64),
         ("complete40", 30, 30)]


@pytest.mark.parametrize("order", [0, 1], ids=["cta", "atc"])
@pytest.mark.parametrize("gname,d,ld", CASES, ids=[f"{c[0]}-d{c[1]}" for c in CASES])
def test_dense_round_matches_oracle(B, orc, gname, d, ld, order):
    rowptr, colidx = _graph(gname)
    n = rowptr.size - 1
    deg = np.diff(rowptr)
    g = np.random.default_rng(213)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, order=order, mix_path=B.MIX_DENSE)
    hs = B.dbw_create(rowptr, colidx, n, d, ld=ld, order=order, mix_path=B.MIX_CSR)
    try:
        assert B.dbw_mix_path(h) == B.MIX_DENSE and B.dbw_mix_path(hs) == B.MIX_CSR
        x = g.standard_normal((n, ld)).astype(np.float32)
        for rnd in range(3):
            gr = (g.standard_normal((n, ld)) * 0.01).astype(np.float32)
            t = g.standard_exponential(n).astype(np.float32)
            b = g.integers(0, deg // 2 + 1).astype(np.int32) if rnd else np.zeros(n, np.int32)
            lr = np.float32(0.05)
            dx, dg, dt, db = dev(x), dev(gr) if rnd < 2 else None, dev(t), dev(b)
            outs = []
            for hh in (h, hs):
                out = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
                B.dbw_select(hh, dt, db)
                B.dbw_round(hh, dx, out, lr, ext_grads=dg)
                outs.append(out.cpu().numpy())
            mask, p, _ = orc.select(rowptr, colidx, t, b)
            want = orc.round_(rowptr, colidx, mask, p, x, gr if rnd < 2 else None, lr, order, d=d)
            assert_params_close(outs[0], want, d=d, what=f"dense {gname} round {rnd}")
            assert_params_close(outs[1], want, d=d, what=f"sparse {gname} round {rnd}")
            assert np.all(outs[0][:, d:] == 7.0)
            x = want
            x[:, d:] = 0
    finally:
        B.dbw_destroy(h)
        B.dbw_destroy(hs)


def test_auto_path_choice(B):
    for graph, want in [(inputs.graph_complete(64), "dense"), (inputs.graph_ring(64), "csr")]:
        h = B.dbw_create(*graph, 64, 256)
        assert B.dbw_mix_path(h) == (B.MIX_DENSE if want == "dense" else B.MIX_CSR)
        B.dbw_destroy(h)
    rowptr, colidx = inputs.graph_ring(300)
    with pytest.raises(B.DbwError) as e:
        B.dbw_create(rowptr, colidx, 300, 64, mix_path=B.MIX_DENSE)
    assert e.value.code == B.ERR_UNSUPPORTED
