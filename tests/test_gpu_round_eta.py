"""GPU parity of rounds with a learning rate per worker (dbw_round_eta) on every mixing
kernel: LDS tiles, gather, scalar tail, dense with and without guards; both orders."""
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
    g = np.random.default_rng(301)
    return {"ring8": inputs.graph_ring(8), "reg4x32": inputs.graph_regular(32, 4, g),
            "reg8x128": inputs.graph_regular(128, 8, g), "er40": inputs.graph_er(40, 0.2, g),
            "complete40": inputs.graph_complete(40), "complete256": inputs.graph_complete(256),
            "complete130": inputs.graph_complete(130)}


CASES = [
    # graph, d, ld, path
    ("ring8", 7850, 7850, "csr"),          # scalar kernel only
    ("ring8", 7850, 7872, "csr"),          # gather kernel + tail
    ("reg4x32", 159010, 159040, "csr"),    # LDS tiles + tail
    ("reg8x128", 70001, 70016, "csr"),     # LDS tiles, narrow tile
    ("er40", 5000, 5120, "csr"),
    ("complete40", 4100, 4160, "dense"),   # guarded dense kernel
    ("complete130", 777, 832, "dense"),
    ("complete256", 8192, 8192, "dense"),  # unguarded dense kernel
    ("complete256", 8192 + 70, 8320, "dense"),
]


@pytest.mark.parametrize("order", [0, 1], ids=["cta", "atc"])
@pytest.mark.parametrize("gname,d,ld,path", CASES, ids=[f"{c[0]}-d{c[1]}-ld{c[2]}-{c[3]}" for c in CASES])
def test_round_eta_matches_oracle(B, orc, gname, d, ld, path, order):
    rowptr, colidx = _graphs()[gname]
    n = rowptr.size - 1
    deg = np.diff(rowptr)
    g = np.random.default_rng(303)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, order=order,
                     mix_path=B.MIX_DENSE if path == "dense" else B.MIX_CSR)
    try:
        x = g.standard_normal((n, ld)).astype(np.float32)
        for rnd in range(2):
            gr = (g.standard_normal((n, ld)) * 0.1).astype(np.float32)
            t = g.standard_exponential(n).astype(np.float32)
            b = g.integers(0, deg + 1).astype(np.int32) if rnd else np.zeros(n, np.int32)
            eta = g.uniform(0.0, 0.5, n).astype(np.float32)
            eta[g.integers(0, n)] = 0.0
            dout = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
            B.dbw_select(h, dev(t), dev(b))
            B.dbw_round_eta(h, dev(x), dout, dev(eta), ext_grads=dev(gr))
            got = dout.cpu().numpy()
            mask, p, _ = orc.select(rowptr, colidx, t, b)
            want = orc.round_eta(rowptr, colidx, mask, p, x, gr, eta, order, d=d)
            assert_params_close(got, want, d=d, what=f"{gname} round {rnd}")
            assert np.all(got[:, d:] == 7.0)
            x = want
            x[:, d:] = 0
    finally:
        B.dbw_destroy(h)


def test_round_eta_equal_entries_is_bitwise_the_scalar_round(B):
    rowptr, colidx = inputs.graph_regular(32, 4, np.random.default_rng(305))
    n, d = 32, 159010
    ld = inputs.pad_ld(d)
    g = np.random.default_rng(306)
    for order in (0, 1):
        h = B.dbw_create(rowptr, colidx, n, d, ld=ld, order=order)
        try:
            x, gr = dev(g.standard_normal((n, ld)).astype(np.float32)), dev(g.standard_normal((n, ld)).astype(np.float32))
            B.dbw_select(h, dev(g.standard_exponential(n).astype(np.float32)), dev(np.ones(n, np.int32)))
            a, e = torch.zeros_like(x), torch.zeros_like(x)
            B.dbw_round(h, x, a, 0.25, ext_grads=gr)
            B.dbw_round_eta(h, x, e, dev(np.full(n, 0.25, np.float32)), ext_grads=gr)
            assert torch.equal(a, e)
        finally:
            B.dbw_destroy(h)


def test_round_eta_with_model_and_null_checks(B, orc):
    """Per-worker rates on computed gradients (config 2's model), and the error path."""
    cfg = inputs.CONFIGS[2]
    desc = inputs.model_dims(cfg.model)
    rowptr, colidx = inputs.make_graph(cfg)
    ld = inputs.pad_ld(cfg.d)
    kind, od = orc.model_desc(desc)
    h = B.dbw_create(rowptr, colidx, cfg.n, cfg.d, ld=ld, model=B.make_model(B.MODEL_MLP, cfg.batch, desc["dims"]))
    try:
        x = inputs.init_params(desc, cfg.n, ld, inputs.rng(2, inputs.P_PARAMS))
        t, b = inputs.response_times(cfg, 1), inputs.backup_counts(cfg, 1, rowptr)
        bx, by = inputs.batch(cfg, 1)
        eta = np.linspace(0.01, 0.2, cfg.n).astype(np.float32)
        out = torch.zeros((cfg.n, ld), device="cuda")
        B.dbw_select(h, dev(t), dev(b))
        with pytest.raises(B.DbwError) as e:
            B.dbw_round_eta(h, dev(x), out, None, batch_x=dev(bx), batch_y=dev(by))
        assert e.value.code == B.ERR_NULL
        B.dbw_round_eta(h, dev(x), out, dev(eta), batch_x=dev(bx), batch_y=dev(by))
        mask, p, _ = orc.select(rowptr, colidx, t, b)
        grad, _ = orc.grad_all(kind, od, cfg.d, x, bx, by)
        want = orc.round_eta(rowptr, colidx, mask, p, x, grad, eta, 0, d=cfg.d)
        assert_params_close(out.cpu().numpy(), want, d=cfg.d, what="config 2 with per-worker rates")
    finally:
        B.dbw_destroy(h)
