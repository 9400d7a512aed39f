"""GPU parity of the tile-major storage layout: the layout converter, rounds against the
oracle (both orders, with and without gradients, per-worker rates), padding, error paths."""
import numpy as np
import pytest
import torch

from paper_2102_06280_amd import inputs
from gpu_util import assert_params_close, dev

pytestmark = pytest.mark.gpu
W = 64


@pytest.fixture(scope="module")
def B():
    from paper_2102_06280_amd import binding
    return binding


def to_tiles(a):
    """[N, ld] row layout -> the same container holding the tile-major order."""
    n, ld = a.shape
    return np.ascontiguousarray(a.reshape(n, ld // W, W).transpose(1, 0, 2)).reshape(n, ld)


def to_rows(a):
    n, ld = a.shape
    return np.ascontiguousarray(a.reshape(ld // W, n, W).transpose(1, 0, 2)).reshape(n, ld)


def _graphs():
    g = np.random.default_rng(601)
    return {"ring8": inputs.graph_ring(8), "ring3": inputs.graph_ring(3), "er40": inputs.graph_er(40, 0.2, g),
            "reg4x100": inputs.graph_regular(100, 4, g), "reg8x128": inputs.graph_regular(128, 8, g),
            "er130": inputs.graph_er(130, 0.05, g), "complete256": inputs.graph_complete(256),
            "reg6x200": inputs.graph_regular(200, 6, g)}


def test_layout_converter_round_trip(B):
    rowptr, colidx = inputs.graph_ring(8)
    n, ld = 8, 640
    h = B.dbw_create(rowptr, colidx, n, 600, ld=ld)
    try:
        a = np.arange(n * ld, dtype=np.float32).reshape(n, ld)
        t, back = torch.zeros((n, ld), device="cuda"), torch.zeros((n, ld), device="cuda")
        B.dbw_convert_layout(h, dev(a), t, True)
        assert np.array_equal(t.cpu().numpy(), to_tiles(a))
        B.dbw_convert_layout(h, t, back, False)
        assert np.array_equal(back.cpu().numpy(), a)
        assert np.array_equal(to_rows(to_tiles(a)), a)
        with pytest.raises(B.DbwError) as e:
            B.dbw_convert_layout(h, t, t, True)
        assert e.value.code == B.ERR_ALIAS
    finally:
        B.dbw_destroy(h)


CASES = [
    # graph, d, ld
    ("ring8", 7850, 7872),         # 16 layout tiles per workgroup, d % 64 and d % 4 != 0
    ("ring3", 200, 256),           # 42 tiles per workgroup, more than there are
    ("er40", 5000, 5056),
    ("reg4x100", 9001, 9024),      # N does not divide 128
    ("reg8x128", 70001, 70016),
    ("er130", 3000, 3008),         # one tile per workgroup, 8 float4 per thread
    ("reg6x200", 1111, 1152),
    ("complete256", 777, 832),     # lists too long for LDS
    ("ring8", 3, 64),
]


@pytest.mark.parametrize("order", [0, 1], ids=["cta", "atc"])
@pytest.mark.parametrize("gname,d,ld", CASES, ids=[f"{c[0]}-d{c[1]}" for c in CASES])
def test_tile_major_round_matches_oracle(B, orc, gname, d, ld, order):
    rowptr, colidx = _graphs()[gname]
    n = rowptr.size - 1
    deg = np.diff(rowptr)
    g = np.random.default_rng(603)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, order=order, layout=B.LAYOUT_TILES)
    try:
        assert B.dbw_mix_path(h) == B.MIX_CSR
        x = g.standard_normal((n, ld)).astype(np.float32)
        for rnd in range(4):
            gr = (g.standard_normal((n, ld)) * 0.1).astype(np.float32)
            t = g.standard_exponential(n).astype(np.float32)
            b = g.integers(0, deg + 1).astype(np.int32) if rnd else np.zeros(n, np.int32)
            eta = g.uniform(0.0, 0.3, n).astype(np.float32)
            dout = dev(to_tiles(np.full((n, ld), 7.0, np.float32)))
            B.dbw_select(h, dev(t), dev(b))
            mask, p, _ = orc.select(rowptr, colidx, t, b)
            if rnd == 2:                                    # gradient-free
                B.dbw_round(h, dev(to_tiles(x)), dout, 0.05)
                want = orc.round_(rowptr, colidx, mask, p, x, None, 0.05, order, d=d)
            elif rnd == 3:                                  # a rate per worker
                B.dbw_round_eta(h, dev(to_tiles(x)), dout, dev(eta), ext_grads=dev(to_tiles(gr)))
                want = orc.round_eta(rowptr, colidx, mask, p, x, gr, eta, order, d=d)
            else:
                B.dbw_round(h, dev(to_tiles(x)), dout, 0.05, ext_grads=dev(to_tiles(gr)))
                want = orc.round_(rowptr, colidx, mask, p, x, gr, np.float32(0.05), order, d=d)
            got = to_rows(dout.cpu().numpy())
            assert_params_close(got, want, d=d, what=f"{gname} round {rnd}")
            assert np.all(got[:, d:] == 7.0), "padding columns were written"
            x = want
            x[:, d:] = g.standard_normal((n, ld - d)).astype(np.float32)   # padding may hold anything
    finally:
        B.dbw_destroy(h)


def test_tile_major_bitwise_equal_to_row_layout(B):
    """Same summation order in both layouts: identical bits."""
    rowptr, colidx = inputs.graph_regular(32, 4, np.random.default_rng(605))
    n, d, ld = 32, 159010, 159040
    g = np.random.default_rng(606)
    x, gr = g.standard_normal((n, ld)).astype(np.float32), g.standard_normal((n, ld)).astype(np.float32)
    t, b = g.standard_exponential(n).astype(np.float32), g.integers(0, 3, n).astype(np.int32)
    outs = []
    for layout in (B.LAYOUT_ROWS, B.LAYOUT_TILES):
        h = B.dbw_create(rowptr, colidx, n, d, ld=ld, layout=layout)
        try:
            conv = to_tiles if layout == B.LAYOUT_TILES else (lambda a: a)
            out = torch.zeros((n, ld), device="cuda")
            B.dbw_select(h, dev(t), dev(b))
            B.dbw_round(h, dev(conv(x)), out, 0.05, ext_grads=dev(conv(gr)))
            o = out.cpu().numpy()
            outs.append(to_rows(o) if layout == B.LAYOUT_TILES else o)
        finally:
            B.dbw_destroy(h)
    assert np.array_equal(outs[0][:, :d], outs[1][:, :d])


def test_tile_major_unsupported_combinations(B):
    rowptr, colidx = inputs.graph_ring(8)
    with pytest.raises(B.DbwError) as e:
        B.dbw_create(rowptr, colidx, 8, 100, ld=100, layout=B.LAYOUT_TILES)        # ld not a multiple of 64
    assert e.value.code == B.ERR_INVALID
    with pytest.raises(B.DbwError) as e:
        B.dbw_create(rowptr, colidx, 8, 7850, ld=7872, layout=B.LAYOUT_TILES,
                     model=B.make_model(B.MODEL_MLP, 4, [784, 10]))
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.DbwError) as e:
        B.dbw_create(rowptr, colidx, 8, 128, ld=128, layout=B.LAYOUT_TILES, mix_path=B.MIX_DENSE)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.DbwError) as e:
        B.dbw_create(*inputs.graph_ring(300), 300, 128, ld=128, layout=B.LAYOUT_TILES)
    assert e.value.code == B.ERR_UNSUPPORTED
    h = B.dbw_create(rowptr, colidx, 8, 128, ld=128, layout=B.LAYOUT_TILES)
    try:
        x, y = torch.zeros((8, 128), device="cuda"), torch.zeros((8, 128), device="cuda")
        with pytest.raises(B.DbwError) as e:
            B.dbw_consensus_rounds(h, x, y, torch.ones((1, 8), device="cuda"),
                                   torch.zeros((1, 8), dtype=torch.int32, device="cuda"), 1)
        assert e.value.code == B.ERR_UNSUPPORTED
    finally:
        B.dbw_destroy(h)
