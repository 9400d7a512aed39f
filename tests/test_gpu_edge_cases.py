"""Degenerate and extreme shapes through the C ABI: a single worker, two workers, one column,
more workers than the LDS-tile kernel takes, rows longer than the selection kernel's LDS key
buffer."""
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


def _tiles(a, back=False):
    """[N, ld] rows <-> the same container in tile-major order (64-column tiles)."""
    n, ld = a.shape
    if back:
        return np.ascontiguousarray(a.reshape(ld // 64, n, 64).transpose(1, 0, 2)).reshape(n, ld)
    return np.ascontiguousarray(a.reshape(n, ld // 64, 64).transpose(1, 0, 2)).reshape(n, ld)


def one_round(B, orc, rowptr, colidx, d, ld, order, t, b, layout=0, mix=0):
    n = rowptr.size - 1
    conv = (lambda a: _tiles(a)) if layout else (lambda a: a)
    g = np.random.default_rng(701)
    x = g.standard_normal((n, ld)).astype(np.float32)
    gr = g.standard_normal((n, ld)).astype(np.float32)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, order=order, layout=layout, mix_path=mix)
    try:
        out = torch.full((n, ld), 7.0, device="cuda")
        B.dbw_select(h, dev(t), dev(b))
        B.dbw_round(h, dev(conv(x)), out, 0.1, ext_grads=dev(conv(gr)))
        p_d = torch.empty(n, dtype=torch.int32, device="cuda")
        mask_d = torch.empty(max(colidx.size, 1), dtype=torch.uint8, device="cuda")
        wait_d = torch.empty(n, dtype=torch.float32, device="cuda")
        B.dbw_get_selection(h, p_d, mask_d, wait_d)
        mask, p, wait = orc.select(rowptr, colidx, t, b)
        assert np.array_equal(p_d.cpu().numpy(), p)
        assert np.array_equal(mask_d.cpu().numpy()[:colidx.size], mask)
        assert np.array_equal(wait_d.cpu().numpy(), wait)
        want = orc.round_(rowptr, colidx, mask, p, x, gr, np.float32(0.1), order, d=d)
        got = out.cpu().numpy()
        if layout:
            got = _tiles(got, back=True)
        assert_params_close(got, want, d=d)
        assert np.all(got[:, d:] == 7.0)
        return got, x, gr
    finally:
        B.dbw_destroy(h)


@pytest.mark.parametrize("order", [0, 1])
def test_single_worker_is_plain_sgd(B, orc, order):
    rowptr, colidx = np.array([0, 0], np.int32), np.zeros(0, np.int32)
    for d, ld in ((1, 1), (5, 8), (1000, 1024)):
        got, x, gr = one_round(B, orc, rowptr, colidx, d, ld, order, np.array([1.5], np.float32), np.zeros(1, np.int32))
        assert np.allclose(got[:, :d], x[:, :d] - np.float32(0.1) * gr[:, :d], rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("b", [[0, 0], [1, 0], [1, 1]])
def test_two_workers(B, orc, order, b):
    rowptr, colidx = np.array([0, 1, 2], np.int32), np.array([1, 0], np.int32)
    one_round(B, orc, rowptr, colidx, 333, 384, order, np.array([2.0, 1.0], np.float32), np.array(b, np.int32))
    one_round(B, orc, rowptr, colidx, 333, 384, order, np.array([2.0, 1.0], np.float32), np.array(b, np.int32),
              mix=B.MIX_DENSE)
    one_round(B, orc, rowptr, colidx, 333, 384, order, np.array([2.0, 1.0], np.float32), np.array(b, np.int32),
              layout=B.LAYOUT_TILES)


def test_more_workers_than_the_tile_kernels_take(B, orc):
    """N = 600: the gather kernel; all response times equal, so ties go by index."""
    rowptr, colidx = inputs.graph_regular(600, 6, np.random.default_rng(703))
    t = np.ones(600, np.float32)
    b = np.random.default_rng(704).integers(0, 7, 600).astype(np.int32)
    one_round(B, orc, rowptr, colidx, 4100, 4160, 0, t, b)
    one_round(B, orc, rowptr, colidx, 4100, 4160, 1, t, b)


def test_rows_longer_than_the_key_buffer(B, orc):
    """Complete graph on 2100 workers: 2099 neighbours per row, more than the selection kernel
    keeps in LDS; selection, wait times and a narrow round."""
    n = 2100
    rowptr, colidx = inputs.graph_complete(n)
    g = np.random.default_rng(705)
    t = np.round(g.standard_exponential(n) * 8).astype(np.float32) / 8      # many ties
    b = g.integers(0, n, n).astype(np.int32)
    one_round(B, orc, rowptr, colidx, 8, 8, 0, t, b, mix=B.MIX_CSR)


def test_dense_path_limits(B):
    """The matrix-core path is refused at create beyond its limits (N > 256 workers, or rows so
    long that its 32-bit lane offsets would wrap), and the automatic choice avoids it there."""
    rowptr, colidx = inputs.graph_complete(16)
    too_long = 26_843_545 + 1 + 63
    too_long -= too_long % 64
    with pytest.raises(RuntimeError, match="not supported"):
        B.dbw_create(rowptr, colidx, 16, too_long, ld=too_long, mix_path=B.MIX_DENSE)
    h = B.dbw_create(rowptr, colidx, 16, too_long, ld=too_long)
    assert B.dbw_mix_path(h) == B.MIX_CSR
    B.dbw_destroy(h)
    h = B.dbw_create(rowptr, colidx, 16, 4096)
    assert B.dbw_mix_path(h) == B.MIX_DENSE
    B.dbw_destroy(h)
    rowptr, colidx = inputs.graph_complete(300)
    with pytest.raises(RuntimeError, match="not supported"):
        B.dbw_create(rowptr, colidx, 300, 64, mix_path=B.MIX_DENSE)
