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


def test_label_out_of_range_is_clamped_and_reported(B, orc):
    """A label outside [0, classes) cannot index outside the logits: it is clamped, the round's
    result is that of the clamped label, and dbw_check reports DBW_ERR_INVALID."""
    dims, batch, n = [20, 6], 5, 3
    g = np.random.default_rng(711)
    desc = {"kind": "mlp", "dims": dims}
    d = inputs.param_count(desc)
    ld = inputs.pad_ld(d)
    rowptr, colidx = inputs.graph_ring(n)
    params = inputs.init_params(desc, n, ld, g)
    x = g.standard_normal((n, batch, dims[0])).astype(np.float32)
    y = g.integers(0, dims[-1], (n, batch)).astype(np.int32)
    bad = y.copy()
    bad[1, 2], bad[2, 0] = 6 + 1000, -5
    clamped = bad.clip(0, dims[-1] - 1)
    for model_kind in (B.MODEL_MLP, B.MODEL_SOFTMAX):       # the one-layer model under both of its names
        h = B.dbw_create(rowptr, colidx, n, d, ld=ld, model=B.make_model(model_kind, batch, dims))
        try:
            grads = torch.zeros((n, ld), device="cuda")
            loss = torch.zeros(n, device="cuda")
            B.dbw_grad(h, dev(params), dev(x), dev(bad), grads, loss)
            with pytest.raises(B.DbwError) as e:
                B.dbw_check(h)
            assert e.value.code == B.ERR_INVALID
            assert B.dbw_check(h) == B.OK                   # cleared by the report
            kind, od = orc.model_desc(desc)
            want, wl = orc.grad_all(kind, od, d, params, x, clamped)
            assert np.allclose(loss.cpu().numpy(), wl, rtol=1e-5)
            got = grads.cpu().numpy()
            assert np.allclose(got[:, :d], want[:, :d], rtol=1e-4, atol=1e-7)
            B.dbw_grad(h, dev(params), dev(x), dev(y), grads, loss)
            assert B.dbw_check(h) == B.OK
        finally:
            B.dbw_destroy(h)


def test_threshold_rule_state_round_trip_and_warning(B, orc):
    """The epoch state of the threshold rule can be taken out and put back (checkpoint / resume);
    dbw_dtur_reset needs no synchronisation to take effect in stream order; a round in which no
    unvisited link can be established leaves the theta = +inf warning."""
    rowptr, colidx = inputs.graph_er(12, 0.3, np.random.default_rng(713))
    n = 12
    g = np.random.default_rng(715)
    ts = g.standard_exponential((9, n)).astype(np.float32)
    h1 = B.dbw_create(rowptr, colidx, n, 8)
    h2 = B.dbw_create(rowptr, colidx, n, 8)
    try:
        b1 = torch.zeros(n, dtype=torch.int32, device="cuda")
        b2 = torch.zeros(n, dtype=torch.int32, device="cuda")
        dt = orc.Dtur(rowptr, colidx)
        for k in range(5):
            B.dbw_dtur_b(h1, dev(ts[k]), b1)
            dt.step(ts[k])
        visited, nv = B.dbw_dtur_get_state(h1, n)
        assert nv == 5 and visited.sum() == 5 and np.array_equal(visited, dt.visited[:n - 1])
        B.dbw_dtur_set_state(h2, visited, nv)               # a fresh context resumes the epoch
        for k in range(5, 9):
            B.dbw_dtur_b(h1, dev(ts[k]), b1)
            B.dbw_dtur_b(h2, dev(ts[k]), b2)
            assert torch.equal(b1, b2), k
            assert np.array_equal(b1.cpu().numpy(), dt.step(ts[k])[0]), k
        with pytest.raises(B.DbwError) as e:
            B.dbw_dtur_set_state(h2, visited, nv + 1)
        assert e.value.code == B.ERR_INVALID
        # reset queued on the stream right before the next step, no synchronisation in between
        B.dbw_dtur_reset(h1)
        B.dbw_dtur_b(h1, dev(ts[0]), b1)
        assert np.array_equal(b1.cpu().numpy(), orc.Dtur(rowptr, colidx).step(ts[0])[0])
        assert B.dbw_check(h1) == B.OK
        # every worker dead: no link can be established
        th = torch.zeros(1, device="cuda")
        B.dbw_dtur_b(h1, dev(np.full(n, np.inf, np.float32)), b1, th)
        assert B.dbw_check(h1) == B.WARN_THETA_INF and np.isinf(th.item())
        assert "theta" in B.dbw_strerror(B.WARN_THETA_INF)
        assert B.dbw_check(h1) == B.OK
    finally:
        B.dbw_destroy(h1)
        B.dbw_destroy(h2)


def test_non_finite_row_of_a_backup_worker(B, orc):
    """A worker whose parameters hold inf and that nobody waits for: the sparse path never reads
    its row for the others, so every other row stays finite and equals the oracle; the dense
    path multiplies the row by its zero weights and turns every row into NaN (documented)."""
    rowptr, colidx = inputs.graph_complete(40)
    n, d = 40, 256
    g = np.random.default_rng(717)
    x = g.standard_normal((n, d)).astype(np.float32)
    gr = (g.standard_normal((n, d)) * 0.01).astype(np.float32)
    x[7, 13] = np.inf
    t = g.standard_exponential(n).astype(np.float32)
    t[7] = 1e9                                             # the diverged worker is also the slowest
    b = np.full(n, 5, np.int32)                            # everybody drops its 5 slowest neighbours
    mask, p, _ = orc.select(rowptr, colidx, t, b)
    assert not any(mask[e] for i in range(n) for e in range(rowptr[i], rowptr[i + 1]) if colidx[e] == 7)
    want = orc.round_(rowptr, colidx, mask, p, x, gr, 0.05, 0)
    others = np.arange(n) != 7
    for mix, finite in ((B.MIX_CSR, True), (B.MIX_DENSE, False)):
        h = B.dbw_create(rowptr, colidx, n, d, mix_path=mix)
        try:
            out = torch.zeros((n, d), device="cuda")
            B.dbw_select(h, dev(t), dev(b))
            B.dbw_round(h, dev(x), out, 0.05, ext_grads=dev(gr))
            got = out.cpu().numpy()
            if finite:
                assert np.isfinite(got[others]).all()
                assert_params_close(got[others], want[others], what="sparse path, rows that do not wait for the diverged worker")
                assert np.isinf(got[7, 13])
            else:
                assert np.isnan(got[others][:, 13]).all()   # 0 x inf in column 13 of every row
                assert np.isfinite(np.delete(got[others], 13, axis=1)).all()
        finally:
            B.dbw_destroy(h)
