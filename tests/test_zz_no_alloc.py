"""GPU test of dbw_consensus_rounds_static, the entry point for callers that cannot allocate:
its output against dbw_consensus_rounds on a context of the same graph, on two calls in a row
that share the library's fixed device array, the second with a smaller problem."""
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


def _case(B, rowptr, colidx, d, ld, r, seed, bad_b=False):
    n = rowptr.size - 1
    deg = np.diff(rowptr)
    g = np.random.default_rng(seed)
    x = g.standard_normal((n, ld)).astype(np.float32)
    t = g.standard_exponential((r, n)).astype(np.float32)
    t[0] = np.round(t[0] * 4) / 4
    b = np.stack([g.integers(0, deg + 1) for _ in range(r)]).astype(np.int32)
    if bad_b:
        b[r - 1, 0] = deg[0] + 3
    dx, dt, db = dev(x), dev(t), dev(b)
    # existing entry point on a context
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, mix_path=B.MIX_CSR)
    try:
        want = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
        B.dbw_consensus_rounds(h, dx, want, dt, db, r)
        torch.cuda.synchronize()
    finally:
        B.dbw_destroy(h)
    return n, dx, dt, db, want


def _static(B, n, d, ld, rowptr, colidx, dx, dt, db, r):
    drow = dev(rowptr.astype(np.int32))
    dcol = dev(colidx.astype(np.int32)) if colidx.size else torch.zeros(0, dtype=torch.int32, device="cuda")
    out = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
    status = torch.full((1,), 99, dtype=torch.int32, device="cuda")
    B.dbw_consensus_rounds_static(n, d, ld, drow, dcol, dx, out, dt, db, r, status)
    torch.cuda.synchronize()
    return out, int(status.item())


def test_static_entry_matches_context_entry_on_two_calls_in_a_row(B):
    g = np.random.default_rng(901)
    big = inputs.graph_complete(200)                 # padded to 256 workers, 39 800 links
    small = inputs.graph_er(40, 0.2, g)              # padded to 64: lies inside what the first call left behind
    for (rowptr, colidx), d, ld, r, seed in [(big, 5003, 5056, 5, 11), (small, 1001, 1008, 3, 12),
                                             (small, 999, 999, 2, 13)]:      # the last: unaligned rows, scalar kernel
        n, dx, dt, db, want = _case(B, rowptr, colidx, d, ld, r, seed)
        got, status = _static(B, n, d, ld, rowptr, colidx, dx, dt, db, r)
        assert status == B.OK
        assert torch.equal(got, want), f"N={n} d={d}: max diff {(got - want).abs().max().item():.3e}"
        assert_params_close(got.cpu().numpy(), want.cpu().numpy(), d=d, what=f"static N={n}")
        assert torch.all(got[:, d:] == 7.0)


def test_static_entry_status_and_limits(B):
    rowptr, colidx = inputs.graph_ring(8)
    n, d, ld, r = 8, 64, 64, 2
    _, dx, dt, db, want = _case(B, rowptr, colidx, d, ld, r, 21, bad_b=True)
    got, status = _static(B, n, d, ld, rowptr, colidx, dx, dt, db, r)
    assert status == B.ERR_INVALID                    # out-of-range backup count: clamped and reported
    assert torch.equal(got, want)
    # an asymmetric graph is refused on the device: parameters pass through unchanged
    bad_col = colidx.copy()
    bad_col[0] = 3                                    # row 0 lists worker 3, row 3 does not list worker 0
    bad_col[:2] = np.sort(bad_col[:2])
    zero_b = torch.zeros((r, n), dtype=torch.int32, device="cuda")
    got, status = _static(B, n, d, ld, rowptr, bad_col, dx, dt, zero_b, r)
    assert status == B.ERR_GRAPH
    assert torch.equal(got[:, :d], dx[:, :d])
    # every way a graph can be wrong is caught by the staging kernel, and the parameters pass through
    bad_graphs = {
        "self loop": (rowptr, np.where(np.arange(colidx.size) == 0, 0, colidx)),
        "out of range": (rowptr, np.where(np.arange(colidx.size) == 5, 99, colidx)),
        "negative index": (rowptr, np.where(np.arange(colidx.size) == 5, -1, colidx)),
        "row not ascending": (rowptr, np.concatenate([colidx[:2][::-1], colidx[2:]])),
        "offsets decrease": (np.concatenate([rowptr[:3], [rowptr[3] - 3], rowptr[4:]]), colidx),
        "offsets do not start at zero": (np.concatenate([[1], rowptr[1:]]), colidx),
        "last offset is not the number of entries": (np.concatenate([rowptr[:-1], [rowptr[-1] - 1]]), colidx),
    }
    for what, (rp_bad, ci_bad) in bad_graphs.items():
        got, status = _static(B, n, d, ld, rp_bad.astype(np.int32), ci_bad.astype(np.int32), dx, dt, zero_b, r)
        assert status == B.ERR_GRAPH, what
        assert torch.equal(got[:, :d], dx[:, :d]), what
    # host-side limits and argument checks
    x = torch.zeros((300, 64), device="cuda")
    y = torch.zeros((300, 64), device="cuda")
    rp, ci = inputs.graph_ring(300)
    tt, bb = torch.ones((1, 300), device="cuda"), torch.zeros((1, 300), dtype=torch.int32, device="cuda")
    with pytest.raises(B.DbwError) as e:
        B.dbw_consensus_rounds_static(300, 64, 64, dev(rp), dev(ci), x, y, tt, bb, 1)
    assert e.value.code == B.ERR_UNSUPPORTED
    with pytest.raises(B.DbwError) as e:
        B.dbw_consensus_rounds_static(8, 64, 64, dev(rowptr), dev(colidx), dx, dx, dt, db, r)
    assert e.value.code == B.ERR_ALIAS
    with pytest.raises(B.DbwError) as e:
        B.dbw_consensus_rounds_static(8, 64, 32, dev(rowptr), dev(colidx), dx, y, dt, db, r)
    assert e.value.code == B.ERR_INVALID


def test_static_entry_under_graph_capture(B):
    """The entry point is meant for callers that record their work into a HIP graph: capture one
    call, replay it several times with unrelated eager work and synchronisations in between, and
    compare every replay with the eager result (new response times are written into the same
    device arrays between replays)."""
    rowptr, colidx = inputs.graph_regular(64, 6, np.random.default_rng(905))
    n, d, ld, r = 64, 3001, 3008, 4
    g = np.random.default_rng(906)
    deg = np.diff(rowptr)
    x = dev(g.standard_normal((n, ld)).astype(np.float32))
    drow, dcol = dev(rowptr.astype(np.int32)), dev(colidx.astype(np.int32))
    t = torch.zeros((r, n), dtype=torch.float32, device="cuda")
    b = torch.zeros((r, n), dtype=torch.int32, device="cuda")
    out = torch.zeros((n, ld), dtype=torch.float32, device="cuda")
    status = torch.zeros(1, dtype=torch.int32, device="cuda")

    def fresh_inputs():
        t.copy_(dev(g.standard_exponential((r, n)).astype(np.float32)))
        b.copy_(dev(np.stack([g.integers(0, deg + 1) for _ in range(r)]).astype(np.int32)))

    fresh_inputs()
    B.dbw_consensus_rounds_static(n, d, ld, drow, dcol, x, out, t, b, r, status)    # set-up happens outside the capture
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        B.dbw_consensus_rounds_static(n, d, ld, drow, dcol, x, out, t, b, r, status)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, mix_path=B.MIX_CSR)
    try:
        for rep in range(3):
            fresh_inputs()
            out.fill_(7.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            _ = torch.randn(1000, device="cuda").sum().item()              # unrelated eager work in between
            want = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
            B.dbw_consensus_rounds(h, x, want, t, b, r)
            torch.cuda.synchronize()
            assert int(status.item()) == B.OK
            assert torch.equal(out, want), f"replay {rep}"
    finally:
        B.dbw_destroy(h)
