"""GPU parity of the batched per-worker gradients of fully connected models, and of whole
rounds (gradient + selection + masked average + SGD step) in lock-step with the oracle."""
import numpy as np
import pytest
import torch

from paper_2102_06280_amd import inputs
from gpu_util import GradientResolver, assert_params_close, dev, involved_workers, match_gradients, match_round

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2102_06280_amd import binding
    return binding


def rel_l2(a, b):
    return np.linalg.norm(a.astype(np.float64) - b) / max(np.linalg.norm(b), 1e-30)


SHAPES = [
    # dims, batch, workers, loss
    ([784, 10], 32, 8, "xent"),            # config 1 model
    ([784, 200, 10], 64, 32, "xent"),      # config 2 model
    ([256, 256, 256, 10], 128, 6, "xent"), # the 2NN's layers (Appendix B, Table 1), smaller batch
    ([37, 19, 5], 7, 3, "xent"),           # ragged everything
    ([100, 70, 33, 65, 3], 50, 4, "xent"),
    ([5, 2], 1, 2, "xent"),
    ([256, 256, 256, 10], 1024, 10, "mse"),  # the 2NN as trained in Appendix B
    ([256, 10], 1024, 6, "xent"),            # the LRM of Section 5
    ([37, 19, 5], 7, 3, "mse"),
    ([5, 2], 1, 2, "mse"),
    # batch 32 with wide layers: the streaming kernels (forward split along k or along the outputs,
    # masked data gradient, weight gradient), worker counts that are not multiples of 8
    ([512, 96, 10], 32, 9, "xent"),
    ([1024, 256, 128, 10], 32, 5, "xent"),
    ([64, 512, 64, 10], 32, 11, "xent"),
    ([1536, 384, 10], 32, 3, "mse"),
    # the last layer through the fused head in each of its chunk sizes, with ragged chunks, 16 classes,
    # one class; and around its limits: 20 classes and a 2000-wide last layer take the GEMM kernels
    ([48, 24, 16], 70, 3, "xent"),
    ([30, 1], 5, 2, "xent"),
    ([203, 77, 9], 97, 40, "mse"),
    ([64, 40, 20], 33, 3, "xent"),
    ([2000, 12], 20, 2, "xent"),
    ([1100, 7], 40, 2, "mse"),
]


def check_gradients(B, orc, dims, batch, n, loss_kind, grad_path=0, expect=None):
    g = np.random.default_rng(401)
    desc = {"kind": "mlp", "dims": dims, "loss": loss_kind}
    d = inputs.param_count(desc)
    ld = inputs.pad_ld(d)
    rowptr, colidx = inputs.graph_ring(max(n, 3)) if n >= 3 else (np.array([0, 1, 2], np.int32), np.array([1, 0], np.int32))
    n = rowptr.size - 1
    params = inputs.init_params(desc, n, ld, g)
    params[:, :d] += (g.standard_normal((n, d)) * 0.05).astype(np.float32)      # non-zero biases too
    x = g.standard_normal((n, batch, dims[0])).astype(np.float32)
    y = g.integers(0, dims[-1], (n, batch)).astype(np.int32)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld,
                     model=B.make_model(B.MODEL_MLP, batch, dims, B.LOSS_MSE if loss_kind == "mse" else B.LOSS_XENT,
                                        grad_path=grad_path))
    try:
        grads = torch.full((n, ld), 7.0, dtype=torch.float32, device="cuda")
        loss = torch.zeros(n, dtype=torch.float32, device="cuda")
        B.dbw_set_timing(h, True)
        B.dbw_grad(h, dev(params), dev(x), dev(y), grads, loss)
        kernels = set(B.dbw_get_timing(h))
        B.dbw_set_timing(h, False)
        if expect is not None:
            assert expect <= kernels, kernels
        elif batch == 32 and any(a % 512 == 0 and b % 32 == 0 for a, b in zip(dims[:-1], dims[1:])):
            assert {"fc32_forward", "fc32_wgrad"} <= kernels, kernels       # the streaming kernels really ran
            if any(a % 512 == 0 and b % 32 == 0 for a, b in zip(dims[1:-1], dims[2:])):
                assert "fc32_dgrad" in kernels, kernels
        got, gl = grads.cpu().numpy(), loss.cpu().numpy()
        kind, od = orc.model_desc(desc)
        res = GradientResolver(orc, kind, od, d, params, x, y, threads=min(n, 8))
        assert np.allclose(gl, res.loss, rtol=2e-6, atol=1e-6)
        assert np.all(got[:, d:] == 7.0)

        def layers_close(g_row, w_row, tol=2e-5):
            # every layer's weights and biases: relative L2 error, and the largest element error
            # relative to the layer's largest element
            off = 0
            for fan_in, nw, nb in inputs.layer_shapes(desc):
                for lo, hi in ((off, off + nw), (off + nw, off + nw + nb)):
                    w = w_row[lo:hi].astype(np.float64)
                    diff = g_row[lo:hi] - w
                    if np.linalg.norm(diff) > tol * np.linalg.norm(w) or np.abs(diff).max() > tol * np.abs(w).max():
                        return False
                off += nw + nb
            return True
        match_gradients(res, got, layers_close, d, what=f"dims {dims} batch {batch}")
        print(res.summary())
    finally:
        B.dbw_destroy(h)


@pytest.mark.parametrize("dims,batch,n,loss_kind", SHAPES,
                         ids=[f"{'-'.join(map(str, s[0]))}-B{s[1]}-N{s[2]}-{s[3]}" for s in SHAPES])
def test_mlp_gradients_match_oracle(B, orc, dims, batch, n, loss_kind):
    check_gradients(B, orc, dims, batch, n, loss_kind)


# The chain of layers in one launch (equal hidden widths of 128, 256, 512): one, two and three hidden layers,
# input widths with and without a whole 64-wide k-chunk, ragged last blocks of samples, both losses; batch and
# worker counts chosen so that blocks of 16, 32, 48 and 64 samples are taken ("blocks" below).
CHAIN_SHAPES = [
    # dims, batch, workers, loss, blocks of
    ([64, 128, 10], 50, 3, "xent", 16),
    ([48, 128, 128, 128, 5], 100, 4, "mse", 16),
    ([80, 512, 512, 16], 37, 2, "xent", 16),
    ([784, 256, 256, 10], 70, 5, "xent", 16),
    ([256, 256, 10], 1037, 3, "xent", 16),
    ([128, 128, 128, 10], 509, 10, "mse", 32),
    ([256, 256, 256, 10], 1024, 10, "xent", 48),
    ([64, 512, 512, 10], 1500, 10, "xent", 64),
]


@pytest.mark.parametrize("dims,batch,n,loss_kind,blocks", CHAIN_SHAPES,
                         ids=[f"{'-'.join(map(str, s[0]))}-B{s[1]}-N{s[2]}-{s[3]}" for s in CHAIN_SHAPES])
def test_chain_gradients_match_oracle(B, orc, dims, batch, n, loss_kind, blocks):
    check_gradients(B, orc, dims, batch, n, loss_kind, grad_path=B.GRAD_CHAIN, expect={"mlp_chain_kernel"})


# Layered path with the weight gradients of all layers in one launch (long batches, widths that divide by 4):
# unequal hidden widths and a head with per-chunk sums; more than 16 classes (no head, every bias sum from the
# weight-gradient kernel); one wide layer with 12 outputs (a partial tile of rows), split over the batch.
GROUPED_SHAPES = [
    ([64, 96, 40, 12], 300, 5, "xent"),
    ([64, 40, 20], 260, 3, "xent"),
    ([2000, 12], 256, 2, "mse"),
    ([128, 72, 8], 1000, 2, "mse"),
]


@pytest.mark.parametrize("dims,batch,n,loss_kind", GROUPED_SHAPES,
                         ids=[f"{'-'.join(map(str, s[0]))}-B{s[1]}-N{s[2]}-{s[3]}" for s in GROUPED_SHAPES])
def test_grouped_weight_gradients_match_oracle(B, orc, dims, batch, n, loss_kind):
    check_gradients(B, orc, dims, batch, n, loss_kind, expect={"mlp_wgrad_kernel"})
    check_gradients(B, orc, dims, batch, n, loss_kind, grad_path=B.GRAD_LAYERS, expect={"mlp_wgrad_gemm"})


# Batches of at most 64 samples with widths that divide by 4: forward products and weight gradients straight from
# global memory into matrix-instruction fragments.  One, two, three and four blocks of 16 samples; batches that
# end inside a group of four samples; input widths with a partial chunk of 16 (100, 20) and below one chunk (12);
# output widths with partial tiles of 32 columns and of 64 rows; 20 classes (no fused head: the logits go through
# the same forward kernel without ReLU, and every bias gradient comes from the weight-gradient kernel).
THIN_SHAPES = [
    ([784, 200, 10], 64, 32, "xent"),
    ([100, 72, 36, 68, 3], 50, 4, "xent"),
    ([20, 12, 8], 3, 2, "mse"),
    ([256, 128, 10], 17, 5, "mse"),
    ([64, 40, 20], 33, 3, "xent"),
    ([48, 24, 16], 48, 3, "xent"),
]


@pytest.mark.parametrize("dims,batch,n,loss_kind", THIN_SHAPES,
                         ids=[f"{'-'.join(map(str, s[0]))}-B{s[1]}-N{s[2]}-{s[3]}" for s in THIN_SHAPES])
def test_short_batch_kernels_match_oracle(B, orc, dims, batch, n, loss_kind):
    check_gradients(B, orc, dims, batch, n, loss_kind, expect={"mlp_thin_forward", "mlp_wgrad_kernel"})
    check_gradients(B, orc, dims, batch, n, loss_kind, grad_path=B.GRAD_LAYERS, expect={"mlp_forward_gemm", "mlp_wgrad_gemm"})


def test_chain_falls_back_when_the_batch_is_not_16_byte_aligned(B, orc):
    """The chain kernel fetches the batch with 128-bit loads.  A batch that starts 4 bytes into an allocation takes
    the layered path under DBW_GRAD_AUTO (same gradients), and is refused under DBW_GRAD_CHAIN."""
    dims, batch, n = [256, 256, 256, 10], 1024, 10
    desc = {"kind": "mlp", "dims": dims, "loss": "mse"}
    d = inputs.param_count(desc)
    ld = inputs.pad_ld(d)
    rowptr, colidx = inputs.graph_ring(n)
    g = np.random.default_rng(409)
    params = dev(inputs.init_params(desc, n, ld, g))
    x = g.standard_normal((n, batch, dims[0])).astype(np.float32)
    y = dev(g.integers(0, 10, (n, batch)).astype(np.int32))
    store = torch.zeros(x.size + 1, dtype=torch.float32, device="cuda")
    store[1:] = torch.from_numpy(x.ravel()).cuda()
    shifted = store[1:].view(n, batch, dims[0])
    assert shifted.data_ptr() % 16 == 4
    out = {}
    for name, path, bx in (("aligned", B.GRAD_AUTO, dev(x)), ("shifted", B.GRAD_AUTO, shifted)):
        h = B.dbw_create(rowptr, colidx, n, d, ld=ld, model=B.make_model(B.MODEL_MLP, batch, dims, B.LOSS_MSE, grad_path=path))
        try:
            grads = torch.zeros((n, ld), device="cuda")
            loss = torch.zeros(n, device="cuda")
            B.dbw_set_timing(h, True)
            B.dbw_grad(h, params, bx, y, grads, loss)
            out[name] = (grads.cpu().numpy(), loss.cpu().numpy(), set(B.dbw_get_timing(h)))
        finally:
            B.dbw_destroy(h)
    assert "mlp_chain_kernel" in out["aligned"][2] and "mlp_chain_kernel" not in out["shifted"][2]
    scale = np.abs(out["aligned"][0]).max()
    # two summation orders, and a ReLU unit within rounding of zero may fall either way: a loose bound, the strict
    # comparison with the oracle is test_chain_gradients_match_oracle and test_mlp_gradients_match_oracle
    assert np.abs(out["aligned"][0] - out["shifted"][0]).max() <= 1e-4 * scale
    assert np.allclose(out["aligned"][1], out["shifted"][1], rtol=2e-6)
    h = B.dbw_create(rowptr, colidx, n, d, ld=ld, model=B.make_model(B.MODEL_MLP, batch, dims, B.LOSS_MSE, grad_path=B.GRAD_CHAIN))
    try:
        with pytest.raises(B.DbwError) as e:
            B.dbw_grad(h, params, shifted, y, torch.zeros((n, ld), device="cuda"), torch.zeros(n, device="cuda"))
        assert e.value.code == B.ERR_UNSUPPORTED
    finally:
        B.dbw_destroy(h)


def test_short_batch_kernels_fall_back_when_the_batch_is_not_16_byte_aligned(B, orc):
    """The short-batch kernels fetch the batch with 128-bit loads.  A batch that starts 4 bytes into an allocation
    takes the GEMM kernels for the first layer instead (forward and weight gradient), with the same gradients."""
    dims, batch, n = [784, 200, 10], 64, 8
    desc = {"kind": "mlp", "dims": dims, "loss": "xent"}
    d = inputs.param_count(desc)
    ld = inputs.pad_ld(d)
    rowptr, colidx = inputs.graph_ring(n)
    g = np.random.default_rng(411)
    params = dev(inputs.init_params(desc, n, ld, g))
    x = g.standard_normal((n, batch, dims[0])).astype(np.float32)
    y = dev(g.integers(0, 10, (n, batch)).astype(np.int32))
    store = torch.zeros(x.size + 1, dtype=torch.float32, device="cuda")
    store[1:] = torch.from_numpy(x.ravel()).cuda()
    shifted = store[1:].view(n, batch, dims[0])
    assert shifted.data_ptr() % 16 == 4
    out = {}
    for name, bx in (("aligned", dev(x)), ("shifted", shifted)):
        h = B.dbw_create(rowptr, colidx, n, d, ld=ld, model=B.make_model(B.MODEL_MLP, batch, dims, B.LOSS_XENT))
        try:
            grads = torch.zeros((n, ld), device="cuda")
            loss = torch.zeros(n, device="cuda")
            B.dbw_set_timing(h, True)
            B.dbw_grad(h, params, bx, y, grads, loss)
            out[name] = (grads.cpu().numpy(), loss.cpu().numpy(), set(B.dbw_get_timing(h)))
        finally:
            B.dbw_destroy(h)
    assert {"mlp_thin_forward", "mlp_wgrad_kernel"} <= out["aligned"][2]
    assert not ({"mlp_thin_forward", "mlp_wgrad_kernel"} & out["shifted"][2])
    assert {"mlp_forward_gemm", "mlp_wgrad_gemm"} <= out["shifted"][2]
    scale = np.abs(out["aligned"][0]).max()
    # two summation orders, and a ReLU unit within rounding of zero may fall either way: a loose bound, the strict
    # comparison with the oracle is test_short_batch_kernels_match_oracle
    assert np.abs(out["aligned"][0] - out["shifted"][0]).max() <= 1e-4 * scale
    assert np.allclose(out["aligned"][1], out["shifted"][1], rtol=2e-6)


def test_chain_is_picked_for_the_2nn_and_refused_where_it_cannot_run(B):
    rowptr, colidx = inputs.graph_ring(10)

    def kernels_of(dims, batch, grad_path):
        desc = {"kind": "mlp", "dims": dims, "loss": "mse"}
        d = inputs.param_count(desc)
        ld = inputs.pad_ld(d)
        h = B.dbw_create(rowptr, colidx, 10, d, ld=ld, model=B.make_model(B.MODEL_MLP, batch, dims, B.LOSS_MSE,
                                                                           grad_path=grad_path))
        try:
            B.dbw_set_timing(h, True)
            B.dbw_grad(h, torch.zeros((10, ld), device="cuda"), torch.zeros((10, batch, dims[0]), device="cuda"),
                       torch.zeros((10, batch), dtype=torch.int32, device="cuda"),
                       torch.zeros((10, ld), device="cuda"), torch.zeros(10, device="cuda"))
            return set(B.dbw_get_timing(h))
        finally:
            B.dbw_destroy(h)
    assert "mlp_chain_kernel" in kernels_of([256, 256, 256, 10], 1024, B.GRAD_AUTO)
    assert "mlp_wgrad_kernel" in kernels_of([256, 256, 256, 10], 1024, B.GRAD_AUTO)
    assert "mlp_chain_kernel" not in kernels_of([256, 256, 256, 10], 1024, B.GRAD_LAYERS)
    assert "mlp_chain_kernel" not in kernels_of([256, 256, 256, 10], 16, B.GRAD_AUTO)       # too few blocks to fill the chip
    for dims in ([256, 200, 10], [250, 256, 10], [256, 256, 128, 10], [256, 256, 20], [256, 10]):
        desc = {"kind": "mlp", "dims": dims, "loss": "mse"}
        d = inputs.param_count(desc)
        with pytest.raises(B.DbwError) as e:
            B.dbw_create(rowptr, colidx, 10, d, ld=inputs.pad_ld(d),
                         model=B.make_model(B.MODEL_MLP, 64, dims, B.LOSS_MSE, grad_path=B.GRAD_CHAIN))
        assert e.value.code == B.ERR_UNSUPPORTED, dims


def test_softmax_zero_init_round_one(B, orc):
    """Config 1, round 1: all parameters zero, so every worker's loss is ln 10."""
    cfg = inputs.CONFIGS[1]
    rowptr, colidx = inputs.make_graph(cfg)
    ld = inputs.pad_ld(cfg.d)
    x, y = inputs.batch(cfg, 0)
    h = B.dbw_create(rowptr, colidx, cfg.n, cfg.d, ld=ld, model=B.make_model(B.MODEL_MLP, cfg.batch, [784, 10]))
    try:
        grads = torch.zeros((cfg.n, ld), device="cuda")
        loss = torch.zeros(cfg.n, device="cuda")
        B.dbw_grad(h, torch.zeros((cfg.n, ld), device="cuda"), dev(x), dev(y), grads, loss)
        assert np.allclose(loss.cpu().numpy(), np.log(10.0), rtol=1e-6)
    finally:
        B.dbw_destroy(h)


@pytest.mark.parametrize("cid,rounds,order", [(1, 10, 0), (1, 10, 1), (2, 100, 0), (2, 100, 1)],
                         ids=["config1-cta", "config1-atc", "config2-cta", "config2-atc"])
def test_rounds_lock_step(B, orc, cid, rounds, order):
    """All rounds of configurations 1 and 2 (10 and 100).  Each round both sides start from the
    oracle's previous output, and every worker's parameters must agree to 1e-5 (a row that
    misses the oracle's default evaluation must match its evaluation for one common assignment of
    the ReLU decisions it lists as within rounding of zero).  The free-running GPU trajectory is
    carried along and its drift reported; it is discontinuous in those decisions and not gated
    beyond a sanity bound."""
    cfg = inputs.CONFIGS[cid]
    desc = inputs.model_dims(cfg.model)
    rowptr, colidx = inputs.make_graph(cfg)
    ld = inputs.pad_ld(cfg.d)
    kind, od = orc.model_desc(desc)
    h = B.dbw_create(rowptr, colidx, cfg.n, cfg.d, ld=ld, order=order,
                     model=B.make_model(B.MODEL_MLP, cfg.batch, desc["dims"]))
    try:
        x = inputs.init_params(desc, cfg.n, ld, inputs.rng(cid, inputs.P_PARAMS), zero=cfg.zero_init)
        free = dev(x)
        for rnd in range(rounds):
            t = inputs.response_times(cfg, rnd)
            b = inputs.backup_counts(cfg, rnd, rowptr) if rnd else np.zeros(cfg.n, np.int32)
            bx, by = inputs.batch(cfg, rnd)
            dt, db, dbx, dby = dev(t), dev(b), dev(bx), dev(by)
            out = torch.zeros((cfg.n, ld), device="cuda")
            loss = torch.zeros(cfg.n, device="cuda")
            B.dbw_select(h, dt, db)
            B.dbw_round(h, dev(x), out, cfg.lr, batch_x=dbx, batch_y=dby, loss_out=loss)
            free_out = torch.zeros((cfg.n, ld), device="cuda")
            B.dbw_round(h, free, free_out, cfg.lr, batch_x=dbx, batch_y=dby)
            free = free_out
            mask, p, _ = orc.select(rowptr, colidx, t, b)
            mask_d = torch.empty(colidx.size, dtype=torch.uint8, device="cuda")
            B.dbw_get_selection(h, None, mask_d, None)
            assert np.array_equal(mask_d.cpu().numpy(), mask)
            res = GradientResolver(orc, kind, od, cfg.d, x, bx, by)
            round_fn = lambda grad: orc.round_(rowptr, colidx, mask, p, x, grad, cfg.lr, order, d=cfg.d)
            inv = involved_workers(order, cfg.lr, rowptr, colidx, mask, lambda: orc.weights(rowptr, colidx, mask, p))
            got = out.cpu().numpy()
            want = match_round(res, got, round_fn, inv, cfg.d, what=f"config {cid} round {rnd}")
            assert_params_close(got, want, d=cfg.d, what=f"config {cid} round {rnd}")
            if any(res.resolved.values()):
                print(f"round {rnd}: {res.summary()}", flush=True)
            assert np.allclose(loss.cpu().numpy(), res.loss, rtol=1e-5, atol=1e-6)
            x = want
        drift = rel_l2(free.cpu().numpy()[:, :cfg.d], x[:, :cfg.d])
        print(f"config {cid}: free-running drift after {rounds} rounds: {drift:.2e}")
        assert drift < 0.1
    finally:
        B.dbw_destroy(h)


@pytest.mark.parametrize("cid,order", [(6, 0), (7, 0), (7, 1)], ids=["lrm-cta", "2nn-mse-cta", "2nn-mse-atc"])
def test_paper_models_lock_step(B, orc, cid, order):
    """The experiment shapes of Section 5 / Appendix B (LRM with cross-entropy, 2NN with MSE
    on the softmax outputs, batch 1024, learning rate decayed by 0.95 per round, backup
    counts from the threshold rule, at least one straggler per round) through the Workload
    helper, round by round against the oracle, every worker to 1e-5.  With 1024 x 512 ReLU
    inputs per worker and round, some land within fp32 rounding of zero: a row that misses the
    oracle's default evaluation must match its evaluation for one common assignment of the
    decisions it lists as that close."""
    from paper_2102_06280_amd.workload import Workload
    cfg = inputs.CONFIGS[cid]
    rounds = 8
    wl = Workload(cid, rounds=rounds, order=order)
    try:
        desc = wl.desc
        kind, od = orc.model_desc(desc)
        assert kind == (2 if cid == 7 else 0)
        dt = orc.Dtur(wl.rowptr, wl.colidx)
        x = wl.x[0].cpu().numpy()
        for rnd in range(rounds):
            t = wl.t_host[rnd]
            b = dt.step(t)[0] if rnd else np.zeros(cfg.n, np.int32)
            wl.x[wl.cur].copy_(dev(x))
            wl.step()
            got = wl.params().cpu().numpy()
            bx, by = inputs.batch(cfg, rnd)
            mask, p, _ = orc.select(wl.rowptr, wl.colidx, t, b)
            mask_d = torch.empty(wl.colidx.size, dtype=torch.uint8, device="cuda")
            B.dbw_get_selection(wl.h, None, mask_d, None)
            assert np.array_equal(mask_d.cpu().numpy(), mask), f"round {rnd}"
            lr = inputs.learning_rate(cfg, rnd)
            res = GradientResolver(orc, kind, od, cfg.d, x, bx, by)
            round_fn = lambda grad: orc.round_(wl.rowptr, wl.colidx, mask, p, x, grad, lr, order, d=cfg.d)
            inv = involved_workers(order, lr, wl.rowptr, wl.colidx, mask,
                                   lambda: orc.weights(wl.rowptr, wl.colidx, mask, p))
            want = match_round(res, got, round_fn, inv, cfg.d, what=f"config {cid} round {rnd}")
            assert_params_close(got, want, d=cfg.d, what=f"config {cid} round {rnd}")
            print(f"round {rnd}: {res.summary()}", flush=True)
            assert np.allclose(wl.loss.cpu().numpy(), res.loss, rtol=1e-5, atol=1e-6)
            x = want
        # the decayed step really is in use
        assert inputs.learning_rate(cfg, rounds - 1) == pytest.approx(cfg.lr * 0.95 ** (rounds - 1))
    finally:
        wl.close()


@pytest.mark.parametrize("cid", [2, 7], ids=["config2", "config7-chain-and-threshold-rule"])
def test_graph_replay_matches_eager(B, cid):
    """Rounds captured as HIP graphs (one per round) give the same bits as eager rounds, on
    every replay, with eager work and synchronisations between replays.  Configuration 7 runs the chain kernels
    and the one-launch threshold rule + selection, whose epoch state is put back before every replay."""
    from paper_2102_06280_amd.workload import Workload
    eager = Workload(cid, rounds=6)
    graphed = Workload(cid, rounds=6)
    try:
        for _ in range(6):
            eager.step()
        torch.cuda.synchronize()
        want = eager.params().clone()
        start = graphed.x[0].clone()
        graphs = graphed.capture_steps(6)
        for rep in range(3):
            graphed.x[0].copy_(start)
            graphed.cur, graphed.k = 0, 0
            if graphed.dynamic_b:
                B.dbw_dtur_reset(graphed.h)
            torch.cuda.synchronize()
            graphed.replay(graphs[:3])
            torch.cuda.synchronize()
            scratch = torch.randn(1000, device="cuda").sum().item()     # unrelated eager work in between
            graphed.replay(graphs[3:])
            torch.cuda.synchronize()
            assert torch.equal(graphed.params(), want), f"replay {rep}"
    finally:
        eager.close()
        graphed.close()
