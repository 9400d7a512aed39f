"""Pins for the oracle's mini-batch gradients (Section 2.1, stochastic gradient of the
local loss; cross-entropy loss as in Section 5): central finite differences of an
independently written float64 forward pass, PyTorch CPU autograd on the real shapes,
and the closed form of softmax regression at zero parameters."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from paper_2102_06280_amd import inputs


# ---- independent forward passes (loss only), float64 NumPy

def xent(logits, y):
    z = logits - logits.max(1, keepdims=True)
    logp = z - np.log(np.exp(z).sum(1, keepdims=True))
    return -logp[np.arange(len(y)), y].mean()


def mlp_loss(dims, params, x, y):
    a, off = x.astype(np.float64), 0
    for l in range(len(dims) - 1):
        i, o = dims[l], dims[l + 1]
        W = params[off:off + o * i].reshape(o, i); off += o * i
        b = params[off:off + o]; off += o
        a = a @ W.T + b
        if l + 2 < len(dims):
            a = np.maximum(a, 0)
    return xent(a, y)


def conv_same(x, W, b):
    B, C, H, Wd = x.shape
    K = W.shape[-1]
    pad = K // 2
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    out = np.zeros((B, W.shape[0], H, Wd))
    for kh in range(K):
        for kw in range(K):
            out += np.einsum("bchw,oc->bohw", xp[:, :, kh:kh + H, kw:kw + Wd], W[:, :, kh, kw])
    return out + b[None, :, None, None]


def pool2(x):
    B, C, H, W = x.shape
    return x.reshape(B, C, H // 2, 2, W // 2, 2).max(axis=(3, 5))


def cnn_loss(shape, params, x, y):
    C0, H, W, C1, C2, K, Fc, NC = shape
    params = params.astype(np.float64)
    off = 0
    def take(*s):
        nonlocal off
        n = int(np.prod(s)); v = params[off:off + n].reshape(s); off += n
        return v
    W1, b1 = take(C1, C0, K, K), take(C1)
    W2, b2 = take(C2, C1, K, K), take(C2)
    flat = C2 * (H // 4) * (W // 4)
    W3, b3 = take(Fc, flat), take(Fc)
    W4, b4 = take(NC, Fc), take(NC)
    a = pool2(np.maximum(conv_same(x.astype(np.float64), W1, b1), 0))
    a = pool2(np.maximum(conv_same(a, W2, b2), 0))
    a = np.maximum(a.reshape(len(y), -1) @ W3.T + b3, 0)
    return xent(a @ W4.T + b4, y)


def fd_check(loss_fn, params, grad, n_probe, g, eps=1e-5):
    idx = g.choice(params.size, size=min(n_probe, params.size), replace=False)
    for k in idx:
        pp, pm = params.astype(np.float64).copy(), params.astype(np.float64).copy()
        pp[k] += eps; pm[k] -= eps
        fd = (loss_fn(pp) - loss_fn(pm)) / (2 * eps)
        assert abs(fd - grad[k]) <= 1e-6 + 2e-5 * abs(fd), (k, fd, grad[k])


@pytest.mark.parametrize("dims", [[12, 5], [9, 7, 4], [6, 8, 5, 3]])
def test_mlp_finite_differences(orc, dims):
    g = np.random.default_rng(71)
    d = sum(dims[l + 1] * (dims[l] + 1) for l in range(len(dims) - 1))
    params = (g.standard_normal(d) * 0.5).astype(np.float32)
    x = g.standard_normal((6, dims[0])).astype(np.float32)
    y = g.integers(0, dims[-1], 6).astype(np.int32)
    grad, loss = orc.grad_mlp(dims, params, x, y)
    assert abs(loss - mlp_loss(dims, params.astype(np.float64), x, y)) < 1e-12
    fd_check(lambda p: mlp_loss(dims, p, x, y), params, grad, 200, g)


def test_cnn_finite_differences(orc):
    g = np.random.default_rng(73)
    shape = (2, 8, 8, 3, 4, 3, 6, 5)
    C0, H, W, C1, C2, K, Fc, NC = shape
    d = C1 * C0 * K * K + C1 + C2 * C1 * K * K + C2 + Fc * C2 * (H // 4) * (W // 4) + Fc + NC * Fc + NC
    params = (g.standard_normal(d) * 0.3).astype(np.float32)
    x = g.standard_normal((4, C0, H, W)).astype(np.float32)
    y = g.integers(0, NC, 4).astype(np.int32)
    grad, loss = orc.grad_cnn(shape, params, x, y)
    assert abs(loss - cnn_loss(shape, params, x, y)) < 1e-12
    fd_check(lambda p: cnn_loss(shape, p, x, y), params, grad, 150, g)
    # 5x5 kernels as in the full-size model
    shape = (3, 8, 8, 2, 3, 5, 4, 3)
    C0, H, W, C1, C2, K, Fc, NC = shape
    d = C1 * C0 * K * K + C1 + C2 * C1 * K * K + C2 + Fc * C2 * (H // 4) * (W // 4) + Fc + NC * Fc + NC
    params = (g.standard_normal(d) * 0.3).astype(np.float32)
    x = g.standard_normal((3, C0, H, W)).astype(np.float32)
    y = g.integers(0, NC, 3).astype(np.int32)
    grad, loss = orc.grad_cnn(shape, params, x, y)
    fd_check(lambda p: cnn_loss(shape, p, x, y), params, grad, 150, g)


def test_softmax_zero_init_closed_form(orc):
    """All-zero parameters: logits 0, probabilities 1/10, loss ln 10,
    dW = (1/B) sum_l (1/10 - e_{y_l}) x_l^T, db = (1/B) sum_l (1/10 - e_{y_l})."""
    cfg = inputs.CONFIGS[1]
    x, y = inputs.batch(cfg, 0, workers=[3])
    x, y = x[0], y[0]
    grad, loss = orc.grad_mlp([784, 10], np.zeros(7850, np.float32), x, y)
    assert abs(loss - np.log(10.0)) < 1e-12
    E = np.full((len(y), 10), 0.1)
    E[np.arange(len(y)), y] -= 1.0
    dW = E.T @ x.astype(np.float64) / len(y)
    assert np.allclose(grad[:7840].reshape(10, 784), dW, rtol=1e-6, atol=1e-9)
    assert np.allclose(grad[7840:], E.mean(0), rtol=1e-6, atol=1e-9)


def _torch_mlp_grad(dims, params, x, y):
    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    a, off = torch.tensor(x, dtype=torch.float64), 0
    for l in range(len(dims) - 1):
        i, o = dims[l], dims[l + 1]
        W = p[off:off + o * i].view(o, i); off += o * i
        b = p[off:off + o]; off += o
        a = F.linear(a, W, b)
        if l + 2 < len(dims):
            a = F.relu(a)
    loss = F.cross_entropy(a, torch.tensor(y, dtype=torch.long))
    loss.backward()
    return p.grad.numpy(), float(loss.detach())


@pytest.mark.parametrize("cid", [1, 2])
def test_mlp_matches_autograd_full_shape(orc, cid):
    cfg = inputs.CONFIGS[cid]
    desc = inputs.model_dims(cfg.model)
    params = inputs.init_params(desc, 2, cfg.d, inputs.rng(cid, inputs.P_PARAMS))[1]
    x, y = inputs.batch(cfg, 0, workers=[1])
    grad, loss = orc.grad_mlp(desc["dims"], params, x[0], y[0])
    want, wl = _torch_mlp_grad(desc["dims"], params, x[0], y[0])
    assert abs(loss - wl) < 1e-10
    assert np.allclose(grad, want, rtol=1e-6, atol=1e-9)


def test_cnn_matches_autograd_full_shape(orc):
    cfg = inputs.CONFIGS[3]
    desc = inputs.model_dims("cnn")
    params = inputs.init_params(desc, 1, cfg.d, inputs.rng(3, inputs.P_PARAMS))[0]
    x, y = inputs.batch(cfg, 0, workers=[0])
    x, y = x[0][:4], y[0][:4]              # 4 samples keep the direct loops to a few seconds
    shape = (3, 32, 32, 32, 64, 5, 512, 10)
    grad, loss = orc.grad_cnn(shape, params, x, y)
    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    off = 0
    def take(*s):
        nonlocal off
        n = int(np.prod(s)); v = p[off:off + n].view(*s); off += n
        return v
    W1, b1, W2, b2 = take(32, 3, 5, 5), take(32), take(64, 32, 5, 5), take(64)
    W3, b3, W4, b4 = take(512, 4096), take(512), take(10, 512), take(10)
    a = torch.tensor(x, dtype=torch.float64).view(-1, 3, 32, 32)
    a = F.max_pool2d(F.relu(F.conv2d(a, W1, b1, padding=2)), 2)
    a = F.max_pool2d(F.relu(F.conv2d(a, W2, b2, padding=2)), 2)
    a = F.relu(F.linear(a.flatten(1), W3, b3))
    l = F.cross_entropy(F.linear(a, W4, b4), torch.tensor(y, dtype=torch.long))
    l.backward()
    assert abs(loss - float(l)) < 1e-10
    assert np.allclose(grad, p.grad.numpy(), rtol=1e-6, atol=1e-9)


def test_grad_all_rows_and_padding(orc):
    """orc.grad_all = the single-worker routine applied row by row, padding zeroed."""
    dims = [10, 6, 4]
    d = 6 * 11 + 4 * 7
    g = np.random.default_rng(79)
    n, ld, B = 3, 96, 5
    params = np.zeros((n, ld), np.float32)
    params[:, :d] = g.standard_normal((n, d))
    x = g.standard_normal((n, B, 10)).astype(np.float32)
    y = g.integers(0, 4, (n, B)).astype(np.int32)
    kind, desc = orc.model_desc({"kind": "mlp", "dims": dims})
    grad, loss = orc.grad_all(kind, desc, d, params, x, y)
    assert not grad[:, d:].any()
    for i in range(n):
        gi, li = orc.grad_mlp(dims, params[i, :d], x[i], y[i])
        assert np.array_equal(grad[i, :d], gi) and loss[i] == li


U = 2.0 ** -24


def test_near_decisions_of_fully_connected_layers(orc):
    """The decisions listed next to the gradients: every hidden ReLU whose |z| is below
    near_scale rounding units (2^-24 times |bias| + sum |w a|, recomputed here with NumPy),
    with the opposite outcome as `alt`, and nothing else."""
    dims = [9, 7, 6, 4]
    g = np.random.default_rng(83)
    d = sum(dims[l + 1] * (dims[l] + 1) for l in range(3))
    params = np.zeros((2, 192), np.float32)
    params[:, :d] = g.standard_normal((2, d)) * 0.5
    x = g.standard_normal((2, 5, 9)).astype(np.float32)
    y = g.integers(0, 4, (2, 5)).astype(np.int32)
    kind, desc = orc.model_desc({"kind": "mlp", "dims": dims})
    scale = 3e6                                       # wide enough to list about a third of the units
    grad, _, near = orc.grad_all(kind, desc, d, params, x, y, near_scale=scale)
    assert np.array_equal(grad, orc.grad_all(kind, desc, d, params, x, y)[0])      # listing changes nothing
    for i in range(2):
        a, off, want = x[i].astype(np.float64), 0, {}
        for l in range(2):
            o, k = dims[l + 1], dims[l]
            W = params[i, off:off + o * k].reshape(o, k).astype(np.float64); off += o * k
            b = params[i, off:off + o].astype(np.float64); off += o
            z = a @ W.T + b
            gap = np.abs(z) / (U * (np.abs(a) @ np.abs(W).T + np.abs(b)))
            for s_, u_ in zip(*np.nonzero(gap < scale)):
                want[(16 + l, int(s_), int(u_), int(z[s_, u_] <= 0))] = gap[s_, u_]
            a = np.maximum(z, 0)
        got = {e.key(): e.gap for e in near[i]}
        assert 10 < len(want) < 60 and set(got) == set(want)
        assert all(abs(got[k] - want[k]) <= 1e-9 * want[k] for k in want)


def _cnn_forward_numpy(shape, params, x):
    """Pre-activations of both convolutional stages and of the first fully connected layer,
    with their rounding units, through the independent forward pass of this file."""
    C0, H, W, C1, C2, K, Fc, NC = shape
    p = params.astype(np.float64)
    off = 0
    def take(*s):
        nonlocal off
        n = int(np.prod(s)); v = p[off:off + n].reshape(s); off += n
        return v
    W1, b1, W2, b2 = take(C1, C0, K, K), take(C1), take(C2, C1, K, K), take(C2)
    flat = C2 * (H // 4) * (W // 4)
    W3, b3 = take(Fc, flat), take(Fc)
    xi = x.reshape(-1, C0, H, W).astype(np.float64)
    z1, m1 = conv_same(xi, W1, b1), conv_same(np.abs(xi), np.abs(W1), np.abs(b1))
    p1 = pool2(np.maximum(z1, 0))
    z2, m2 = conv_same(p1, W2, b2), conv_same(np.abs(p1), np.abs(W2), np.abs(b2))
    p2 = pool2(np.maximum(z2, 0)).reshape(len(xi), -1)
    z3, m3 = p2 @ W3.T + b3, np.abs(p2) @ np.abs(W3).T + np.abs(b3)
    return (z1, m1), (z2, m2), (z3, m3)


def test_near_decisions_of_pooling_windows(orc):
    """Listed decisions of a small convolutional network against a brute-force walk over all
    windows: with a positive maximum, every other position closer to it than the bound (gap =
    difference over the two rounding units) and the maximum's own distance from zero; with no
    positive value, every position's distance from zero."""
    shape = (2, 8, 8, 3, 4, 3, 6, 5)
    g = np.random.default_rng(85)
    desc = {"kind": "cnn", "in": (2, 8, 8), "c1": 3, "c2": 4, "k": 3, "fc": 6, "classes": 5}
    d = inputs.param_count(desc)
    params = inputs.init_params(desc, 1, d, g)[0] + (g.standard_normal(d) * 0.05).astype(np.float32)
    x = g.standard_normal((3, 2 * 8 * 8)).astype(np.float32)
    y = g.integers(0, 5, 3).astype(np.int32)
    scale = 1.5e6
    grad, loss, near = orc.grad_cnn(shape, params, x, y, near_scale=scale)
    assert np.array_equal(grad, orc.grad_cnn(shape, params, x, y)[0])
    stages = _cnn_forward_numpy(shape, params, x)
    want = {}
    for stage, (z, m) in enumerate(stages[:2]):
        B_, C_, H_, W_ = z.shape
        for s_ in range(B_):
            for c in range(C_):
                for oh in range(H_ // 2):
                    for ow in range(W_ // 2):
                        unit = (c * (H_ // 2) + oh) * (W_ // 2) + ow
                        win = [(z[s_, c, 2 * oh + q // 2, 2 * ow + q % 2], m[s_, c, 2 * oh + q // 2, 2 * ow + q % 2])
                               for q in range(4)]
                        top = max(range(4), key=lambda q: (win[q][0], -q))
                        if win[top][0] > 0:
                            for q in range(4):
                                if q != top:
                                    want[(stage, s_, unit, q)] = (win[top][0] - win[q][0]) / (U * (win[top][1] + win[q][1]))
                            want[(stage, s_, unit, 4)] = win[top][0] / (U * win[top][1])
                        else:
                            for q in range(4):
                                want[(stage, s_, unit, q)] = -win[q][0] / (U * win[q][1])
    z3, m3 = stages[2]
    for s_ in range(z3.shape[0]):
        for o in range(z3.shape[1]):
            want[(16, s_, o, int(z3[s_, o] <= 0))] = abs(z3[s_, o]) / (U * m3[s_, o])
    want = {k: v for k, v in want.items() if v < scale}
    got = {e.key(): e.gap for e in near}
    assert len(want) > 20 and set(got) == set(want)
    assert all(abs(got[k] - want[k]) <= 1e-9 * max(want[k], 1e-300) for k in want)


def _straight_through_relu(z, on):
    """Forward relu(z) where `on`, else 0; gradient 1 where `on`, whatever the sign of z."""
    return (z - z.detach() + F.relu(z).detach()) * on


def test_flipped_relu_decisions_match_autograd(orc):
    """Gradient with chosen ReLU decisions taken the other way = autograd of the same network
    with those units forced active / inactive for those samples."""
    dims = [9, 7, 6, 4]
    g = np.random.default_rng(87)
    d = sum(dims[l + 1] * (dims[l] + 1) for l in range(3))
    params = (g.standard_normal(d) * 0.5).astype(np.float32)
    x = g.standard_normal((5, 9)).astype(np.float32)
    y = g.integers(0, 4, 5).astype(np.int32)
    for loss_kind in ("xent", "mse"):
        _, _, near = orc.grad_mlp(dims, params, x, y, loss_kind=loss_kind, near_scale=1e9)
        assert len(near) == 5 * 13                      # every hidden unit of every sample
        flips = [near[k] for k in (0, 7, 20, 33, 64)]
        grad, loss = orc.grad_mlp(dims, params, x, y, loss_kind=loss_kind, flips=flips)
        p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
        a, off = torch.tensor(x, dtype=torch.float64), 0
        for l in range(3):
            i, o = dims[l], dims[l + 1]
            Wt = p[off:off + o * i].view(o, i); off += o * i
            bt = p[off:off + o]; off += o
            z = F.linear(a, Wt, bt)
            if l < 2:
                on = (z > 0).to(torch.float64)
                for f in flips:
                    if f.stage == 16 + l:
                        on[f.sample, f.unit] = float(f.alt)
                a = _straight_through_relu(z, on)
        if loss_kind == "xent":
            lt = F.cross_entropy(z, torch.tensor(y, dtype=torch.long))
        else:
            target = F.one_hot(torch.tensor(y, dtype=torch.long), 4).to(torch.float64)
            lt = F.mse_loss(F.softmax(z, 1), target, reduction="sum") / len(y)
        lt.backward()
        assert abs(loss - float(lt.detach())) < 1e-12
        assert np.allclose(grad, p.grad.numpy(), rtol=1e-6, atol=1e-10)
        base = orc.grad_mlp(dims, params, x, y, loss_kind=loss_kind)[0]
        assert np.abs(grad - base).max() > 1e-3         # the flips did change the gradient


def test_flipped_pooling_decisions_match_autograd(orc):
    """The same for the convolutional network: a window forced to hand its gradient to another
    position, or to none; a fully connected ReLU forced on."""
    shape = (2, 8, 8, 3, 4, 3, 6, 5)
    C0, H, W, C1, C2, K, Fc, NC = shape
    g = np.random.default_rng(91)
    desc = {"kind": "cnn", "in": (2, 8, 8), "c1": 3, "c2": 4, "k": 3, "fc": 6, "classes": 5}
    d = inputs.param_count(desc)
    params = inputs.init_params(desc, 1, d, g)[0] + (g.standard_normal(d) * 0.05).astype(np.float32)
    x = g.standard_normal((3, C0 * H * W)).astype(np.float32)
    y = g.integers(0, 5, 3).astype(np.int32)
    _, _, near = orc.grad_cnn(shape, params, x, y, near_scale=1e12)
    by_stage = {st: [e for e in near if e.stage == st] for st in (0, 1, 16)}
    pick = lambda lst, alt, skip=0: [e for e in lst if (e.alt == 4) == (alt == 4)][skip]
    flips = [pick(by_stage[0], 0), pick(by_stage[0], 4, 3), pick(by_stage[1], 0, 2), pick(by_stage[1], 4, 1),
             by_stage[16][4]]
    assert len({(f.stage, f.sample, f.unit) for f in flips}) == 5
    grad, loss = orc.grad_cnn(shape, params, x, y, flips=flips)

    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    off = 0
    def take(*s):
        nonlocal off
        n = int(np.prod(s)); v = p[off:off + n].view(*s); off += n
        return v
    W1, b1, W2, b2 = take(C1, C0, K, K), take(C1), take(C2, C1, K, K), take(C2)
    W3, b3, W4, b4 = take(Fc, C2 * (H // 4) * (W // 4)), take(Fc), take(NC, Fc), take(NC)

    def stage(inp, Wc, bc, st):
        z = F.conv2d(inp, Wc, bc, padding=K // 2)
        B_, C_, H_, W_ = z.shape
        win = z.view(B_, C_, H_ // 2, 2, W_ // 2, 2).permute(0, 1, 2, 4, 3, 5).reshape(B_, C_, H_ // 2, W_ // 2, 4)
        arg = torch.relu(win).detach().argmax(dim=-1, keepdim=True)     # first maximum in window order
        on = (win.detach().gather(-1, arg) > 0).to(torch.float64)
        for f in flips:
            if f.stage == st:
                c, r = divmod(f.unit, (H_ // 2) * (W_ // 2))
                oh, ow = divmod(r, W_ // 2)
                on[f.sample, c, oh, ow, 0] = 0.0 if f.alt == 4 else 1.0
                if f.alt != 4:
                    arg[f.sample, c, oh, ow, 0] = f.alt
        return _straight_through_relu(win.gather(-1, arg), on).squeeze(-1)

    a = torch.tensor(x, dtype=torch.float64).view(-1, C0, H, W)
    a = stage(a, W1, b1, 0)
    a = stage(a, W2, b2, 1).reshape(len(x), -1)
    z3 = F.linear(a, W3, b3)
    on3 = (z3 > 0).to(torch.float64)
    for f in flips:
        if f.stage == 16:
            on3[f.sample, f.unit] = float(f.alt)
    z4 = F.linear(_straight_through_relu(z3, on3), W4, b4)
    lt = F.cross_entropy(z4, torch.tensor(y, dtype=torch.long))
    lt.backward()
    assert abs(loss - float(lt.detach())) < 1e-12
    assert np.allclose(grad, p.grad.numpy(), rtol=1e-6, atol=1e-10)
    assert np.abs(grad - orc.grad_cnn(shape, params, x, y)[0]).max() > 1e-4


def mlp_mse_loss(dims, params, x, y):
    a, off = x.astype(np.float64), 0
    for l in range(len(dims) - 1):
        i, o = dims[l], dims[l + 1]
        W = params[off:off + o * i].reshape(o, i); off += o * i
        b = params[off:off + o]; off += o
        a = a @ W.T + b
        if l + 2 < len(dims):
            a = np.maximum(a, 0)
    z = a - a.max(1, keepdims=True)
    p = np.exp(z) / np.exp(z).sum(1, keepdims=True)
    p[np.arange(len(y)), y] -= 1.0
    return (p ** 2).sum(1).mean()


@pytest.mark.parametrize("dims", [[12, 5], [9, 7, 4], [6, 8, 5, 3]])
def test_mlp_mse_finite_differences(orc, dims):
    """MSE on the softmax outputs (Appendix B, 2NN): loss value against an independent NumPy
    forward pass, gradient against central differences of it."""
    g = np.random.default_rng(89)
    d = sum(dims[l + 1] * (dims[l] + 1) for l in range(len(dims) - 1))
    params = (g.standard_normal(d) * 0.5).astype(np.float32)
    x = g.standard_normal((6, dims[0])).astype(np.float32)
    y = g.integers(0, dims[-1], 6).astype(np.int32)
    grad, loss = orc.grad_mlp(dims, params, x, y, loss_kind="mse")
    assert abs(loss - mlp_mse_loss(dims, params.astype(np.float64), x, y)) < 1e-12
    fd_check(lambda p: mlp_mse_loss(dims, p, x, y), params, grad, 200, g)


def test_2nn_mse_matches_autograd(orc):
    """The paper's 2NN (Appendix B, Table 1: 256-256-256-10, softmax outputs, MSE loss)."""
    dims = [256, 256, 256, 10]
    g = np.random.default_rng(97)
    desc = {"kind": "mlp", "dims": dims}
    params = inputs.init_params(desc, 1, inputs.param_count(desc), g)[0]
    x = g.standard_normal((64, 256)).astype(np.float32)
    y = g.integers(0, 10, 64).astype(np.int32)
    grad, loss = orc.grad_mlp(dims, params, x, y, loss_kind="mse")
    p = torch.tensor(params, dtype=torch.float64, requires_grad=True)
    a, off = torch.tensor(x, dtype=torch.float64), 0
    for l in range(3):
        i, o = dims[l], dims[l + 1]
        W = p[off:off + o * i].view(o, i); off += o * i
        b = p[off:off + o]; off += o
        a = F.linear(a, W, b)
        if l < 2:
            a = F.relu(a)
    target = F.one_hot(torch.tensor(y, dtype=torch.long), 10).to(torch.float64)
    l = F.mse_loss(F.softmax(a, 1), target, reduction="sum") / len(y)
    l.backward()
    assert abs(loss - float(l.detach())) < 1e-12
    assert np.allclose(grad, p.grad.numpy(), rtol=1e-6, atol=1e-10)
