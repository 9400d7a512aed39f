"""Seeded synthetic inputs: communication graphs, initial parameters, mini-batches,
response times and backup counts.

This module draws numbers and builds graph index arrays; it contains none of the
method's arithmetic (no selection, no mixing weights, no averaging, no gradients), so
that the checker and the GPU library can both be fed from it without sharing any
computation.  Everything is NumPy on the host; callers copy to the device.

The shapes stand in for the paper's MNIST / CIFAR-10 experiments (Section 5 and
Appendix B: 784-dimensional grey images, 3x32x32 colour images, 10 classes); none of
those datasets' records are used.
"""
from __future__ import annotations

import dataclasses
import numpy as np

SEED = 210206280

# purpose ids of the independent random streams
P_GRAPH, P_PARAMS, P_GRADS, P_BATCH_X, P_BATCH_Y, P_TIMES, P_BACKUP, P_SLOW, P_TEACHER = range(1, 10)


def rng(config: int, purpose: int, rnd: int = 0) -> np.random.Generator:
    """Counter-based generator keyed by (seed, config, purpose, round)."""
    stream = ((config * 1000 + purpose) << 32) | (rnd & 0xFFFFFFFF)
    return np.random.Generator(np.random.Philox(key=[SEED, stream]))


# --------------------------------------------------------------------------- graphs

def _csr_from_adj(adj: np.ndarray):
    n = adj.shape[0]
    rowptr = np.zeros(n + 1, dtype=np.int32)
    cols = []
    for i in range(n):
        nb = np.flatnonzero(adj[i]).astype(np.int32)
        cols.append(nb)
        rowptr[i + 1] = rowptr[i] + nb.size
    colidx = np.concatenate(cols).astype(np.int32) if n else np.zeros(0, np.int32)
    return rowptr, colidx


def _connected(adj: np.ndarray) -> bool:
    n = adj.shape[0]
    seen = np.zeros(n, dtype=bool)
    stack = [0]
    seen[0] = True
    while stack:
        u = stack.pop()
        for v in np.flatnonzero(adj[u]):
            if not seen[v]:
                seen[v] = True
                stack.append(int(v))
    return bool(seen.all())


def graph_ring(n: int):
    adj = np.zeros((n, n), dtype=bool)
    for i in range(n):
        adj[i, (i + 1) % n] = adj[(i + 1) % n, i] = True
    np.fill_diagonal(adj, False)
    return _csr_from_adj(adj)


def graph_complete(n: int):
    adj = np.ones((n, n), dtype=bool)
    np.fill_diagonal(adj, False)
    return _csr_from_adj(adj)


def graph_regular(n: int, k: int, g: np.random.Generator):
    """Random simple connected k-regular graph: a circulant k-regular graph randomised by
    degree-preserving double edge swaps (a-b, c-d -> a-d, c-b), redone until connected."""
    assert (n * k) % 2 == 0 and k < n
    while True:
        adj = np.zeros((n, n), dtype=bool)
        for i in range(n):
            for s in range(1, k // 2 + 1):
                adj[i, (i + s) % n] = adj[(i + s) % n, i] = True
            if k % 2:
                adj[i, (i + n // 2) % n] = adj[(i + n // 2) % n, i] = True
        edges = [(i, j) for i in range(n) for j in range(i + 1, n) if adj[i, j]]
        m = len(edges)
        picks = g.integers(0, m, size=(20 * m, 2))
        flips = g.integers(0, 2, size=20 * m)
        for (e1, e2), f in zip(picks, flips):
            a, b = edges[e1]
            c, d = edges[e2]
            if f:
                c, d = d, c
            if len({a, b, c, d}) < 4 or adj[a, d] or adj[c, b]:
                continue
            adj[a, b] = adj[b, a] = adj[c, d] = adj[d, c] = False
            adj[a, d] = adj[d, a] = adj[c, b] = adj[b, c] = True
            edges[e1], edges[e2] = (a, d), (c, b)
        assert np.all(adj.sum(1) == k)
        if _connected(adj):
            return _csr_from_adj(adj)


def graph_er(n: int, p: float, g: np.random.Generator):
    """Erdos-Renyi G(n, p), redrawn until connected."""
    while True:
        upper = np.triu(g.random((n, n)) < p, k=1)
        adj = upper | upper.T
        if _connected(adj):
            return _csr_from_adj(adj)


def graph_random_connected(n: int, p: float, g: np.random.Generator):
    return graph_er(n, p, g)


# --------------------------------------------------------------------------- models

def model_dims(model: str):
    """Layer description per model name; parameter layout inside a worker's row is
    layer by layer, weight [out][in] (conv [Cout][Cin][kh][kw]) then bias."""
    if model == "softmax":
        return {"kind": "mlp", "dims": [784, 10]}
    if model == "mlp":
        return {"kind": "mlp", "dims": [784, 200, 10]}
    if model == "2nn":  # Appendix B, Table 1 (inputs already reduced to 256 dims), MSE loss
        return {"kind": "mlp", "dims": [256, 256, 256, 10], "loss": "mse"}
    if model == "lrm":  # Section 5: logistic regression on 256 reduced dimensions, cross-entropy
        return {"kind": "mlp", "dims": [256, 10]}
    if model == "cnn":
        return {"kind": "cnn", "in": (3, 32, 32), "c1": 32, "c2": 64, "k": 5, "fc": 512, "classes": 10}
    raise ValueError(model)


def param_count(desc) -> int:
    if desc["kind"] == "mlp":
        dims = desc["dims"]
        return sum(dims[l + 1] * dims[l] + dims[l + 1] for l in range(len(dims) - 1))
    c, h, w = desc["in"]
    k = desc["k"]
    flat = desc["c2"] * (h // 4) * (w // 4)
    return (desc["c1"] * c * k * k + desc["c1"] + desc["c2"] * desc["c1"] * k * k + desc["c2"]
            + desc["fc"] * flat + desc["fc"] + desc["classes"] * desc["fc"] + desc["classes"])


def layer_shapes(desc):
    """[(fan_in, n_weights, n_bias)] in layout order."""
    if desc["kind"] == "mlp":
        dims = desc["dims"]
        return [(dims[l], dims[l + 1] * dims[l], dims[l + 1]) for l in range(len(dims) - 1)]
    c, h, w = desc["in"]
    k = desc["k"]
    flat = desc["c2"] * (h // 4) * (w // 4)
    return [(c * k * k, desc["c1"] * c * k * k, desc["c1"]),
            (desc["c1"] * k * k, desc["c2"] * desc["c1"] * k * k, desc["c2"]),
            (flat, desc["fc"] * flat, desc["fc"]),
            (desc["fc"], desc["classes"] * desc["fc"], desc["classes"])]


def init_params(desc, n_workers: int, ld: int, g: np.random.Generator, zero: bool = False):
    """[N, ld] fp32; Kaiming-normal weights (std = sqrt(2 / fan_in)), zero biases, drawn
    independently per worker; padding columns [d, ld) are zero."""
    d = param_count(desc)
    out = np.zeros((n_workers, ld), dtype=np.float32)
    if zero:
        return out
    for i in range(n_workers):
        off = 0
        for fan_in, nw, nb in layer_shapes(desc):
            out[i, off:off + nw] = g.standard_normal(nw, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))
            off += nw + nb
        assert off == d
    return out


# --------------------------------------------------------------------------- configs

@dataclasses.dataclass
class Config:
    cid: int
    name: str
    n: int
    graph: str            # ring | regular | er | complete
    graph_arg: float
    model: str            # softmax | mlp | cnn | none | 2nn
    d: int
    batch: int
    lr: float
    rounds: int
    times: str            # exp | shifted_exp | lognormal_slow
    backup: str           # const | uniform | dtur
    backup_arg: int
    x_dist: str = "normal"   # batch input distribution: uniform | normal
    zero_init: bool = False
    lr_decay: float = 1.0    # lr(k) = lr * lr_decay ** k (Section 5: 0.95)
    labels: str = "uniform"  # uniform: labels independent of the inputs | teacher: a learnable rule


CONFIGS = {
    1: Config(1, "ring8-softmax", 8, "ring", 0, "softmax", 7850, 32, 0.05, 10, "exp", "const", 1,
              x_dist="uniform", zero_init=True),
    2: Config(2, "reg4x32-mlp", 32, "regular", 4, "mlp", 159010, 64, 0.05, 100, "shifted_exp", "uniform", 2),
    3: Config(3, "er64-cnn", 64, "er", 0.1, "cnn", 2156490, 32, 0.01, 50, "lognormal_slow", "dtur", 0),
    4: Config(4, "reg8x128-consensus", 128, "regular", 8, "none", 11_200_000, 0, 0.05, 20, "exp", "uniform", 4),
    5: Config(5, "complete256-dense", 256, "complete", 0, "none", 1_000_000, 0, 0.05, 20, "exp", "uniform", 128),
    # the paper's own experiment shapes (Section 5 / Appendix B) on synthetic 256-dimensional inputs
    6: Config(6, "paper-lrm", 6, "er", 0.5, "lrm", 2570, 1024, 0.2, 20, "lognormal_slow", "dtur", 0, lr_decay=0.95),
    7: Config(7, "paper-2nn", 10, "er", 0.4, "2nn", 134154, 1024, 1.0, 20, "lognormal_slow", "dtur", 0, lr_decay=0.95),
}


def make_graph(cfg: Config):
    g = rng(cfg.cid, P_GRAPH)
    if cfg.graph == "ring":
        return graph_ring(cfg.n)
    if cfg.graph == "complete":
        return graph_complete(cfg.n)
    if cfg.graph == "regular":
        return graph_regular(cfg.n, int(cfg.graph_arg), g)
    if cfg.graph == "er":
        return graph_er(cfg.n, float(cfg.graph_arg), g)
    raise ValueError(cfg.graph)


def slow_workers(cfg: Config) -> np.ndarray:
    """Fixed set of slowed-down workers (10 % of N, rounded down), chosen once."""
    g = rng(cfg.cid, P_SLOW)
    k = max(1, int(0.1 * cfg.n))       # Appendix B: at least one straggler in each iteration
    return np.sort(g.choice(cfg.n, size=k, replace=False)).astype(np.int32)


def response_times(cfg: Config, rnd: int) -> np.ndarray:
    g = rng(cfg.cid, P_TIMES, rnd)
    if cfg.times == "exp":
        t = g.standard_exponential(cfg.n)
    elif cfg.times == "shifted_exp":
        t = 0.5 + g.standard_exponential(cfg.n)
    elif cfg.times == "lognormal_slow":
        t = g.lognormal(0.0, 0.5, cfg.n)
        t[slow_workers(cfg)] *= 5.0
    else:
        raise ValueError(cfg.times)
    return t.astype(np.float32)


def backup_counts(cfg: Config, rnd: int, rowptr: np.ndarray) -> np.ndarray:
    """b[N] for rounds where the caller (not the threshold rule) chooses it."""
    deg = np.diff(rowptr).astype(np.int32)
    if cfg.backup == "const":
        b = np.full(cfg.n, cfg.backup_arg, dtype=np.int32)
    elif cfg.backup == "uniform":
        b = rng(cfg.cid, P_BACKUP, rnd).integers(0, cfg.backup_arg + 1, cfg.n).astype(np.int32)
    else:
        raise ValueError("backup counts of this config come from the threshold rule")
    return np.minimum(b, deg).astype(np.int32)


def learning_rate(cfg: Config, rnd: int) -> float:
    return cfg.lr * cfg.lr_decay ** rnd


def teacher(cfg: Config, in_dim: int) -> np.ndarray:
    """[in_dim, 10] fixed random linear map: with labels == "teacher" a sample's class is the
    largest of its ten scores, so that a model can learn the labels and a loss curve means
    something (the stand-in for a real data set's structure)."""
    return rng(cfg.cid, P_TEACHER).standard_normal((in_dim, 10))


def batch(cfg: Config, rnd: int, workers=None):
    """(x [n, B, in] fp32, y [n, B] int32) for the given workers (default all)."""
    desc = model_dims(cfg.model)
    in_dim = desc["dims"][0] if desc["kind"] == "mlp" else int(np.prod(desc["in"]))
    workers = range(cfg.n) if workers is None else workers
    scores = teacher(cfg, in_dim) if cfg.labels == "teacher" else None
    xs, ys = [], []
    for i in workers:
        gx = rng(cfg.cid, P_BATCH_X, rnd * 4096 + i)
        gy = rng(cfg.cid, P_BATCH_Y, rnd * 4096 + i)
        if cfg.x_dist == "uniform":
            xs.append(gx.random((cfg.batch, in_dim), dtype=np.float32))
        else:
            xs.append(gx.standard_normal((cfg.batch, in_dim), dtype=np.float32))
        if scores is None:
            ys.append(gy.integers(0, 10, cfg.batch).astype(np.int32))
        else:
            ys.append(np.argmax(xs[-1].astype(np.float64) @ scores, axis=1).astype(np.int32))
    return np.stack(xs), np.stack(ys)


def flat_params(cfg: Config, n_rows: int, cols: int, purpose: int, std: float, rnd: int = 0) -> np.ndarray:
    """[n_rows, cols] fp32 N(0, std^2): parameter vectors (std 1) or supplied gradients
    (std 0.01) of the consensus-only configurations."""
    g = rng(cfg.cid, purpose, rnd)
    return (g.standard_normal((n_rows, cols), dtype=np.float32) * np.float32(std)).astype(np.float32)


def pad_ld(d: int, mult: int = 64) -> int:
    return (d + mult - 1) // mult * mult
