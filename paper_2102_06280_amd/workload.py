"""Device-resident synthetic workloads for the benchmark configurations, and the
round loop that drives the library over them.  Plumbing only: tensors are allocated and
filled here (torch is used for memory, random fills and streams), every step of a round
runs inside the library.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch

from . import binding as B
from . import inputs


class Workload:
    """All inputs of `rounds` rounds of one configuration, resident in HBM."""

    def __init__(self, cid: int, rounds: int, order: int = B.ORDER_CTA, mix_path: int = B.MIX_AUTO,
                 d_override: int | None = None, ld_override: int | None = None, layout: int = B.LAYOUT_ROWS,
                 labels: str | None = None):
        cfg = inputs.CONFIGS[cid]
        if labels is not None:
            cfg = dataclasses.replace(cfg, labels=labels)
        self.cfg, self.cid, self.rounds, self.order = cfg, cid, rounds, order
        self.rowptr, self.colidx = inputs.make_graph(cfg)
        self.n = cfg.n
        self.d = d_override or cfg.d
        self.ld = ld_override or inputs.pad_ld(self.d)
        assert self.ld >= self.d
        self.desc = inputs.model_dims(cfg.model) if cfg.model != "none" else None
        model = None
        if self.desc is not None:
            if self.desc["kind"] == "mlp":
                model = B.make_model(B.MODEL_MLP, cfg.batch, self.desc["dims"],
                                     B.LOSS_MSE if self.desc.get("loss") == "mse" else B.LOSS_XENT)
            else:
                c, h, w = self.desc["in"]
                model = B.make_model(B.MODEL_CNN, cfg.batch, [c, h, w, self.desc["c1"], self.desc["c2"],
                                                              self.desc["k"], self.desc["fc"], self.desc["classes"]])
        self.layout = layout
        self.h = B.dbw_create(self.rowptr, self.colidx, self.n, self.d, ld=self.ld, order=order,
                              mix_path=mix_path, model=model, layout=layout)
        dev = torch.device("cuda")
        # response times and backup counts of every round
        self.t_host = np.stack([inputs.response_times(cfg, r) for r in range(rounds)])
        self.t = torch.from_numpy(self.t_host).to(dev)
        self.dynamic_b = cfg.backup == "dtur"
        if self.dynamic_b:
            self.b_host = None
            self.b = torch.zeros((rounds, self.n), dtype=torch.int32, device=dev)   # round 0 stays b = 0
        else:
            self.b_host = np.stack([inputs.backup_counts(cfg, r, self.rowptr) for r in range(rounds)])
            self.b = torch.from_numpy(self.b_host).to(dev)
        # parameters (ping-pong) and gradients / batches
        if self.desc is None:
            gen = torch.Generator(device=dev)
            gen.manual_seed(inputs.SEED + cid)
            self.x = [torch.empty((self.n, self.ld), dtype=torch.float32, device=dev) for _ in range(2)]
            self.x[0].normal_(0.0, 1.0, generator=gen)
            self.x[1].zero_()
            self.g = torch.empty((self.n, self.ld), dtype=torch.float32, device=dev)
            self.g.normal_(0.0, 0.01, generator=gen)          # one fixed gradient matrix for all rounds
            if layout == B.LAYOUT_TILES:                      # the same values, stored tile-major
                B.dbw_convert_layout(self.h, self.x[0], self.x[1], True)
                self.x[0].zero_()
                self.x.reverse()
                tmp = torch.empty_like(self.g)
                B.dbw_convert_layout(self.h, self.g, tmp, True)
                self.g = tmp
                torch.cuda.synchronize()
            self.bx = self.by = None
        else:
            x0 = inputs.init_params(self.desc, self.n, self.ld, inputs.rng(cid, inputs.P_PARAMS), zero=cfg.zero_init)
            self.x = [torch.from_numpy(x0).to(dev), torch.zeros((self.n, self.ld), dtype=torch.float32, device=dev)]
            self.g = None
            bx, by = zip(*[inputs.batch(cfg, r) for r in range(rounds)])
            self.bx = torch.from_numpy(np.stack(bx)).to(dev)
            self.by = torch.from_numpy(np.stack(by)).to(dev)
        self.loss = torch.zeros(self.n, dtype=torch.float32, device=dev)
        self.cur = 0
        self.k = 0

    def step(self):
        """One round: (threshold rule,) selection, gradient, masked average, SGD step."""
        r = self.k % self.rounds
        if self.dynamic_b and r > 0:
            B.dbw_dtur_select(self.h, self.t[r], self.b[r])     # threshold rule + selection, one launch for small graphs
        else:
            B.dbw_select(self.h, self.t[r], self.b[r])
        src, dst = self.x[self.cur], self.x[self.cur ^ 1]
        if self.desc is None:
            B.dbw_round(self.h, src, dst, self.cfg.lr, ext_grads=self.g)
        else:
            B.dbw_round(self.h, src, dst, inputs.learning_rate(self.cfg, r), batch_x=self.bx[r], batch_y=self.by[r],
                        loss_out=self.loss)
        self.cur ^= 1
        self.k += 1

    def capture_steps(self, n_steps: int):
        """Capture the next `n_steps` rounds, one HIP graph per round (every round has its own
        response times, backup counts, batch and ping-pong direction), so that a launch-bound
        round replays as one submission.  A round calls no allocation, memset or
        synchronisation, so it can be captured as it is.  Returns the list of graphs; replaying
        them in order is equivalent to calling step() n_steps times from the current state."""
        torch.cuda.synchronize()
        graphs = []
        k0, cur0 = self.k, self.cur
        stream = torch.cuda.Stream()
        for _ in range(n_steps):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                self.step()
            graphs.append(g)
        torch.cuda.synchronize()
        self.k, self.cur = k0, cur0          # capturing ran nothing: restore the bookkeeping
        return graphs

    def replay(self, graphs):
        for g in graphs:
            g.replay()
            self.cur ^= 1
            self.k += 1

    def params(self):
        return self.x[self.cur]

    def columns(self, t, start: int, stop: int):
        """Columns [start, stop) of all workers as an [N, stop - start] tensor, whatever the
        layout `t` (one of this workload's [N * ld] arrays) is stored in."""
        if self.layout == B.LAYOUT_ROWS:
            return t[:, start:stop]
        w = B.TILE_COLUMNS
        t0, t1 = start // w, (stop + w - 1) // w
        block = t.view(self.ld // w, self.n, w)[t0:t1].permute(1, 0, 2).reshape(self.n, (t1 - t0) * w)
        return block[:, start - t0 * w: stop - t0 * w]

    def close(self):
        if self.h is not None:
            B.dbw_destroy(self.h)
            self.h = None
