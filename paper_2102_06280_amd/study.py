"""Loss against simulated wall-clock time: dynamic backup workers against full participation.

The experiment of Section 5 / Appendix B in miniature, on synthetic inputs: the same model,
graph, mini-batches, learning rates and response times are trained twice, once with the
backup counts of the threshold rule (Section 4.1) and once with b = 0 (every worker waits
for all its neighbours).  A round lasts T(k) (Section 3.2.2), the slowest wait of the
round; the study reports the loss of every round, T(k), and the time each policy needs to
reach a common loss level.  Labels follow a fixed random linear rule of the inputs, so
that there is something to learn; the mini-batches cycle through a pool.

Plumbing only: every step of a round runs inside the library, on one stream, with one
synchronisation at the end of a run.

    python -m paper_2102_06280_amd.study [--config 6|7] [--rounds 60] [--order cta|atc]
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import binding as B
from . import inputs
from .workload import Workload

POLICIES = ("dybw", "full")


def run(cid: int, rounds: int, policy: str, order: int = B.ORDER_CTA, pool: int = 16):
    """Train `rounds` rounds of configuration `cid` under one policy.  Returns a dict of host
    arrays: loss [rounds, N] (each worker's mini-batch loss at its parameters before the
    round's update), duration [rounds] = T(k), b [rounds, N], and the final parameters."""
    assert policy in POLICIES
    pool = min(pool, rounds)
    wl = Workload(cid, rounds=pool, order=order, labels="teacher")
    try:
        cfg, n = wl.cfg, wl.n
        assert wl.desc is not None, "the study needs a configuration with a model"
        dev = torch.device("cuda")
        t = torch.from_numpy(np.stack([inputs.response_times(cfg, k) for k in range(rounds)])).to(dev)
        b = torch.zeros((rounds, n), dtype=torch.int32, device=dev)      # "full": b = 0 in every round
        threshold_rule = cfg.backup == "dtur"                            # then round 0 has b = 0 (Algorithm 1)
        if policy == "dybw" and not threshold_rule:
            b = torch.from_numpy(np.stack([inputs.backup_counts(cfg, k, wl.rowptr) for k in range(rounds)])).to(dev)
        loss = torch.zeros((rounds, n), dtype=torch.float32, device=dev)
        T = torch.zeros((rounds, 2), dtype=torch.float32, device=dev)
        cur = 0
        for k in range(rounds):
            if policy == "dybw" and threshold_rule and k > 0:
                B.dbw_dtur_select(wl.h, t[k], b[k])
            else:
                B.dbw_select(wl.h, t[k], b[k])
            B.dbw_round(wl.h, wl.x[cur], wl.x[cur ^ 1], inputs.learning_rate(cfg, k),
                        batch_x=wl.bx[k % pool], batch_y=wl.by[k % pool], loss_out=loss[k])
            B.dbw_round_time(wl.h, T[k])
            cur ^= 1
        torch.cuda.synchronize()
        B.dbw_check(wl.h)
        return {"loss": loss.cpu().numpy(), "duration": T[:, 1].cpu().numpy(), "b": b.cpu().numpy(),
                "params": wl.x[cur][:, :cfg.d].cpu().numpy(), "t": t.cpu().numpy()}
    finally:
        wl.close()


def time_to_loss(loss: np.ndarray, duration: np.ndarray, target: float):
    """Simulated time at the end of the first round whose (pre-update) loss is at or below
    `target`, counting the durations of the rounds before it; None if never reached."""
    hit = np.flatnonzero(loss <= target)
    if hit.size == 0:
        return None
    return float(np.sum(duration[:hit[0]], dtype=np.float64))


def compare(cid: int, rounds: int, order: int = B.ORDER_CTA, pool: int = 16):
    runs = {p: run(cid, rounds, p, order, pool) for p in POLICIES}
    mean_loss = {p: runs[p]["loss"].astype(np.float64).mean(axis=1) for p in POLICIES}
    # a level both runs reach: the larger of the two best losses
    target = float(max(mean_loss[p].min() for p in POLICIES))
    mean_dur = {p: float(runs[p]["duration"].astype(np.float64).mean()) for p in POLICIES}
    cfg = inputs.CONFIGS[cid]
    return {
        "workload": f"config {cid}: {cfg.name}, labels from a linear teacher, batches cycle through "
                    f"{min(pool, rounds)} per worker",
        "rounds": rounds, "order": "cta" if order == B.ORDER_CTA else "atc",
        "mean_round_duration": {**mean_dur, "reduction": 1.0 - mean_dur["dybw"] / mean_dur["full"]},
        "loss_first_round": {p: float(mean_loss[p][0]) for p in POLICIES},
        "loss_last_round": {p: float(mean_loss[p][-1]) for p in POLICIES},
        "time_to_loss": {"target": target,
                         **{p: time_to_loss(mean_loss[p], runs[p]["duration"], target) for p in POLICIES}},
        "mean_backup_workers": float(runs["dybw"]["b"][1:].mean()) if rounds > 1 else 0.0,
        "curves": {p: {"time": np.cumsum(runs[p]["duration"], dtype=np.float64).round(4).tolist(),
                       "loss": mean_loss[p].round(6).tolist()} for p in POLICIES},
    }


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", type=int, default=6, choices=[1, 2, 3, 6, 7])
    ap.add_argument("--rounds", type=int, default=60)
    ap.add_argument("--order", choices=["cta", "atc"], default="cta")
    ap.add_argument("--pool", type=int, default=16)
    args = ap.parse_args()
    out = compare(args.config, args.rounds, B.ORDER_CTA if args.order == "cta" else B.ORDER_ATC, args.pool)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
