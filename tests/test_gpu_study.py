"""The loss-against-simulated-time study (Section 5, Appendix B in miniature) against the same
loop written with the oracle: backup counts, round durations, losses and final parameters of
both policies, free-running over all rounds."""
import dataclasses

import numpy as np
import pytest

from paper_2102_06280_amd import inputs
from gpu_util import assert_params_close

pytestmark = pytest.mark.gpu

ROUNDS, POOL = 12, 5


@pytest.fixture(scope="module")
def B():
    from paper_2102_06280_amd import binding
    return binding


def oracle_run(orc, cid, policy, order):
    cfg = dataclasses.replace(inputs.CONFIGS[cid], labels="teacher")
    rowptr, colidx = inputs.make_graph(cfg)
    desc = inputs.model_dims(cfg.model)
    kind, od = orc.model_desc(desc)
    ld = inputs.pad_ld(cfg.d)
    x = inputs.init_params(desc, cfg.n, ld, inputs.rng(cid, inputs.P_PARAMS), zero=cfg.zero_init)
    dt = orc.Dtur(rowptr, colidx)
    loss, dur, bs = [], [], []
    for k in range(ROUNDS):
        t = inputs.response_times(cfg, k)
        b = np.zeros(cfg.n, np.int32)
        if policy == "dybw" and k > 0:
            b = dt.step(t)[0]
        mask, p, wait = orc.select(rowptr, colidx, t, b)
        bx, by = inputs.batch(cfg, k % POOL)
        g, l = orc.grad_all(kind, od, cfg.d, x, bx, by)
        x = orc.round_(rowptr, colidx, mask, p, x, g, inputs.learning_rate(cfg, k), order, d=cfg.d)
        loss.append(l)
        dur.append(orc.round_time(rowptr, colidx, mask, wait)[1])
        bs.append(b)
    return np.array(loss), np.array(dur, dtype=np.float32), np.array(bs), x[:, :cfg.d]


@pytest.mark.parametrize("order", [0, 1], ids=["cta", "atc"])
def test_study_matches_oracle_loop(B, orc, order):
    """Logistic regression has no ReLU or pooling decision, so the two free-running
    trajectories stay together: averaging is a convex combination and the step is a
    contraction-like map, so per-round rounding differences (about 1e-7) add up at most
    linearly over the 12 rounds; the per-round tolerance is kept."""
    from paper_2102_06280_amd import study
    cid = 6
    for policy in study.POLICIES:
        got = study.run(cid, ROUNDS, policy, order, pool=POOL)
        loss, dur, b, x = oracle_run(orc, cid, policy, order)
        assert np.array_equal(got["b"], b), policy
        assert np.array_equal(got["duration"], dur), policy
        assert np.allclose(got["loss"], loss, rtol=1e-5, atol=1e-6), policy
        assert_params_close(got["params"], x, tol=1e-5, what=f"{policy} after {ROUNDS} rounds")


def test_study_summary(B):
    """Dynamic backup workers shorten every round (Corollary 4 holds per realisation), both
    runs learn the teacher's rule, and the summary's bookkeeping is consistent."""
    from paper_2102_06280_amd import study
    out = study.compare(6, 40, pool=8)
    cur = out["curves"]
    d_dy = np.diff(np.concatenate([[0.0], cur["dybw"]["time"]]))
    d_fu = np.diff(np.concatenate([[0.0], cur["full"]["time"]]))
    assert np.all(d_dy <= d_fu + 1e-3)
    assert out["mean_round_duration"]["reduction"] > 0.1
    for p in study.POLICIES:
        assert out["loss_last_round"][p] < 0.8 * out["loss_first_round"][p]
        assert out["time_to_loss"][p] is not None
    print({k: out[k] for k in ("mean_round_duration", "loss_first_round", "loss_last_round", "time_to_loss",
                               "mean_backup_workers")})
