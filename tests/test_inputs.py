"""The seeded input recipes: structure only (the generators hold none of the method's
arithmetic)."""
import numpy as np
import pytest

from paper_2102_06280_amd import inputs


@pytest.mark.parametrize("cid", sorted(inputs.CONFIGS))
def test_graph_is_simple_symmetric_connected(cid):
    cfg = inputs.CONFIGS[cid]
    rowptr, colidx = inputs.make_graph(cfg)
    n = cfg.n
    assert rowptr.size == n + 1 and rowptr[0] == 0 and rowptr[-1] == colidx.size
    adj = [set(colidx[rowptr[i]:rowptr[i + 1]].tolist()) for i in range(n)]
    for i in range(n):
        row = colidx[rowptr[i]:rowptr[i + 1]]
        assert np.all(np.diff(row) > 0) and i not in adj[i]
        assert all(i in adj[j] for j in adj[i])
    seen, stack = {0}, [0]
    while stack:
        for j in adj[stack.pop()]:
            if j not in seen:
                seen.add(j)
                stack.append(j)
    assert len(seen) == n


@pytest.mark.parametrize("cid", sorted(inputs.CONFIGS))
def test_parameter_count_matches_model(cid):
    cfg = inputs.CONFIGS[cid]
    if cfg.model != "none":
        assert inputs.param_count(inputs.model_dims(cfg.model)) == cfg.d


def test_inputs_are_reproducible_and_round_dependent():
    cfg = inputs.CONFIGS[7]
    assert np.array_equal(inputs.response_times(cfg, 3), inputs.response_times(cfg, 3))
    assert not np.array_equal(inputs.response_times(cfg, 3), inputs.response_times(cfg, 4))
    x0, y0 = inputs.batch(cfg, 0, workers=[2])
    x1, y1 = inputs.batch(cfg, 0, workers=[2])
    assert np.array_equal(x0, x1) and np.array_equal(y0, y1)
    assert x0.shape == (1, 1024, 256) and y0.min() >= 0 and y0.max() < 10


@pytest.mark.parametrize("cid", [6, 7])
def test_paper_shaped_configs_have_a_straggler_and_decayed_rate(cid):
    """Appendix B: every iteration has at least one straggler; Section 5: the learning rate
    shrinks by 0.95 per round."""
    cfg = inputs.CONFIGS[cid]
    assert inputs.slow_workers(cfg).size >= 1
    assert inputs.learning_rate(cfg, 0) == cfg.lr
    assert inputs.learning_rate(cfg, 5) == pytest.approx(cfg.lr * 0.95 ** 5)
    assert inputs.learning_rate(inputs.CONFIGS[2], 5) == inputs.CONFIGS[2].lr


def test_teacher_labels_follow_the_inputs():
    """labels == "teacher": same inputs as the uniform-label recipe, labels a deterministic
    function of each sample (argmax of a fixed linear map), all ten classes in use."""
    import dataclasses
    cfg = inputs.CONFIGS[6]
    tcfg = dataclasses.replace(cfg, labels="teacher")
    x0, y0 = inputs.batch(cfg, 3)
    x1, y1 = inputs.batch(tcfg, 3)
    assert np.array_equal(x0, x1) and not np.array_equal(y0, y1)
    T = inputs.teacher(tcfg, 256)
    assert T.shape == (256, 10)
    assert np.array_equal(y1, np.argmax(x1.astype(np.float64) @ T, axis=-1))
    assert np.bincount(y1.ravel(), minlength=10).min() > 0
    x2, y2 = inputs.batch(tcfg, 3, workers=[2])
    assert np.array_equal(y2[0], y1[2])


def test_time_to_loss():
    from paper_2102_06280_amd.study import time_to_loss
    loss = np.array([2.3, 2.0, 1.5, 1.6, 1.0])
    dur = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    assert time_to_loss(loss, dur, 2.3) == 0.0          # the loss of a round is measured before its update
    assert time_to_loss(loss, dur, 1.5) == 3.0
    assert time_to_loss(loss, dur, 1.2) == 10.0
    assert time_to_loss(loss, dur, 0.5) is None
