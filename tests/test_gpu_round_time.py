"""GPU parity of the round duration T(k) (Section 3.2.2) and the duration comparison of
dynamic backup workers against full participation on the same response times."""
import numpy as np
import pytest
import torch

from paper_2102_06280_amd import inputs
from gpu_util import dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cid", [1, 2, 3, 4, 5])
def test_round_time_matches_oracle(orc, cid):
    from paper_2102_06280_amd import binding as B
    cfg = inputs.CONFIGS[cid]
    rowptr, colidx = inputs.make_graph(cfg)
    n = cfg.n
    h = B.dbw_create(rowptr, colidx, n, 64, mix_path=B.MIX_CSR)
    try:
        T = torch.zeros(2, device="cuda")
        dt = orc.Dtur(rowptr, colidx)
        shorter = 0
        for rnd in range(12):
            t = inputs.response_times(cfg, rnd)
            if rnd == 7:
                t[3] = np.inf
            b = dt.step(t)[0] if cfg.backup == "dtur" else inputs.backup_counts(cfg, rnd, rowptr)
            for bb in (b, np.zeros(n, np.int32), np.diff(rowptr).astype(np.int32)):
                B.dbw_select(h, dev(t), dev(bb))
                B.dbw_round_time(h, T)
                mask, p, wait = orc.select(rowptr, colidx, t, bb)
                want = orc.round_time(rowptr, colidx, mask, wait)
                got = T.cpu().numpy()
                assert got[0] == np.float32(want[0]) and got[1] == np.float32(want[1]), (rnd, got, want)
                if bb is b:
                    dy = got[0]
                elif not bb.any():
                    assert dy <= got[0]                     # Corollary 4, per realisation
                    shorter += dy < got[0]
        assert B.dbw_check(h) == 0
    finally:
        B.dbw_destroy(h)
