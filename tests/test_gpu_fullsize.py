"""Parity at the full benchmark sizes, in the launch configuration bench.py times: the
consensus-only stress (N = 128, d = 11.2 M, sparse path) and the dense-mixing stress
(N = 256, d = 1 M, matrix-core path), the former in both storage layouts.  The averaging is column-separable, so the oracle
is evaluated on sampled column blocks (first, last, and random ones) of the device data."""
import numpy as np
import pytest
import torch

from gpu_util import assert_params_close

pytestmark = pytest.mark.gpu


# d = None: the benchmark's own size.  The larger d make N * d exceed 2^31 elements per matrix
# (8.7 GB each), so that element offsets no longer fit 32 bits: N = 128 x 17 M on both sparse
# kernels, N = 256 x 8.5 M on the matrix-core kernel.
@pytest.mark.parametrize("cid,order,tiles,d", [(4, 0, False, None), (4, 1, False, None), (5, 0, False, None),
                                               (5, 1, False, None), (4, 0, True, None), (4, 1, True, None),
                                               (4, 0, False, 17_000_006), (4, 1, True, 17_000_006),
                                               (5, 0, False, 8_500_003)],
                         ids=["c4-cta", "c4-atc", "c5-cta", "c5-atc", "c4-cta-tiles", "c4-atc-tiles",
                              "c4-rows-2g-elements", "c4-tiles-2g-elements", "c5-2g-elements"])
def test_full_size_sampled_columns(orc, cid, order, tiles, d):
    from paper_2102_06280_amd import binding as B
    from paper_2102_06280_amd.workload import Workload
    wl = Workload(cid, rounds=2, order=order, layout=B.LAYOUT_TILES if tiles else B.LAYOUT_ROWS, d_override=d)
    try:
        assert d is None or wl.n * wl.ld > 2 ** 31
        cfg = wl.cfg
        blk = 4096
        g = np.random.default_rng(311 + cid)
        starts = [0, wl.d - blk] + [int(s) for s in g.integers(0, wl.d - blk, 6)]
        starts.append(int(g.integers(0, wl.d - blk)) | 1)       # an odd, unaligned start
        for rnd in range(2):
            src = wl.params()
            before = [wl.columns(src, s, s + blk).cpu().numpy() for s in starts]
            grads = [wl.columns(wl.g, s, s + blk).cpu().numpy() for s in starts]
            wl.step()
            assert B.dbw_check(wl.h) == 0
            dst = wl.params()
            mask_d = torch.empty(wl.colidx.size, dtype=torch.uint8, device="cuda")
            p_d = torch.empty(wl.n, dtype=torch.int32, device="cuda")
            B.dbw_get_selection(wl.h, p_d, mask_d, None)
            mask, p, _ = orc.select(wl.rowptr, wl.colidx, wl.t_host[rnd], wl.b_host[rnd])
            assert np.array_equal(mask_d.cpu().numpy(), mask) and np.array_equal(p_d.cpu().numpy(), p)
            for s, xb, gb in zip(starts, before, grads):
                want = orc.round_(wl.rowptr, wl.colidx, mask, p, xb, gb, cfg.lr, order)
                got = wl.columns(dst, s, s + blk).cpu().numpy()
                assert_params_close(got, want, what=f"config {cid} round {rnd} columns {s}..{s + blk}")
            # padding columns (if any) and the source buffer are untouched
            assert torch.equal(wl.columns(src, 0, blk), torch.from_numpy(before[0]).cuda())
    finally:
        wl.close()
