"""cwac_calibrate_stats_static (the statistics pass on the library's own fixed scratch buffer, for
callers that cannot allocate) against cwac_calibrate_stats on a caller's workspace, through the C
ABI: two calls in a row, the second with a smaller input, must leave states bit-identical to the
workspace form's (same kernels, same row split), and moments within 1e-5 of the fp64 oracle."""
import numpy as np
import pytest
import torch

import paper_2505_20932_amd as P
from paper_2505_20932_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
RTOL = 1e-5


def _inputs(seed, rows, c):
    yq = synth.normal(seed, 0, rows * c).view(rows, c)
    yq[:, 3 % c] = yq[:, 3 % c] * 0.01 + 250.0                      # mean >> spread
    gain = 1.0 + 0.1 * synth.normal(seed, 1, c)
    yf = yq * gain[None, :] + 0.05 * synth.normal(seed, 2, rows * c).view(rows, c) + 0.02
    return yf.contiguous(), yq.contiguous()


def _moments(st, c):
    alpha = torch.empty(c, dtype=torch.float32, device=DEV)
    beta = torch.empty(c, dtype=torch.float32, device=DEV)
    mom = torch.empty(5, c, dtype=torch.float64, device=DEV)
    P.cwac_solve(st, c, alpha, beta, mom)
    torch.cuda.synchronize()
    return mom.cpu().numpy()


def test_static_scratch_statistics_match_the_workspace_form(orc):
    assert P.cwac_static_scratch_bytes() == 8 << 20
    words = lambda c: P.cwac_stats_bytes(c) // 8
    # first call: several row groups and channel groups; second call: smaller in both dimensions,
    # so that it re-uses a part of the buffer the first call left full
    for seed, rows, c in ((11, 9000, 1536), (12, 700, 260)):
        print(f"static-scratch statistics: {rows} x {c}", flush=True)
        yf, yq = _inputs(seed, rows, c)
        yf_d, yq_d = yf.to(DEV), yq.to(DEV)
        assert P.cwac_calibrate_stats_workspace(rows, c) <= P.cwac_static_scratch_bytes()
        st_a = torch.empty(words(c) + 2, dtype=torch.float64, device=DEV)
        st_b = torch.empty(words(c) + 2, dtype=torch.float64, device=DEV)
        P.cwac_stats_reset(st_a, c)
        P.cwac_stats_reset(st_b, c)
        ws = torch.empty(P.cwac_calibrate_stats_workspace(rows, c), dtype=torch.uint8, device=DEV)
        cut = rows // 3
        for lo, hi in ((0, cut), (cut, rows)):                        # two batches into each state
            P.cwac_calibrate_stats(yf_d[lo:hi], yq_d[lo:hi], st_a, ws)
            P.cwac_calibrate_stats_static(yf_d[lo:hi], yq_d[lo:hi], st_b)
        torch.cuda.synchronize()
        assert torch.equal(st_a[:words(c)].view(torch.int64), st_b[:words(c)].view(torch.int64))
        ref = orc.channel_moments(yf.numpy(), yq.numpy())
        got = _moments(st_b, c)
        sf, sq = np.sqrt(ref[4]), np.sqrt(ref[2])
        floors = [sf, sq, sq * sq, sq * sf, sf * sf]
        for i in range(5):
            err = np.abs(got[i] - ref[i]) / (np.maximum(np.abs(ref[i]), floors[i]) + 1e-300)
            assert err.max() <= RTOL, (i, err.max())


def test_static_scratch_argument_errors():
    a = torch.zeros(8, 4, dtype=torch.float32, device=DEV)
    st = torch.zeros(P.cwac_stats_bytes(4) // 8 + 2, dtype=torch.float64, device=DEV)
    with pytest.raises(P.CwacError):
        P.binding._check(P.binding.lib().cwac_calibrate_stats_static(None, 4, None, 4, 8, 4, None, None), "x")
    with pytest.raises(P.CwacError):                                    # ld < c_out
        P.binding._check(P.binding.lib().cwac_calibrate_stats_static(
            a.data_ptr(), 2, a.data_ptr(), 4, 8, 4, st.data_ptr(), None), "x")
    P.cwac_stats_reset(st, 4)
    P.cwac_calibrate_stats_static(a[:0], a[:0], st)                     # empty batch: no-op
    torch.cuda.synchronize()
    assert int(st.view(torch.int64)[0]) == 0
