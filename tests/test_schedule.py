"""The library's host-side training-phase schedule against the oracle's (no device work: runs without a GPU)."""
import math

import pytest

from oracle import evomoe_oracle as orc
from paper_2112_14397_amd import binding as B


@pytest.mark.parametrize("T_S,T_D", [(5000, 5000), (10000, 5000), (0, 15000), (3, 1), (0, 6), (7, 0)])
def test_schedule_matches_oracle(T_S, T_D):
    its = sorted({0, 1, max(T_S - 1, 0), T_S, T_S + 1, T_S + T_D // 2, max(T_S + T_D - 1, 0), T_S + T_D,
                  T_S + T_D + 1, T_S + T_D + 12345})
    for i in its:
        ph, ref = B.evomoe_schedule(i, T_S, T_D, 2.0, 0.3), orc.schedule(i, T_S, T_D, 2.0, 0.3)
        assert (ph.stage, bool(ph.top1)) == (ref.stage, ref.top1), (i, T_S, T_D)
        if ref.stage == 1:
            assert math.isnan(ph.tau)
        else:
            assert ph.tau == pytest.approx(ref.tau, rel=1e-6)


def test_schedule_argument_errors():
    with pytest.raises(B.EvoMoEError):
        B.evomoe_schedule(-1, 0, 10)
    with pytest.raises(B.EvoMoEError):
        B.evomoe_schedule(0, 0, 10, tau_hi=0.0)
