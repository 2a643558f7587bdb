"""The iteration schedule of Fig. 1(a) and Section III-A, pinned to the paper's own worked example."""
import os

import pytest

from oracle.fdg_oracle import fdg_schedule

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig1_k3_delay.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append(tuple(int(v) for v in line.split()))
    return rows


def test_fig1_worked_example():
    for K, k, batch, t_fwd, t_bwd in _golden_rows():
        fwd, bwd, _ = fdg_schedule(K, 12)
        assert fwd[k][t_fwd] == batch
        assert bwd[k][t_bwd] == batch
        assert t_bwd - t_fwd == 2 * (K - k)


@pytest.mark.parametrize("K", [1, 2, 3, 4])
def test_batch_indices_follow_section_3a(K):
    """Module k forwards batch t-k+1 and back-propagates batch t-2K+k+1 at iteration t (ids < 1: idle),
    and holds at most 2(K-k)+1 saved forwards (the new one plus a history of 2(K-k))."""
    T = 20
    fwd, bwd, depth = fdg_schedule(K, T)
    for k in range(1, K + 1):
        for t in range(1, T + 1):
            assert fwd[k][t] == max(0, t - k + 1)
            assert bwd[k][t] == max(0, t - 2 * K + k + 1)
        assert depth[k] == 2 * (K - k) + 1
