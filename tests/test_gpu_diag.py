"""The library's diagnostics (hardware measurements that the kernel layout and the benchmark's
ceilings rest on, not part of the method) run and return sane figures."""
import math

import pytest

pytestmark = pytest.mark.gpu


def test_coexecution_measurement(lp):
    ns = lp.lp_diag_coexecution()
    assert len(ns) == 10 and all(math.isfinite(v) and v > 0 for v in ns)
    # one wave: vector work after a matrix product adds to its time (no overlap inside a wave)
    assert ns[3] > ns[0]
    # two waves of one SIMD: both working takes less than the sum of each working alone
    assert ns[6] < ns[4] + ns[5]


def test_atomic_line_rate_measurement(lp):
    r = lp.lp_diag_atomic_rate()
    assert len(r) == 6 and all(math.isfinite(v) for v in r)
    assert all(1e9 < v < 1e12 for v in r), r
