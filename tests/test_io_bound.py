"""The I/O yardstick reproduces the figures tabulated for the five workloads (constant 1,
Table-1 form, M in elements) and the regime split of the main theorem (M vs d^2)."""
import pytest

from paper_2410_09397_amd import io_bound, synth

MB = 1e6
# (workload, compulsory MB, Theta-term MB at 160 KB / 672 KB / 4 MB, regime at LDS)
TABLE = [
    (2, 134.7, 26.8, 6.4, 1.0, "large"),
    (3, 1075.8, 859.0, 204.5, 33.6, "large"),
    (4, 268.6, 480.2, 204.5, 33.6, "small"),
    (5, 537.9, 1270.5, 409.0, 67.1, "small"),
]


@pytest.mark.parametrize("idx,comp,t160,t672,t4m,reg", TABLE)
def test_bounds_match_tabulated_values(idx, comp, t160, t672, t4m, reg):
    w = synth.workload(idx)
    assert io_bound.compulsory_bytes(w) / MB == pytest.approx(comp, abs=0.06)
    got = [io_bound.theta_bytes(w, m) / MB for m in io_bound.M_EFF_BYTES.values()]
    for g, want in zip(got, (t160, t672, t4m)):
        assert g == pytest.approx(want, rel=2e-3, abs=0.06)
    assert io_bound.regime(w, io_bound.M_EFF_BYTES["lds_160KB"]) == reg
    assert io_bound.yardstick(w) / MB == pytest.approx(max(comp, t160), rel=2e-3)


def test_crossing_point_of_the_two_regimes():
    """At M = d^2 both branches equal n^2 d (the n^2 + nd crossing value of Sec. 4, n >> d)."""
    w = synth.workload(3)
    m_bytes = w.d * w.d * 2
    n, d = w.n, w.d
    per_head_items = io_bound.theta_bytes(w, m_bytes) / (2 * w.batch * w.heads * w.kept_fraction())
    assert per_head_items == pytest.approx(n * n, rel=1e-12)
    assert io_bound.regime(w, m_bytes) == "large" and io_bound.regime(w, m_bytes - 2) == "small"
