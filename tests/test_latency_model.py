"""The paper's Table 1 regenerated from the closed forms of Sec. 3.1, and the corollary's bounds."""
import os

from paper_2507_12000_amd import latency_model as M


def _table1(golden_dir):
    with open(os.path.join(golden_dir, "table1_reject_probability.txt")) as f:
        return [(int(g), float(a), float(p), float(t)) for g, a, p, t in
                (line.split() for line in f if line.strip() and not line.startswith("#"))]


def test_table1_is_reproduced(golden_dir):
    # The table fits T_NTT = 20 ms and |V| b_prob / R_down = 8 ms, e.g. a 50 000-entry
    # vocabulary at 16 bit over 100 Mbit/s.
    link = M.Link(t_ntt=20e-3, rate_up=100e6, rate_down=100e6)
    V, b = 50000, 16
    assert abs(M.distribution_bits(V, b) / link.rate_down - 8e-3) < 1e-15
    for gamma, alpha, printed_p, printed_t in _table1(golden_dir):
        assert abs(M.reject_probability(alpha, gamma) - printed_p) <= 0.005 + 1e-12
        t = M.dssd_expected_comm_time(alpha, gamma, V, b, link) * 1e3
        assert abs(t - printed_t) <= 0.005 + 1e-9, (gamma, alpha, t, printed_t)
        lo, hi = M.dssd_comm_bounds(V, b, link)
        assert lo <= t / 1e3 <= hi


def test_limits_and_dsd_comparison():
    link = M.Link(t_ntt=20e-3, rate_up=100e6, rate_down=100e6)
    V, b = 50000, 16
    lo, hi = M.dssd_comm_bounds(V, b, link)
    assert abs(M.dssd_expected_comm_time(0.5, 200, V, b, link) - hi) < 1e-12      # gamma -> inf
    assert abs(M.dssd_expected_comm_time(1.0, 8, V, b, link) - lo) < 1e-15        # alpha -> 1
    # DSD uploads gamma distributions, DSSD downloads at most one
    for gamma in (2, 4, 6, 8):
        assert M.dsd_comm_time(gamma, V, b, link) >= gamma * 8e-3 + 20e-3 - 1e-12
        assert M.dssd_expected_comm_time(0.6, gamma, V, b, link) < M.dsd_comm_time(gamma, V, b, link)
    assert M.inference_time(8, 1e-3, 10e-3, 25e-3) == 8 * 1e-3 + 10e-3 + 25e-3
    assert abs(M.dssd_comm_time_from_flags([1, 0, 1, 1], V, b, link) - (0.75 * 8e-3 + 20e-3)) < 1e-15
