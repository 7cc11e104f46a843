"""Pins for oracle/analysis.py: the numbers the paper prints (tests/golden/)."""
import os

import numpy as np

from oracle import analysis

G = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    out = []
    for line in open(os.path.join(G, name)):
        line = line.split("#")[0].strip()
        if line:
            out.append(line.split())
    return out


def test_table1_operations_and_speed():
    for a, g, ops, speed in rows("table1_ops_speed.txt"):
        a, g = float(a), int(g)
        assert abs(analysis.ops_increase(a, g, 0.0) - float(ops)) <= 0.0051
        assert abs(analysis.walltime_improvement(a, g, 0.0) - float(speed)) <= 0.0051


def test_table4_expected_column():
    for g, a, c, exp in rows("table4_expected_speedup.txt"):
        assert abs(analysis.walltime_improvement(float(a), int(g), float(c)) - float(exp)) <= 0.1


def test_misc_printed_numbers():
    for kind, a, g, c, val, tol in rows("misc_closed_forms.txt"):
        assert kind == "walltime"
        assert abs(analysis.walltime_improvement(float(a), int(g), float(c)) - float(val)) <= float(tol)


def test_equation1_is_the_mean_of_the_capped_geometric():
    for a in (0.0, 0.3, 0.75, 0.99):
        for g in (1, 3, 7, 10):
            pmf = analysis.capped_geometric_pmf(a, g)
            assert abs(pmf.sum() - 1) < 1e-12
            assert abs(np.sum((np.arange(g + 1) + 1) * pmf) - analysis.expected_tokens(a, g)) < 1e-12
    assert analysis.expected_tokens(1.0, 5) == 6.0
    assert abs(analysis.expected_tokens(0.999999, 5) - 6.0) < 1e-4


def test_corollary_3_9_and_optimal_gamma():
    for a, c in ((0.5, 0.1), (0.8, 0.02), (0.3, 0.2)):
        assert abs(analysis.walltime_improvement(a, 1, c) - analysis.min_improvement(a, c)) < 1e-12
        g = analysis.optimal_gamma(a, c)
        best = analysis.walltime_improvement(a, g, c)
        assert all(best >= analysis.walltime_improvement(a, k, c) - 1e-12 for k in range(1, 65))
    # negligible-cost drafts: improvement approaches 1/(1-alpha) (section 3.6)
    assert abs(analysis.walltime_improvement(0.5, 60, 0.0) - 2.0) < 1e-9
    # more expensive drafts never call for longer speculation
    assert analysis.optimal_gamma(0.8, 0.01) >= analysis.optimal_gamma(0.8, 0.1)
