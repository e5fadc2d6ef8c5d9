"""Adaptive speculation length selector (paper section 3.3): the oracle against what the mathematics
fixes, then the C-ABI object (host code, no GPU work) against the oracle, decision by decision."""
import math

import numpy as np
import pytest

from oracle import minions_oracle as orc
from paper_2402_15678_amd import synth


# ---------------------------------------------------------------- pins of the oracle
def test_slope_of_an_exact_line_is_its_coefficient():
    for a, b, m in [(3.0, 0.5, 2), (-1.25, 2.0, 7), (0.0, -0.125, 16), (10.0, 0.0, 5)]:
        y = [a + b * i for i in range(m)]          # dyadic values: every step is exact
        assert orc.fit_slope(y) == b


def test_slope_matches_the_library_fit_and_the_normal_equations():
    g = synth.stream(5, 1)
    for m in (2, 3, 8, 33):
        y = g.normal(size=m) * 3.0 + np.arange(m) * 0.1
        x = np.arange(m, dtype=np.float64)
        lib = np.polyfit(x, y, 1)[0]
        # normal equations written out: (m sum xy - sum x sum y) / (m sum x^2 - (sum x)^2)
        ne = (m * (x * y).sum() - x.sum() * y.sum()) / (m * (x * x).sum() - x.sum() ** 2)
        got = orc.fit_slope(list(y))
        assert abs(got - lib) < 1e-11 and abs(got - ne) < 1e-11


def test_slope_is_odd_under_reversal_and_blind_to_offsets():
    g = synth.stream(5, 2)
    y = list(g.normal(size=11))
    assert abs(orc.fit_slope(y) + orc.fit_slope(y[::-1])) < 1e-13
    assert abs(orc.fit_slope(y) - orc.fit_slope([v + 100.0 for v in y])) < 1e-10


def test_selector_decisions_follow_the_text():
    # rising t/vl since the last change: the step was too aggressive -> s goes down by s_penalty
    sel = orc.Selector(8, 1, 16, 4, 2, 1)
    for i in range(3):
        assert sel.observe(10.0 + i, 2.0) == 8          # fewer than decision_threshold samples: no change
    assert sel.observe(13.0, 2.0) == 6 and sel.adjustments == 1 and sel.last_slope == 0.5
    # falling trend: there is room -> s goes up by s_reward; the list starts empty after a decision
    for i in range(3):
        assert sel.observe(9.0 - i, 3.0) == 6
    assert sel.observe(6.0, 3.0) == 7
    # flat trend takes the else branch (reward)
    for _ in range(3):
        sel.observe(5.0, 1.0)
    assert sel.observe(5.0, 1.0) == 8
    # clamped at both ends
    lo = orc.Selector(1, 1, 4, 2, 3, 3)
    lo.observe(1.0, 1.0)
    assert lo.observe(2.0, 1.0) == 1
    hi = orc.Selector(4, 1, 4, 2, 3, 3)
    hi.observe(2.0, 1.0)
    assert hi.observe(1.0, 1.0) == 4


def test_selector_settles_near_the_minimum_of_a_convex_cost():
    # t_LLM / vl as a function of s with its minimum at s = 6 (the shape the paper's motivation reports):
    # the heuristic hovers around it once it gets there
    cost = lambda s: 1.0 + 0.02 * (s - 6) ** 2
    sel = orc.Selector(1, 1, 16, 3, 1, 1)
    prev = sel.s
    trace = []
    for step in range(200):
        # the monitored value drifts from the cost of the previous s to the cost of the current one
        n_in = len(sel.samples)
        y = cost(prev) + (cost(sel.s) - cost(prev)) * (n_in + 1) / 3.0
        before = sel.s
        sel.observe(y, 1.0)
        if sel.s != before or len(sel.samples) == 0:
            prev = before
        trace.append(sel.s)
    assert all(4 <= s <= 8 for s in trace[60:])


# ---------------------------------------------------------------- the C-ABI object against the oracle
@pytest.fixture(scope="module")
def binding():
    from paper_2402_15678_amd import binding as b
    return b


def test_abi_selector_matches_the_oracle_decision_by_decision(binding):
    g = synth.stream(9, 3)
    for case in range(6):
        thr = int(g.integers(2, 9))
        pen, rew = int(g.integers(0, 4)), int(g.integers(0, 4))
        s_min, s_max = 1, int(g.integers(4, 20))
        s0 = int(g.integers(s_min, s_max + 1))
        ref = orc.Selector(s0, s_min, s_max, thr, pen, rew)
        sel = binding.mn_selector_create(s0, s_min, s_max, thr, pen, rew)
        try:
            for step in range(120):
                t = float(g.random() * 40.0 + 5.0)
                vl = float(g.integers(1, 10)) + float(g.integers(0, 4)) * 0.25
                want = ref.observe(t, vl)
                got, slope = binding.mn_selector_observe(sel, t, vl)
                assert got == want == binding.mn_selector_current(sel)
                if math.isnan(ref.last_slope):
                    assert math.isnan(slope)
                else:
                    assert slope == ref.last_slope          # same formula, same order, fp64 on both sides
            assert binding.mn_selector_adjustments(sel) == ref.adjustments
        finally:
            binding.mn_selector_destroy(sel)


def test_abi_selector_rejects_bad_arguments(binding):
    from paper_2402_15678_amd.binding import MinionsError
    for args in [(0, 1, 4, 3, 1, 1), (5, 1, 4, 3, 1, 1), (2, 3, 1, 3, 1, 1), (2, 1, 4, 1, 1, 1), (2, 1, 4, 3, -1, 1)]:
        with pytest.raises(MinionsError):
            binding.mn_selector_create(*args)
    sel = binding.mn_selector_create(3, 1, 8, 2, 1, 1)
    try:
        for t, vl in [(1.0, 0.0), (-1.0, 2.0), (float("nan"), 1.0), (1.0, float("inf"))]:
            with pytest.raises(MinionsError):
                binding.mn_selector_observe(sel, t, vl)
        assert binding.mn_selector_current(sel) == 3 and binding.mn_selector_adjustments(sel) == 0
    finally:
        binding.mn_selector_destroy(sel)
    assert binding.mn_selector_current(None) == -1
