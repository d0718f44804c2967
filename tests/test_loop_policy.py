"""Host policy of the decoding loop: the adaptive N_d / N_i update rule (App. J), checked against the cases
its two equations spell out.  (loop.py is host-only code; importing it does not load the GPU library.)"""
import importlib.util
import os

_spec = importlib.util.spec_from_file_location(
    "hs_loop", os.path.join(os.path.dirname(__file__), "..", "paper_2510_01336_amd", "loop.py"))
loop = importlib.util.module_from_spec(_spec)
import sys
sys.modules["hs_loop"] = loop
_spec.loader.exec_module(loop)


def test_nd_rule_cases():
    # thresholds 0.5 / 0.8, bounds [1, 3] (the appendix's initial bounds)
    step = lambda v, r: loop.adapt_step(v, r, 0.5, 0.8, 1, 3)
    assert step(2, 0.8) == 3          # at the high threshold: up
    assert step(2, 0.95) == 3
    assert step(3, 1.0) == 3          # clamped at the maximum
    assert step(2, 0.49) == 1         # below the low threshold: down
    assert step(1, 0.0) == 1          # clamped at the minimum
    assert step(2, 0.5) == 2          # the low threshold itself is not "below"
    assert step(2, 0.79) == 2         # in between: unchanged


def test_ni_rule_cases():
    step = lambda v, r: loop.adapt_step(v, r, 0.3, 0.8, 3, 8)
    assert [step(4, r) for r in (0.0, 0.29, 0.3, 0.5, 0.8, 1.0)] == [3, 3, 4, 4, 5, 5]
    assert step(8, 0.9) == 8 and step(3, 0.1) == 3


def test_trajectory_is_monotone_under_constant_rate():
    v, seen = 2, []
    for _ in range(5):
        v = loop.adapt_step(v, 0.9, 0.5, 0.8, 1, 6)
        seen.append(v)
    assert seen == [3, 4, 5, 6, 6]
