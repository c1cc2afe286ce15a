"""Pins of the comparison detector's statistic (mean to standard deviation ratio, Section 5.6
"Comparison with Prior Work") and of the switching rule as this build reads it."""
import numpy as np

from oracle import accordion_oracle as orc

F32 = np.float32


def test_streaming_form_equals_the_definition():
    rng = np.random.default_rng(1)
    for n, t in ((1, 2), (7, 3), (300, 10), (5000, 50)):
        gs = [(rng.standard_normal(n) * 0.1 + 0.05).astype(F32) for _ in range(t)]
        direct = orc.msdr(gs)
        a = np.sum(np.asarray(gs, np.float64), axis=0)
        sq = sum(float(np.dot(g.astype(np.float64), g.astype(np.float64))) for g in gs)
        assert np.isclose(orc.msdr_streaming(a, sq, t), direct, rtol=1e-6)


def test_closed_forms():
    # the same gradient every step: no spread at all
    g = np.array([1.0, -2.0, 3.0], F32)
    assert orc.msdr([g, g, g]) == F32(np.inf)
    # two gradients m + d and m - d: mean m, spread ||d||
    m, d = np.array([3.0, 4.0]), np.array([0.0, 2.0])
    assert np.isclose(orc.msdr([(m + d).astype(F32), (m - d).astype(F32)]), 5.0 / 2.0, rtol=1e-7)
    # zero mean: ratio 0
    assert orc.msdr([d.astype(F32), (-d).astype(F32)]) == F32(0.0)
    # scale invariance, and the textbook value for mean mu*1 plus unit noise in n dimensions:
    # ||mean|| ~ mu sqrt(n) (T large), spread ~ sqrt(n (T-1)/T)
    rng = np.random.default_rng(2)
    n, t, mu = 4000, 200, 0.5
    gs = [(mu + rng.standard_normal(n)).astype(F32) for _ in range(t)]
    val = orc.msdr(gs)
    expect = np.sqrt(mu * mu + 1.0 / t) / np.sqrt((t - 1) / t)
    assert abs(val / expect - 1.0) < 0.02
    assert np.isclose(orc.msdr([7.0 * g for g in gs]), val, rtol=1e-5)


def test_switch_rule_reading():
    assert not orc.msdr_should_switch(0.0, 0.1, False, 0.5)        # nothing to compare with
    assert orc.msdr_should_switch(2.0, 1.0, True, 0.5)             # dropped by exactly one half
    assert not orc.msdr_should_switch(2.0, 1.0000001, True, 0.5)
    assert not orc.msdr_should_switch(2.0, 3.0, True, 0.5)         # a rise never switches


def test_detector_trajectory_by_hand():
    """One layer, windows of 8 steps: gradient = mean + noise with the mean shrinking by window.
    Window 0 sets the reference; a window whose ratio is at most half the reference moves the
    layer to the accurate level (1) and becomes the reference; the level never returns."""
    rng = np.random.default_rng(3)
    n = 2000
    o = orc.AccordionOracle(orc.TOPK, [(0, 1, n, 0)], 1, 10, 1, 100, 0.5, 0, None, detector="msdr")
    levels, ratios = [], []
    for mean in (1.0, 0.8, 0.1, 0.1, 2.0, 0.0):
        for _ in range(8):
            o.step([(mean + rng.standard_normal(n)).astype(F32)])
        levels.append(int(o.detect_regime(0.1, 0.01)[0]))          # the rate decay plays no role here
        ratios.append(float(o.norm_curr[0]))
    # ratios ~ sqrt(mean^2 + 1/8) / sqrt(7/8): 1.13, 0.94, 0.39, 0.39, 2.17, 0.38
    expect = [np.sqrt(m * m + 0.125) / np.sqrt(0.875) for m in (1.0, 0.8, 0.1, 0.1, 2.0, 0.0)]
    assert np.allclose(ratios, expect, rtol=0.05)
    assert levels == [0, 0, 1, 1, 1, 1]
    assert np.isclose(o.norm_old[0], ratios[2])               # the reference moved at the switch only
    assert o.T == 0 and np.all(o.sq == 0) and np.all(o.A == 0)
