"""Pins for the oracle's norm accumulation and Algorithm 1 (CPU only)."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc


@pytest.mark.parametrize("old,curr,lr_c,lr_n,has_old,expect", [
    # Algorithm 1 truth table with eta = 0.5
    (2.0, 0.9, 0.1, 0.1, True, True),     # ratio 0.55 >= eta
    (2.0, 1.5, 0.1, 0.1, True, False),    # ratio 0.25 <  eta, no decay
    (2.0, 1.5, 0.1, 0.01, True, True),    # lr decays -> critical regardless
    (2.0, 0.9, 0.1, 0.01, True, True),
    (2.0, 3.5, 0.1, 0.1, True, True),     # growth counts too: |2-3.5|/2 = 0.75
    (2.0, 2.9, 0.1, 0.1, True, False),    # 0.45
    (2.0, 1.0, 0.1, 0.1, True, True),     # exactly eta: ">=" fires
    (2.0, 1.0000001, 0.1, 0.1, True, False),
    (2.0, 1.5, 0.1, 0.4, True, False),    # lr increase (warm-up) is not a trigger
    (0.0, 1.0, 0.1, 0.1, True, True),     # reading: undefined ratio -> critical
    (5.0, 5.0, 0.1, 0.1, False, True),    # reading: no history yet -> critical
])
def test_algorithm1_truth_table(old, curr, lr_c, lr_n, has_old, expect):
    assert orc.regime_is_critical(old, curr, has_old, 0.5, lr_c, lr_n) is expect


def test_layer_norm_closed_forms():
    assert orc.layer_norm(np.array([3, 4], np.float32)) == np.float32(5.0)
    assert orc.layer_norm(np.zeros(7, np.float32)) == 0
    a = np.full(1 << 20, 0.001, np.float32)
    assert abs(float(orc.layer_norm(a)) - float(np.float32(0.001)) * 1024.0) < 1e-6 * 1.024


def test_norm_is_of_the_accumulated_sum_not_sum_of_norms():
    layers = [(0, 1, 4, 0)]
    o = orc.AccordionOracle(orc.TOPK, layers, 1, 100, 100, 100, 0.5, 1)
    g = np.array([1, -2, 3, 0.5], np.float32)
    o.step([g])
    o.step([-g])
    o.detect_regime(0.1, 0.1)
    assert o.norm_curr[0] == 0.0
    o.step([g]); o.step([g])
    o.detect_regime(0.1, 0.1)
    assert o.norm_curr[0] == orc.layer_norm(2 * g)
    assert np.all(o.A == 0)                       # accumulator restarts


def test_hand_built_trajectory_switches_where_eta_predicts():
    """Two layers whose accumulated norms follow prescribed sequences; expected levels
    are written out by hand from Algorithm 1 (eta = 0.5)."""
    layers = [(0, 1, 1, 0), (1, 1, 1, 0)]
    o = orc.AccordionOracle(orc.TOPK, layers, 1, 100, 100, 100, 0.5, 1)
    norms0 = [1.00, 0.30, 0.28, 0.84, 0.28, 0.27]
    norms1 = [1.00, 0.30, 0.28, 0.28, 0.84, 0.28]
    # ratios layer 0:  -,  .70, .067, 2.0, .667, .036  -> 1 1 0 1 1 0
    # ratios layer 1:  -,  .70, .067, 0.0, 2.0,  .667  -> 1 1 0 0 1 1
    expect0 = [1, 1, 0, 1, 1, 0]
    expect1 = [1, 1, 0, 0, 1, 1]
    for wdw in range(6):
        o.step([np.array([norms0[wdw], norms1[wdw]], np.float32)])
        lv = o.detect_regime(0.1, 0.1)
        assert lv.tolist() == [expect0[wdw], expect1[wdw]], wdw
    # a learning-rate decay forces critical even with flat norms
    o.step([np.array([0.27, 0.28], np.float32)])
    assert o.detect_regime(0.1, 0.01).tolist() == [1, 1]


def test_levels_select_rank_and_k():
    layers = [(0, 8, 100, 1), (800, 1, 64, 0)]
    o = orc.AccordionOracle(orc.TOPK, layers, 1, 10, 1, 100, 0.5, 1)
    assert [o.layer_k(0), o.layer_k(1)] == [80, 7]
    o.level[:] = 0
    assert [o.layer_k(0), o.layer_k(1)] == [8, 1]
    q = np.zeros(100 * 4, np.float32)
    p = orc.AccordionOracle(orc.POWERSGD, layers, 1, 4, 1, 100, 0.5, 1, q)
    assert p.layer_rank(0) == 4
    p.level[:] = 0
    assert p.layer_rank(0) == 1


def test_reset_accumulator_without_decision():
    layers = [(0, 1, 3, 0)]
    o = orc.AccordionOracle(orc.TOPK, layers, 1, 100, 100, 100, 0.5, 0)
    o.step([np.ones(3, np.float32)])
    o.reset_accumulator()
    assert np.all(o.A == 0) and o.level.tolist() == [0] and o.has_old.tolist() == [0]
