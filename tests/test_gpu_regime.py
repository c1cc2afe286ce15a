"""GPU parity: accumulated-gradient norms and the Algorithm 1 decision (integer output,
bit-exact) against the oracle and against hand-written expectations."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc
from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _feed(gpu, ora, g):
    out = H.dev_out(gpu.n_params)
    gpu.step_all([H.to_dev(g)], out)
    if ora is not None:
        ora.step([g])


def test_hand_built_trajectory_and_lr_decay():
    layers = wl.make_layers([(1, 1, 0), (1, 1, 0)])
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, 1, 100, 100)
    norms0 = [1.00, 0.30, 0.28, 0.84, 0.28, 0.27]
    norms1 = [1.00, 0.30, 0.28, 0.28, 0.84, 0.28]
    expect = [[1, 1], [1, 1], [0, 0], [1, 0], [1, 1], [0, 1]]      # written by hand from Algorithm 1
    for wdw in range(6):
        _feed(gpu, ora, np.array([norms0[wdw], norms1[wdw]], np.float32))
        gpu.detect_regime(0.1, 0.1)
        ora.detect_regime(0.1, 0.1)
        assert gpu.get_levels().tolist() == expect[wdw] == ora.level.tolist()
    _feed(gpu, ora, np.array([0.27, 0.28], np.float32))
    gpu.detect_regime(0.1, 0.01)                                    # decay forces critical
    assert gpu.get_levels().tolist() == [1, 1]
    gpu.destroy()


def test_exact_boundary_uses_greater_or_equal():
    layers = wl.make_layers([(1, 3, 0), (1, 3, 0), (1, 3, 0)])
    gpu, _ = H.make_pair(B.ACC_TOPK, layers, 1, 100, 100)
    _feed(gpu, None, np.array([2, 0, 0, 0, 2, 0, 0, 0, 0], np.float32))
    gpu.detect_regime(0.1, 0.1)
    assert gpu.get_levels().tolist() == [1, 1, 1]                   # no history
    old, cur = gpu.get_norms()
    assert cur.tolist() == [2.0, 2.0, 0.0] and old.tolist() == [0.0, 0.0, 0.0]
    # layer 0: ratio exactly 0.5 -> critical; layer 1: just below -> not; layer 2: old == 0 -> critical
    _feed(gpu, None, np.array([1, 0, 0, 0, 1.0000001, 0, 0, 0, 5], np.float32))
    gpu.detect_regime(0.1, 0.1)
    assert gpu.get_levels().tolist() == [1, 0, 1]
    old, cur = gpu.get_norms()
    assert old.tolist() == [2.0, 2.0, 0.0]
    # warm-up (lr grows) is no trigger; norms unchanged -> all non-critical
    _feed(gpu, None, np.array([1, 0, 0, 0, 1.0000001, 0, 0, 0, 5], np.float32))
    gpu.detect_regime(0.1, 0.4)
    assert gpu.get_levels().tolist() == [0, 0, 0]
    gpu.destroy()


def test_norms_accumulate_worker0_raw_gradient_over_multi_tile_layers():
    shapes = [(1, 3 * 8192 + 5, 0), (30, 301, 1), (1, 3, 0)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, 2, 10, 1)
    rng = np.random.default_rng(5)
    for window in range(3):
        for step in range(4):
            grads = [(rng.standard_normal(N) * (0.3 ** window)).astype(np.float32) for _ in range(2)]
            out = H.dev_out(N)
            gpu.step_all([H.to_dev(g) for g in grads], out)
            ora.step(grads)
        if window == 1:
            gpu.reset_accumulator()                                  # measure only part of a window
            ora.reset_accumulator()
            grads = [rng.standard_normal(N).astype(np.float32) * 0.09 for _ in range(2)]
            out = H.dev_out(N)
            gpu.step_all([H.to_dev(g) for g in grads], out)
            ora.step(grads)
        gpu.detect_regime(0.1, 0.1)
        ref = ora.detect_regime(0.1, 0.1)
        assert np.array_equal(gpu.get_levels(), ref)
        old, cur = gpu.get_norms()
        assert np.allclose(cur, ora.norm_curr, rtol=1e-6, atol=0)
        st = gpu.unpack_state(gpu.get_state())
        assert np.all(st["A"] == 0)
        assert np.allclose(st["norm_old"], ora.norm_old, rtol=1e-6, atol=0)
        assert gpu.payload_words()[1] == ora.words_cum
    gpu.destroy()


@pytest.mark.parametrize("method", ["topk", "powersgd"])
def test_window_restart_without_a_pass_over_the_accumulator(method):
    """The sums of squares of A are kept by the pass that adds the gradient, and a window end only
    marks A as restarted.  Everything that looks at A or its norm in between must see what a
    cleared A would give: a test right after a test (norm 0), a state export (zeros), a state import
    followed directly by a test (the imported A's norm), a restart without a decision, steps issued
    call by call with worker 0 last; levels, norms and A itself against the oracle throughout."""
    shapes = [(1, 2 * 8192 + 7, 0), (70, 300, 1), (1, 5, 0), (3, 9000, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    if method == "topk":
        gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    else:
        q0 = wl.q_init(layers, 2, 3)
        gpu, ora = H.make_pair(B.ACC_POWERSGD, layers, W, 2, 1, 100, 0.5, 1, q0)
    rng = np.random.default_rng(31)
    out = H.dev_out(N)

    def step(scale, by_call=False):
        grads = [(rng.standard_normal(N) * scale).astype(np.float32) for _ in range(W)]
        dg = [H.to_dev(g) for g in grads]
        if not by_call:
            gpu.step_all(dg, out)
        else:
            for w in (1, 0):                                         # worker 0 (the one that accumulates) last
                gpu.compress_step(w, dg[w], 0)
            gpu.aggregate(0)
            if method == "powersgd":
                for w in (1, 0):
                    gpu.compress_step(w, None, 1)
                gpu.aggregate(1)
            gpu.decompress(out)
        ora.step(grads)

    def test_now(lr_next=0.1):
        gpu.detect_regime(0.1, lr_next)
        ref = ora.detect_regime(0.1, lr_next)
        assert np.array_equal(gpu.get_levels(), ref)
        old, cur = gpu.get_norms()
        assert np.allclose(cur, ora.norm_curr, rtol=1e-6, atol=0) and np.allclose(old, ora.norm_prev, rtol=1e-6, atol=0)

    def same_accumulator():
        H.assert_bits_equal(gpu.unpack_state(gpu.get_state())["A"], ora.A, "accumulator")

    step(1.0); step(1.0)
    same_accumulator()
    test_now()
    same_accumulator()                                               # exported as zeros
    test_now()                                                       # nothing accumulated: norm 0
    assert np.all(gpu.get_norms()[1] == 0)
    step(0.5, by_call=True)
    same_accumulator()
    step(0.5)
    test_now()
    step(0.4)
    gpu.reset_accumulator(); ora.reset_accumulator()                 # restart without a decision
    same_accumulator()
    step(0.45, by_call=True)
    same_accumulator()
    test_now()
    # import a state in the middle of a window and test at once: the imported A's norm
    step(0.3); step(0.3)
    blob = gpu.get_state().copy()
    step(0.9)
    gpu.set_state(blob)
    st = gpu.unpack_state(blob)
    ora.A[:] = st["A"]
    if method == "powersgd":
        gpu.set_state(H.oracle_state_blob(gpu, ora))                 # (the oracle's e and Q went one step further)
    test_now()
    same_accumulator()
    step(0.3)
    test_now(lr_next=0.01)
    gpu.destroy()
