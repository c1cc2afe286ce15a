"""GPU parity of the comparison detector (mean to standard deviation ratio, Section 5.6) against
the oracle: free-running TopK (bit-exact steps), ratios to 1e-6, identical level vectors."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc
from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H
from tests.test_gpu_topk import _check_step

pytestmark = pytest.mark.gpu


def _pair(method, layers, W, crit, noncrit, eta, q0=None):
    lt = H.layer_tuples(layers)
    gpu = B.Accordion(method, lt, W, crit, noncrit, 100, eta, 0, q0, detector=B.ACC_DETECT_MSDR)
    ora = orc.AccordionOracle(method, lt, W, crit, noncrit, 100, eta, 0, q0, detector="msdr")
    return gpu, ora


@pytest.mark.parametrize("mode", ["all", "calls"])
def test_msdr_windows_topk(mode):
    """Per-layer mean shrinking by window at different speeds, so that layers switch at
    different windows; ragged multi-tile layers."""
    print(f"case msdr {mode}", flush=True)
    shapes = [(1, 2 * 8192 + 77, 0), (37, 1001, 1), (1, 5, 0), (3, 8192, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    gpu, ora = _pair(B.ACC_TOPK, layers, W, 10, 1, 0.5)
    rng = np.random.default_rng(3)
    means = {0: [1.0, 0.8, 0.1, 0.1], 1: [1.0, 1.0, 1.0, 0.05], 2: [1.0, 1.0, 1.0, 1.0], 3: [2.0, 0.1, 0.1, 0.0]}
    out = H.dev_out(N)
    history = []
    for window in range(4):
        mu = np.concatenate([np.full(l.numel, means[li][window]) for li, l in enumerate(layers)])
        for s in range(8):
            grads = [(mu + rng.standard_normal(N)).astype(np.float32) for _ in range(W)]
            if mode == "all":
                _check_step(gpu, ora, grads, f"window {window} step {s}")
            else:
                ora.step(grads)
                dg = [H.to_dev(g) for g in grads]
                for w in (1, 0):
                    gpu.compress_step(w, dg[w], 0)
                gpu.aggregate(0)
                gpu.decompress(out)
        if window == 2:                                      # a restart without a decision
            gpu.reset_accumulator()
            ora.reset_accumulator()
            for s in range(8):
                grads = [(mu + rng.standard_normal(N)).astype(np.float32) for _ in range(W)]
                _check_step(gpu, ora, grads, f"window {window} extra step {s}")
        ref = ora.detect_regime(0.1, 0.01)
        gpu.detect_regime(0.1, 0.01)
        lv = gpu.get_levels()
        assert np.array_equal(lv, ref), f"window {window}: {lv} vs {ref}"
        old, cur = gpu.get_norms()
        assert np.allclose(cur, ora.norm_curr, rtol=1e-6), (cur, ora.norm_curr)
        assert np.allclose(old, ora.norm_prev, rtol=1e-6)
        history.append(lv.tolist())
    # layer 0 switches after window 2, layer 3 after window 1, layer 1 after window 3; the
    # 5-element layer only has to agree with the oracle (its ratio is noisy)
    assert [h[0] for h in history] == [0, 0, 1, 1]
    assert [h[3] for h in history] == [0, 1, 1, 1]
    assert [h[1] for h in history] == [0, 0, 0, 1]
    assert gpu.payload_words()[1] == ora.words_cum
    gpu.destroy()


def test_msdr_with_powersgd_and_config_errors():
    layers = wl.make_layers([(64, 576, 1), (1, 300, 0)])
    lt = H.layer_tuples(layers)
    N = wl.total_params(layers)
    rng = np.random.default_rng(5)
    q0 = rng.standard_normal(576 * 2).astype(np.float32)
    gpu, ora = _pair(B.ACC_POWERSGD, layers, 1, 2, 1, 0.5, q0)
    out = H.dev_out(N)
    for window, mean in enumerate((1.0, 0.1)):
        for s in range(6):
            g = [(mean + rng.standard_normal(N)).astype(np.float32)]
            gpu.step_all([H.to_dev(g[0])], out)
            ora.step(g)
        ref = ora.detect_regime(0.1, 0.1)
        gpu.detect_regime(0.1, 0.1)
        assert np.array_equal(gpu.get_levels(), ref)
        assert np.allclose(gpu.get_norms()[1], ora.norm_curr, rtol=1e-6)
    assert ref.tolist() == [1, 1]
    gpu.destroy()
    with pytest.raises(B.AccordionError):
        B.Accordion(B.ACC_BATCH, lt, 1, 1, 1, 100, 0.5, 1, None, batch_multiplier=2, detector=B.ACC_DETECT_MSDR)
    with pytest.raises(B.AccordionError):
        B.Accordion(B.ACC_TOPK, lt, 1, 10, 1, 100, 1.0, 1, None, detector=B.ACC_DETECT_MSDR)
    with pytest.raises(B.AccordionError):
        B.Accordion(B.ACC_TOPK, lt, 1, 10, 1, 100, 0.5, 1, None, detector=7)
