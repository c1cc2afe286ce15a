"""GPU parity at the limits of the configuration: the maximum number of workers (32), ranks above
min(rows, cols), one-element layers, every method."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc
from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H
from tests.test_gpu_powersgd import _forced_step
from tests.test_gpu_topk import _check_step

pytestmark = pytest.mark.gpu

W_MAX = 32


def test_topk_with_the_maximum_number_of_workers():
    print("case limits topk W=32", flush=True)
    layers = wl.make_layers([(1, 8192 + 5, 0), (7, 33, 1), (1, 1, 0)])
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W_MAX, 10, 1)
    rng = np.random.default_rng(1)
    for step in range(2):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W_MAX)]
        _check_step(gpu, ora, grads, f"step {step}")
    common, kept = gpu.topk_overlap(0, W_MAX - 1)
    assert common[2] == 1 and kept[2] == 1                   # the one-element layer is always kept
    gpu.destroy()


def test_powersgd_with_the_maximum_number_of_workers_and_capped_ranks():
    print("case limits powersgd W=32", flush=True)
    layers = wl.make_layers([(3, 700, 1), (70, 2, 1), (1, 50, 0), (40, 300, 1), (1, 1, 1)])
    lt = H.layer_tuples(layers)
    N = wl.total_params(layers)
    rng = np.random.default_rng(2)
    q0 = rng.standard_normal(sum(c for (_, r, c, m) in lt if m) * 4).astype(np.float32)
    gpu, ora = H.make_pair(B.ACC_POWERSGD, layers, W_MAX, 4, 1, 100, 0.5, 1, q0)
    assert [ora.layer_rank(li) for li in (0, 1, 3, 4)] == [3, 2, 4, 1]
    for step in range(2):
        grads = [(rng.standard_normal(N) * 0.01).astype(np.float32) for _ in range(W_MAX)]
        _forced_step(gpu, ora, grads, f"step {step}")
    gpu.destroy()


def test_batch_mode_with_the_maximum_number_of_workers():
    print("case limits batch W=32", flush=True)
    layers = wl.make_layers([(1, 8192 + 5, 0), (7, 33, 1)])
    lt = H.layer_tuples(layers)
    N = wl.total_params(layers)
    gpu = B.Accordion(B.ACC_BATCH, lt, W_MAX, 1, 1, 100, 0.5, 0, None, batch_multiplier=3)
    ora = orc.BatchSizeOracle(lt, W_MAX, 3, 0.5, 0, True)
    rng = np.random.default_rng(3)
    out = H.dev_out(N)
    for t in range(6):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W_MAX)]
        d, n = ora.micro_step(grads)
        gpu.step_all([H.to_dev(g) for g in grads], out)
        if d is not None:
            H.assert_bits_equal(out.cpu().numpy(), d, f"micro-step {t}")
    assert gpu.batch_status()["exchanges"] == 2
    with pytest.raises(B.AccordionError):
        B.Accordion(B.ACC_BATCH, lt, W_MAX + 1, 1, 1, 100, 0.5, 0, None, batch_multiplier=3)
    gpu.destroy()
