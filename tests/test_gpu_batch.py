"""GPU parity of the batch-size mode (method ACC_BATCH) against the oracle's BatchSizeOracle,
through the C ABI: every sum, the exchanged mean, the optimizer step, the accumulator, the
exchange counters and the whole-model decision are bit-exact (fp32 sums in a fixed order; the
norm is an fp64 sum on both sides and is compared to 1e-6)."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc
from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _make(layers, W, M, initial_level=1, monotone=1, eta=0.5):
    lt = H.layer_tuples(layers)
    gpu = B.Accordion(B.ACC_BATCH, lt, W, 1, 1, 100, eta, initial_level, None,
                      batch_multiplier=M, batch_monotone=monotone)
    ora = orc.BatchSizeOracle(lt, W, M, eta, initial_level, bool(monotone))
    assert gpu.n_params == ora.N
    return gpu, ora


def _ragged_layers():
    small = wl.random_layers(seed=31, n_layers=7, max_rows=30, max_cols=200)
    base = max(l.offset + l.rows * l.cols for l in small)
    base = (base + 7) // 4 * 4 + 3                                   # misaligned, with a gap before
    return H.layer_tuples(small) + [(base, 1, 2 * 8192 + 77, 0), (base + 2 * 8192 + 77 + 1, 19, 1001, 1)]


def _check_state(gpu, ora, tag):
    st = gpu.unpack_state(gpu.get_state())
    m = ora.mask
    H.assert_bits_equal(st["A"][m], ora.A[m], f"{tag}: accumulator")
    assert st["pending"] == ora.j, tag
    if ora.j > 0:                                                    # the sums of an open batch
        H.assert_bits_equal(st["e"][:, m], ora.S[:, m], f"{tag}: sums")
    assert np.all(st["level"] == ora.level), tag
    s = gpu.batch_status()
    assert (s["level"], s["pending"], s["exchanges"]) == (ora.level, ora.j, ora.exchanges), tag
    assert gpu.payload_words() == (ora.words_last, ora.words_cum), tag


@pytest.mark.parametrize("W,M", [(1, 2), (3, 4), (5, 3)])
def test_micro_steps_store_path(W, M):
    """Small batch (every micro-step exchanged), then the switch to the large batch by the
    detector, then several large batches; the output buffer must stay untouched on micro-steps
    that complete nothing."""
    print(f"case batch store W={W} M={M}", flush=True)
    gpu, ora = _make(_ragged_layers(), W, M)
    N = ora.N
    rng = np.random.default_rng([4, W, M])
    out = H.to_dev(np.full(N, -7.0, np.float32))
    expect_out = np.full(N, -7.0, np.float32)
    t = 0
    for window in range(3):
        scale = [1.0, 1.0, 0.98][window]                              # window 2 ~ window 1: non-critical
        for _ in range(2 * M + 1):
            grads = [(rng.standard_normal(N) * scale).astype(np.float32) for _ in range(W)]
            d, n_micro = ora.micro_step(grads)
            gpu.step_all([H.to_dev(g) for g in grads], out)
            if d is not None:
                expect_out[ora.mask] = d[ora.mask]
            H.assert_bits_equal(out.cpu().numpy(), expect_out, f"micro-step {t}: out")
            assert gpu.batch_status()["last_batch"] == n_micro
            _check_state(gpu, ora, f"micro-step {t}")
            t += 1
        ref = ora.detect_regime(0.1, 0.1)
        gpu.detect_regime(0.1, 0.1)
        assert np.all(gpu.get_levels() == ref), f"window {window}"
        old, cur = gpu.get_norms()
        assert np.allclose(cur, ora.norm_curr, rtol=1e-6) and np.allclose(old, ora.norm_prev, rtol=1e-6)
        _check_state(gpu, ora, f"after window {window}")
    assert ora.level == 0 and ora.exchanges < t                       # the large batch was reached
    gpu.destroy()


def test_micro_steps_update_path_scales_the_learning_rate():
    print("case batch update", flush=True)
    W, M = 2, 4
    gpu, ora = _make(_ragged_layers(), W, M, initial_level=1)
    N = ora.N
    rng = np.random.default_rng(6)
    w_ref = rng.standard_normal(N).astype(np.float32)
    v_ref = np.zeros(N, np.float32)
    w_dev, v_dev = H.to_dev(w_ref), H.to_dev(v_ref)
    lr, mu, wd = 0.05, 0.9, 1e-4
    applied = []
    for t in range(3 + 3 * M):
        if t == 3:                                                    # by hand: to the large batch
            ora.level = 0
            st = gpu.unpack_state(gpu.get_state())
            gpu.set_state(gpu.pack_state(st["e"], st["A"], None, st["norm_old"], st["has_old"],
                                         np.zeros(gpu.n_layers, np.int32), st["pending"]))
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        applied.append(ora.micro_step_update(grads, w_ref, v_ref, lr, mu, wd))
        gpu.step_all_update([H.to_dev(g) for g in grads], w_dev, v_dev, lr, mu, wd)
        H.assert_bits_equal(w_dev.cpu().numpy(), w_ref, f"micro-step {t}: weights")
        H.assert_bits_equal(v_dev.cpu().numpy(), v_ref, f"micro-step {t}: velocity")
        _check_state(gpu, ora, f"micro-step {t}")
    assert applied == [1, 1, 1] + [0, 0, 0, M] * 3
    gpu.destroy()


def test_state_round_trip_in_the_middle_of_a_batch_and_monotone_rule():
    W, M = 2, 4
    layers = wl.make_layers([(1, 9000, 0), (12, 50, 1)])
    gpu, ora = _make(layers, W, M, initial_level=0, monotone=1)
    twin, _ = _make(layers, W, M, initial_level=0, monotone=0)
    N = ora.N
    rng = np.random.default_rng(8)
    out, out2 = H.dev_out(N), H.dev_out(N)
    for t in range(2):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        ora.micro_step(grads)
        gpu.step_all([H.to_dev(g) for g in grads], out)
    blob = gpu.get_state()
    twin.set_state(blob)                                              # pending = 2 travels along
    assert twin.batch_status()["pending"] == 2
    for t in range(2):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        d, n = ora.micro_step(grads)
        dg = [H.to_dev(g) for g in grads]
        gpu.step_all(dg, out)
        twin.step_all(dg, out2)
    assert n == M
    H.assert_bits_equal(out.cpu().numpy(), d, "batch completed after the round trip")
    H.assert_bits_equal(out2.cpu().numpy(), d, "twin")
    # a learning-rate decay is critical for Algorithm 1; the batch only grows when asked to
    gpu.detect_regime(0.1, 0.01)
    twin.detect_regime(0.1, 0.01)
    assert ora.detect_regime(0.1, 0.01) == 0
    assert np.all(gpu.get_levels() == 0) and np.all(twin.get_levels() == 1)
    gpu.destroy()
    twin.destroy()


def test_errors_of_the_batch_mode():
    layers = wl.make_layers([(1, 40, 0)])
    gpu, _ = _make(layers, 1, 2)
    g = H.to_dev(np.ones(40, np.float32))
    out = H.dev_out(40)
    for call in (lambda: gpu.compress_step(0, g, 0), lambda: gpu.aggregate(0), lambda: gpu.decompress(out)):
        with pytest.raises(B.AccordionError) as ei:
            call()
        assert ei.value.status == B.ACC_EINVAL and "batch-size mode" in str(ei.value)
    st = gpu.unpack_state(gpu.get_state())
    with pytest.raises(B.AccordionError):                             # pending outside [0, M)
        gpu.set_state(gpu.pack_state(st["e"], st["A"], None, st["norm_old"], st["has_old"], st["level"], 2))
    with pytest.raises(B.AccordionError):
        gpu.topk_stats()
    gpu.step_all([g], out)
    assert np.all(out.cpu().numpy() == 1.0)
    gpu.destroy()
