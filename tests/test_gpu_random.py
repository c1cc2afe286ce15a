"""GPU parity on seeded random configurations: layer sets with gaps and misaligned offsets,
1-5 workers, any kept fraction or rank pair, value distributions with and without ties, a level
switch in the middle.  Same bars as the hand-written cases: TopK and the batch-size mode bit for
bit, PowerSGD 1e-5 relative (teacher-forced)."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc
from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H
from tests.test_gpu_powersgd import _forced_step

pytestmark = pytest.mark.gpu


def _values(rng, kind, n):
    if kind == 0:
        return rng.standard_normal(n)
    if kind == 1:
        return rng.integers(-3, 4, n) * 0.25                 # seven values: large tie classes
    if kind == 2:
        return rng.standard_normal(n) * (rng.random(n) < 0.04)   # sparse: threshold among zeros
    if kind == 3:
        return rng.laplace(0, 1e-3, n)
    return np.round(rng.standard_normal(n), 1)


def _random_layers(rng, max_rows, max_cols, max_vec):
    lt, off = [], int(rng.integers(0, 4))
    for _ in range(int(rng.integers(1, 8))):
        if rng.random() < 0.4:
            r, c, m = 1, int(rng.integers(1, max_vec)), 0
        else:
            r, c, m = int(rng.integers(1, max_rows)), int(rng.integers(1, max_cols)), 1
        lt.append((off, r, c, m))
        off += r * c + int(rng.integers(0, 4))
    n = max(o + r * c for (o, r, c, _) in lt)
    mask = np.zeros(n, bool)
    for (o, r, c, _) in lt:
        mask[o:o + r * c] = True
    return lt, n, mask


@pytest.mark.parametrize("seed", range(16))
def test_topk_random_configuration(seed):
    rng = np.random.default_rng(1000 + seed)
    lt, N, mask = _random_layers(rng, 60, 1500, 40000)
    W = int(rng.integers(1, 6))
    den = int(rng.choice([100, 1000, 7]))
    crit, noncrit = int(rng.integers(1, den + 1)), int(rng.integers(1, den + 1))
    print(f"case random topk seed {seed}: {lt} W {W} K {crit}/{noncrit}/{den}", flush=True)
    gpu = B.Accordion(B.ACC_TOPK, lt, W, crit, noncrit, den)
    ora = orc.AccordionOracle(orc.TOPK, lt, W, crit, noncrit, den)
    ora.N, ora.e, ora.A = N, np.zeros((W, N), np.float32), np.zeros(N, np.float32)
    steps = int(rng.integers(3, 7))
    out = H.dev_out(N)
    for s in range(steps):
        grads = [(_values(rng, int(rng.integers(0, 5)), N) * mask).astype(np.float32) for _ in range(W)]
        if s == steps // 2:                                  # switch the level through the state blob
            st = gpu.unpack_state(gpu.get_state())
            H.assert_bits_equal(st["e"][:, mask], ora.e[:, mask], "memory before the switch")
            ora.level[:] = 1 - ora.level
            gpu.set_state(gpu.pack_state(st["e"], st["A"], None, st["norm_old"], st["has_old"], ora.level))
        out_ref = ora.step(grads)
        gpu.step_all([H.to_dev(g) for g in grads], out)
        H.assert_bits_equal(out.cpu().numpy()[mask], out_ref[mask], f"step {s}: mean")
        for w in range(W):
            for li in range(len(lt)):
                idx, val = gpu.get_payload(w, li)
                assert np.array_equal(idx, ora.payload[(w, li)][0]), (s, w, li)
                H.assert_bits_equal(val, ora.payload[(w, li)][1], f"step {s}: values")
    st = gpu.unpack_state(gpu.get_state())
    H.assert_bits_equal(st["e"][:, mask], ora.e[:, mask], "final memory")
    H.assert_bits_equal(st["A"][mask], ora.A[mask], "final accumulator")
    assert gpu.payload_words() == (ora.words_last, ora.words_cum)
    gpu.destroy()


@pytest.mark.parametrize("seed", range(10))
def test_powersgd_random_thin_and_short_matrices(seed):
    """Matrix families on which the orthogonalisation is touchy: one to three columns (P_bar is
    as ill-conditioned as the small random warm start) and fewer than eight rows (the rank is
    capped near the row count), with gradient scales that jump by up to four orders of magnitude
    between steps (the memory then dominates and P_bar is almost rank-deficient).  Same 1e-5."""
    rng = np.random.default_rng(7000 + seed)
    shapes = []
    for _ in range(int(rng.integers(2, 7))):
        u = rng.random()
        if u < 0.4:
            shapes.append((int(rng.integers(1, 700)), int(rng.integers(1, 4)), 1))
        elif u < 0.8:
            shapes.append((int(rng.integers(1, 8)), int(rng.integers(1, 1500)), 1))
        else:
            shapes.append((1, int(rng.integers(1, 3000)), 0))
    layers = wl.make_layers(shapes)
    lt = H.layer_tuples(layers)
    N = wl.total_params(layers)
    W = int(rng.integers(1, 6))
    crit, noncrit = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    print(f"case random thin/short powersgd seed {seed}: {shapes} W {W} ranks {crit}/{noncrit}", flush=True)
    q0 = rng.standard_normal(sum(c for (_, r, c, m) in lt if m) * max(crit, noncrit)).astype(np.float32)
    gpu, ora = H.make_pair(B.ACC_POWERSGD, layers, W, crit, noncrit, 100, 0.5, 1, q0)
    for s in range(4):
        if s == 2:
            ora.level[:] = 0
        scale = 10.0 ** rng.uniform(-4, 0)
        grads = [(rng.standard_normal(N) * scale).astype(np.float32) for _ in range(W)]
        _forced_step(gpu, ora, grads, f"seed {seed} step {s}")
    gpu.destroy()


@pytest.mark.parametrize("seed", range(10))
def test_powersgd_and_batch_mode_random_configuration(seed):
    rng = np.random.default_rng(5000 + seed)
    shapes = []
    for _ in range(int(rng.integers(1, 7))):
        if rng.random() < 0.3:
            shapes.append((1, int(rng.integers(1, 20000)), 0))
        else:
            shapes.append((int(rng.integers(1, 700)), int(rng.integers(1, 1500)), 1))
    layers = wl.make_layers(shapes)
    lt = H.layer_tuples(layers)
    N = wl.total_params(layers)
    W = int(rng.integers(1, 6))
    crit, noncrit = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    print(f"case random powersgd seed {seed}: {shapes} W {W} ranks {crit}/{noncrit}", flush=True)
    q0 = rng.standard_normal(sum(c for (_, r, c, m) in lt if m) * max(crit, noncrit)).astype(np.float32)
    gpu, ora = H.make_pair(B.ACC_POWERSGD, layers, W, crit, noncrit, 100, 0.5, 1, q0)
    for s in range(3):
        if s == 2:
            ora.level[:] = 0
        scale = 10.0 ** rng.uniform(-4, 0)
        grads = [(rng.standard_normal(N) * scale).astype(np.float32) for _ in range(W)]
        _forced_step(gpu, ora, grads, f"seed {seed} step {s}")
    gpu.destroy()
    # the batch-size mode with the fused update on the same layer set
    M = int(rng.integers(1, 5))
    level = int(rng.integers(0, 2))
    gb = B.Accordion(B.ACC_BATCH, lt, W, 1, 1, 100, 0.5, level, None, batch_multiplier=M)
    ob = orc.BatchSizeOracle(lt, W, M, 0.5, level, True)
    w_ref, v_ref = rng.standard_normal(N).astype(np.float32), np.zeros(N, np.float32)
    w_dev, v_dev = H.to_dev(w_ref), H.to_dev(v_ref)
    for s in range(2 * M + 1):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        ob.micro_step_update(grads, w_ref, v_ref, 0.1, 0.9, 1e-4)
        gb.step_all_update([H.to_dev(g) for g in grads], w_dev, v_dev, 0.1, 0.9, 1e-4)
    H.assert_bits_equal(w_dev.cpu().numpy(), w_ref, "batch mode: weights")
    H.assert_bits_equal(v_dev.cpu().numpy(), v_ref, "batch mode: velocity")
    assert gb.batch_status()["exchanges"] == ob.exchanges
    gb.destroy()
