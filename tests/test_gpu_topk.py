"""GPU parity: TopK with error feedback against the oracle, bit for bit, through the C ABI."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc
from paper_2010_16248_amd import binding as B
from paper_2010_16248_amd import workloads as wl
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _check_step(gpu, ora, grads, tag, check_state=True):
    """One batched step on both sides; mean and payloads always compared.  check_state=False
    leaves the library's memory alone (reading it writes the residual out, which the batched
    path otherwise defers to the next step's first pass): the deferred route is then the one
    the next step takes.  Returns the mean."""
    out_ref = ora.step(grads)
    dg = [H.to_dev(g) for g in grads]
    out = H.dev_out(gpu.n_params)
    gpu.step_all(dg, out)
    mean = out.cpu().numpy()
    H.assert_bits_equal(mean, out_ref, f"{tag}: mean")
    for w in range(gpu.n_workers):
        for li in range(gpu.n_layers):
            idx, val = gpu.get_payload(w, li)
            ri, rv = ora.payload[(w, li)]
            assert np.array_equal(idx, ri), f"{tag}: indices worker {w} layer {li}"
            H.assert_bits_equal(val, rv, f"{tag}: values worker {w} layer {li}")
    assert gpu.payload_words() == (ora.words_last, ora.words_cum)
    if not check_state:
        return mean
    st = gpu.unpack_state(gpu.get_state())
    H.assert_bits_equal(st["e"], ora.e, f"{tag}: residual")
    H.assert_bits_equal(st["A"], ora.A, f"{tag}: accumulator")
    return mean


def _case_values(rng, case, n):
    if case == "normal":
        return rng.standard_normal(n)
    if case == "quantised":
        return rng.integers(-3, 4, n) * 0.25
    if case == "all_equal":
        return np.full(n, -1.5)
    if case == "all_zero":
        return np.zeros(n)
    if case == "sparse":
        return rng.standard_normal(n) * (rng.random(n) < 0.05)
    raise KeyError(case)


@pytest.mark.parametrize("W", [1, 3])
def test_kept_entries_concentrated_in_a_few_quarters(W):
    """K = 25 % and 45 % of layers whose large entries sit in one stretch: whole wave quarters
    are kept, so a wave's list of payload entries fills up inside a chunk of groups and is
    written out early, while other quarters keep nothing.  Aligned and misaligned layers, the
    stretch at a different place for every worker."""
    print(f"case concentrated W={W}", flush=True)
    shapes = [(1, 5 * 8192, 0), (1, 3, 0), (3, 8192 + 1001, 1), (1, 2 * 8192 + 6, 0)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 45, 25)
    rng = np.random.default_rng(77 + W)
    for step in range(4):
        if step == 2:
            ora.level[:] = 0
            gpu.set_state(H.oracle_state_blob(gpu, ora))
        grads = []
        for w in range(W):
            g = rng.standard_normal(N) * 1e-3
            for l in layers:
                n = l.numel
                lo = (n // 7) * ((w + step) % 5)
                hi = min(n, lo + int(n * 0.4))
                g[l.offset + lo:l.offset + hi] += np.sign(rng.standard_normal(hi - lo)) * (1.0 + rng.random(hi - lo))
            grads.append(g.astype(np.float32))
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step % 2 == 1))
    gpu.destroy()


@pytest.mark.parametrize("crit,noncrit,den", [(10, 1, 100), (1, 1, 1), (1, 3, 1000), (99, 25, 100)])
def test_ragged_misaligned_layers(crit, noncrit, den):
    """Many small layers at 16-byte-misaligned offsets, W = 3, several steps so that the
    memory feeds back; K from 0.1 % to 100 %."""
    print(f"case ragged crit={crit} noncrit={noncrit} den={den}", flush=True)
    layers = wl.random_layers(seed=11, n_layers=23, max_rows=40, max_cols=300)
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, 3, crit, noncrit, den)
    rng = np.random.default_rng(1)
    for step in range(3):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(3)]
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step == 2))
    # switch every layer to the other level by hand and go on
    blob = H.oracle_state_blob(gpu, ora)
    ora.level[:] = 0
    st = gpu.unpack_state(blob)
    st["level"][:] = 0
    gpu.set_state(blob)
    for step in range(2):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(3)]
        _check_step(gpu, ora, grads, f"noncrit step {step}", check_state=(step == 1))
    gpu.destroy()


@pytest.mark.parametrize("case", ["normal", "quantised", "all_equal", "all_zero", "sparse"])
def test_multi_tile_layers_with_ties(case):
    """Layers that span several 8192-element tiles with ragged tails; value sets with heavy
    ties (the lower index must win) including a tie class far larger than the candidate
    list, which takes the re-read path."""
    print(f"case multi-tile {case}", flush=True)
    shapes = [(1, 3 * 8192 + 77, 0), (37, 1001, 1), (1, 5, 0), (3, 8192, 1), (1, 70001, 0)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, 2, 10, 1)
    rng = np.random.default_rng([7, len(case)])
    for step in range(4):                                    # state read after steps 1 and 3 only
        grads = [_case_values(rng, case, N).astype(np.float32) for _ in range(2)]
        _check_step(gpu, ora, grads, f"{case} step {step}", check_state=(step % 2 == 1))
    gpu.destroy()


@pytest.mark.parametrize("W", [2, 3, 4, 8])
def test_mean_of_subnormal_values_rounds_like_a_division(W):
    """Kept values so small that their mean is subnormal: the mean must round exactly like the
    oracle's division by W (for W a power of two the kernel multiplies by 1 / W, which is the same
    real number), over several steps so that subnormal residuals feed back as well."""
    print(f"case subnormal mean W={W}", flush=True)
    layers = wl.make_layers([(1, 2 * 8192 + 31, 0), (9, 333, 1)])
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 50, 10)
    rng = np.random.default_rng([13, W])
    tiny = np.float32(1.4e-45)
    for step in range(3):
        grads = [(rng.integers(-40, 41, N).astype(np.float32) * tiny) for _ in range(W)]
        assert all(np.all(np.abs(g) < 1.2e-38) for g in grads)
        _check_step(gpu, ora, grads, f"subnormal W={W} step {step}", check_state=(step == 2))
    gpu.destroy()


def test_guessed_bins_hit_drift_and_miss():
    """The error-feedback pass lists its candidates on a guess of where the threshold will lie.
    Over many steps with a stationary distribution the guess must hit (nothing is staged again, the
    compaction works from the lists); a slow drift of the gradient scale is followed by the
    extrapolated guess; a jump makes it miss (the layer is staged again and compacted from Delta).
    Every step is bit-exact whichever route is taken -- against the oracle, and word for word
    against a second context that is driven call by call, where the compaction always reads
    Delta and the mean is formed from the payloads."""
    print("case guessed bins", flush=True)
    shapes = [(1, 5 * 8192 + 13, 0), (64, 577, 1), (1, 100, 0), (6, 8192, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    twin, _ = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    out_twin = H.dev_out(N)
    rng = np.random.default_rng(5)
    scale = 1.0
    restaged = []
    for step in range(14):
        if 6 <= step < 10:
            scale *= 1.09                                   # one level-1 bin per step, about
        if step == 12:
            scale *= 40.0                                   # far outside the guessed bins
        grads = [(rng.standard_normal(N) * scale).astype(np.float32) for _ in range(W)]
        mean = _check_step(gpu, ora, grads, f"step {step}", check_state=(step % 3 == 2 or step == 13))
        restaged.append(gpu.topk_stats()[0])
        dg = [H.to_dev(g) for g in grads]
        for w in range(W):
            twin.compress_step(w, dg[w], 0)
        twin.aggregate(0)
        twin.decompress(out_twin)
        H.assert_bits_equal(out_twin.cpu().numpy(), mean, f"step {step}: the two routes differ in the mean")
        for w in range(W):
            for li in range(gpu.n_layers):
                ia, va = gpu.get_payload(w, li)
                ib, vb = twin.get_payload(w, li)
                assert np.array_equal(ia, ib), f"step {step}: the two routes differ in the indices"
                H.assert_bits_equal(va, vb, f"step {step}: the two routes differ in the values")
    per_step = np.diff([0] + restaged)
    n_multi = 3 * W                                         # (worker, layer) pairs of more than one tile
    assert per_step[0] == n_multi                           # nothing to guess from at the first step
    assert per_step[3:6].sum() == 0, per_step               # stationary: the guess holds
    assert per_step[12] == n_multi, per_step                # the jump is missed ...
    assert per_step[13] <= n_multi                          # ... and everything is still exact
    assert gpu.topk_stats()[1] == 0                         # no tie class needed the sweeps
    twin.destroy()
    gpu.destroy()


def test_a_level_switch_finds_its_bins_guessed_from_the_other_level():
    """While a level runs, the bins of the other level's threshold are taken from the same
    histogram, so the first step after a switch needs no second staging on a stationary
    distribution (its own history at that level is missing or stale); results stay bit-exact."""
    print("case level switch guess", flush=True)
    shapes = [(1, 5 * 8192 + 13, 0), (64, 577, 1), (1, 100, 0), (6, 8192, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    rng = np.random.default_rng(15)
    restaged = []
    for step in range(12):
        if step in (2, 4, 8):                               # windows of 2, 2 and 4 steps
            # no history: critical (K 10 % stays); stationary norms: non-critical (K 1 % from step
            # 4); a learning-rate decay: critical (K 10 % again from step 8)
            lr_next = 0.01 if step == 8 else 0.1
            ref = ora.detect_regime(0.1, lr_next)
            gpu.detect_regime(0.1, lr_next)
            assert np.array_equal(gpu.get_levels(), ref)
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step % 4 == 3))
        restaged.append(gpu.topk_stats()[0])
    per_step = np.diff([0] + restaged)
    assert per_step[0] == 3 * W                             # nothing to guess from at the very first step
    assert ora.level[0] == 1 and ora.words_cum > 0
    assert per_step[4] == 0 and per_step[8] == 0, per_step  # the first steps at a new level
    gpu.destroy()


def test_threshold_among_exact_zeros_is_guessed_too():
    """Sparse gradients of which more is kept than is non-zero (the embedding of a language
    model): the threshold is zero.  After the first step the error-feedback pass stages bin 0
    itself (non-zero keys listed, zeros counted), so nothing is re-staged; a dense step in
    between is a miss and everything stays exact."""
    print("case zero-bin guess", flush=True)
    shapes = [(1, 5 * 8192 + 13, 0), (64, 577, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    rng = np.random.default_rng(15)
    restaged = []
    for step in range(7):
        dense = step == 4
        grads = []
        for _ in range(W):
            g = rng.standard_normal(N)
            if not dense:
                g *= rng.random(N) < 0.03                   # 3 % non-zero, 10 % kept
            grads.append(g.astype(np.float32))
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step in (3, 6)))
        restaged.append(gpu.topk_stats()[0])
    per_step = np.diff([0] + restaged)
    n_multi = 2 * W
    assert per_step[0] == n_multi                           # nothing to guess from
    assert per_step[1:4].sum() == 0, per_step               # bin 0 guessed and found
    assert per_step[4] == n_multi, per_step                 # the dense step misses
    assert per_step[6] == 0, per_step
    gpu.destroy()


def test_zero_threshold_with_dense_rows_and_kept_zeros():
    """An embedding-like layer: a few rows are dense, the rest exactly zero, and more is kept than is
    non-zero.  Once bin 0 is guessed the first pass lists every non-zero entry; the quarters of
    the dense rows overflow their lists, the first quarters of the layer keep exact zeros (which
    no list holds), and both are taken from Delta quarter by quarter and worker by worker while
    the others are served by the lists.  Every step is exact, payload order included."""
    print("case zero threshold, dense rows", flush=True)
    rows, cols = 96, 672                                    # 8 tiles
    shapes = [(rows, cols, 1), (1, 3 * 8192 + 77, 0)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 3
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    rng = np.random.default_rng(31)
    restaged = []
    for step in range(5):
        grads = []
        for w in range(W):
            g = np.zeros(N, np.float32)
            m = np.zeros((rows, cols), np.float32)
            lo = 88 - 3 * w - (step % 2)                    # six dense rows, elsewhere per worker and step
            m[lo:lo + 6] = rng.standard_normal((6, cols))
            g[:rows * cols] = m.reshape(-1)
            v = rng.standard_normal(N - rows * cols) * (rng.random(N - rows * cols) < 0.02)
            g[rows * cols:] = v
            grads.append(g)
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step in (2, 4)))
        restaged.append(gpu.topk_stats()[0])
    per_step = np.diff([0] + restaged)
    assert per_step[2:].sum() == 0, per_step                # bin 0 guessed and found
    gpu.destroy()


def test_a_sparse_layer_running_dry_is_seen_coming():
    """A sparse gradient (3 % non-zero) whose memory has filled up while little was kept: the first
    step that keeps 10 % again finds more than 10 % non-zero entries (threshold above zero) and
    empties the memory to below that, so from the second step on the threshold is zero.  The step
    that decides the first sees it coming (what it leaves behind plus what a gradient brought in
    when everything non-zero was kept last time is less than k) and guesses bin 0 for the second:
    nothing is staged twice there; every step is exact."""
    print("case sparse layer runs dry", flush=True)
    shapes = [(1, 6 * 8192 + 5, 0), (40, 1031, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    rng = np.random.default_rng(23)
    restaged = []
    for step in range(12):
        if step in (2, 4, 10):
            # no history: critical (K 10 % stays); stationary norms: K 1 % from step 4; a
            # learning-rate decay: K 10 % again from step 10
            lr_next = 0.01 if step == 10 else 0.1
            ref = ora.detect_regime(0.1, lr_next)
            gpu.detect_regime(0.1, lr_next)
            assert np.array_equal(gpu.get_levels(), ref)
        grads = [(rng.standard_normal(N) * (rng.random(N) < 0.03)).astype(np.float32) for _ in range(W)]
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step in (5, 11)))
        restaged.append(gpu.topk_stats()[0])
    per_step = np.diff([0] + restaged)
    assert list(ora.level) == [1, 1]
    assert per_step[1:4].sum() == 0, per_step               # threshold zero, guessed
    assert per_step[10] == 0, per_step                      # back at K 10 %: more than 10 % non-zero by now
    assert per_step[11] == 0, per_step                      # and dry again, seen coming
    gpu.destroy()



def test_large_tie_classes_take_the_sweeps_and_stay_exact():
    """Quantised values in layers of several tiles: the tie class of the threshold is far larger
    than the per-quarter key lists, for several steps in a row.  While the threshold jumps from
    one quantised value to another the guess misses (the layer is then decided from re-staged
    keys, which is not counted as a tie sweep); once it rests the guess holds, the lists overflow
    and the sweeps take over."""
    print("case tie sweeps", flush=True)
    shapes = [(1, 4 * 8192 + 5, 0), (3, 9000, 1)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, 2, 10, 1)
    rng = np.random.default_rng(9)
    for step in range(9):
        grads = [(rng.integers(-3, 4, N) * 0.25).astype(np.float32) for _ in range(2)]
        _check_step(gpu, ora, grads, f"step {step}", check_state=(step in (1, 3, 8)))
    restaged, swept = gpu.topk_stats()
    assert restaged > 0 and swept > 0, (restaged, swept)
    gpu.destroy()


@pytest.mark.parametrize("n_tiles,k", [(225, 5000), (800, 20000), (3100, 70000)])
def test_more_keys_around_the_threshold_than_the_pick_kernel_holds_in_lds(n_tiles, k):
    """Twelve keys per wave quarter (2048 elements) lie in one level-2 cell of the key space
    (16384 consecutive key values, so with many ties) and the threshold falls among them: every
    quarter's list is complete, but the layer's lists together exceed what the last pick kernel
    gathers in LDS (225 tiles: 10800 keys; 800 tiles: 38400 keys, the larger instantiation of the
    kernel; 3100 tiles: 148800 keys and more quarters than even that one counts in LDS), so it
    works from the lists in device memory.  Second step: no new gradient, the threshold stays in
    the cell with fewer keys left."""
    print(f"case long lists n_tiles={n_tiles} k={k}", flush=True)
    n = n_tiles * 8192
    layers = wl.make_layers([(1, n, 0)])
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, 1, k, k, n)
    rng = np.random.default_rng([21, n_tiles])
    g = rng.random(n).astype(np.float32) * np.float32(0.9)            # all below the cell
    cell = np.uint32(0x3FC00000)                                      # 1.5f: the low 14 key bits are free
    for q in range(4 * n_tiles):
        pos = q * 2048 + rng.choice(2048, 12, replace=False)
        g[pos] = (cell | rng.integers(0, 1 << 14, 12).astype(np.uint32)).view(np.float32)
    g *= rng.choice(np.array([-1.0, 1.0], np.float32), n)
    _check_step(gpu, ora, [g], "step 0", check_state=False)
    _check_step(gpu, ora, [np.zeros(n, np.float32)], "step 1")
    assert gpu.topk_stats()[1] == 0                                   # no list overflowed: no sweeps
    gpu.destroy()


@pytest.mark.parametrize("crit,noncrit", [(99, 60), (100, 51)])
def test_high_keep_ratios_use_the_values_and_holes_layout(crit, noncrit):
    """The paper's own K = 99 % level: layers that keep more than half store values in index
    order plus the indices of the dropped entries.  Batched and call-by-call paths, layers of
    several tiles at misaligned offsets, heavy ties; the decoded payload, the mean, the residual
    and the layout rule itself are compared with the oracle."""
    print(f"case hole layout {crit}/{noncrit}", flush=True)
    shapes = [(1, 3 * 8192 + 77, 0), (37, 1001, 1), (1, 5, 0), (3, 8192, 1), (1, 1, 0), (1, 2, 0)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 2
    rng = np.random.default_rng([crit, noncrit])
    for mode in ("all", "calls"):
        gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, crit, noncrit)
        for li, l in enumerate(layers):
            for level, num in ((1, crit), (0, noncrit)):
                fmt, kept, words = B.payload_format(gpu.cfg, li, level)
                k = orc.k_from_fraction(l.numel, num, 100)
                assert kept == k and words == orc.payload_words_packed(l.numel, k)
                assert fmt == (B.ACC_PAYLOAD_VALUES_HOLES if 2 * k > l.numel else B.ACC_PAYLOAD_INDEX_VALUE)
        for step in range(4):
            if step == 2:
                ora.level[:] = 0
                gpu.set_state(H.oracle_state_blob(gpu, ora))
            if step % 2:
                grads = [(rng.integers(-3, 4, N) * 0.25).astype(np.float32) for _ in range(W)]
            else:
                grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
            if mode == "all":
                _check_step(gpu, ora, grads, f"{mode} step {step}", check_state=(step in (1, 3)))
            else:
                out_ref = ora.step(grads)
                dg = [H.to_dev(g) for g in grads]
                out = H.dev_out(N)
                for w in range(W):
                    gpu.compress_step(w, dg[w], 0)
                gpu.aggregate(0)
                gpu.decompress(out)
                H.assert_bits_equal(out.cpu().numpy(), out_ref, f"{mode} step {step}: mean")
                for w in range(W):
                    for li in range(gpu.n_layers):
                        idx, val = gpu.get_payload(w, li)
                        assert np.array_equal(idx, ora.payload[(w, li)][0])
                        H.assert_bits_equal(val, ora.payload[(w, li)][1], "values")
                st = gpu.unpack_state(gpu.get_state())
                H.assert_bits_equal(st["e"], ora.e, f"{mode} step {step}: residual")
        gpu.destroy()


@pytest.mark.parametrize("crit", [10, 99])
def test_support_overlap_matches_the_oracle(crit):
    """Per-layer overlap of the kept coordinates of pairs of workers (Section 4.3), for (index,
    value) payloads (K 10 %) and for values + holes payloads (K 99 %); gradients built as a
    common sparse mean plus dense noise, plus one pure-noise worker."""
    print(f"case overlap K={crit}", flush=True)
    shapes = [(1, 3 * 8192 + 77, 0), (37, 1001, 1), (1, 5, 0), (3, 8192, 1), (1, 1, 0)]
    layers = wl.make_layers(shapes)
    N = wl.total_params(layers)
    W = 3
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, crit, 1)
    with pytest.raises(B.AccordionError) as ei:
        gpu.topk_overlap(0, 1)                               # no payloads yet
    assert ei.value.status == B.ACC_ESTATE
    rng = np.random.default_rng(crit)
    mean = np.zeros(N)
    hot = rng.choice(N, N // 10, replace=False)
    mean[hot] = rng.choice([-1.0, 1.0], hot.size) * 5.0
    for step in range(2):
        grads = [(mean + 0.3 * rng.standard_normal(N)).astype(np.float32) for _ in range(2)]
        grads.append(rng.standard_normal(N).astype(np.float32))
        _check_step(gpu, ora, grads, f"step {step}")
        for a, b in ((0, 1), (1, 2), (2, 0), (1, 1)):
            common, kept = gpu.topk_overlap(a, b)
            for li, l in enumerate(layers):
                assert kept[li] == ora.layer_k(li)
                ref = orc.support_overlap(ora.payload[(a, li)][0], ora.payload[(b, li)][0])
                assert common[li] == ref, (step, a, b, li, common[li], ref)
        common, kept = gpu.topk_overlap(0, 1)
        if crit == 10 and step == 0:
            assert common.sum() > 0.9 * kept.sum()           # the paper's "> 90 %" under its model
    with pytest.raises(B.AccordionError):
        gpu.topk_overlap(0, 3)
    gpu.destroy()


def test_call_by_call_equals_step_all_and_is_deterministic():
    layers = wl.make_layers([(20, 900, 1), (1, 64, 0), (9, 9, 1)])
    N = wl.total_params(layers)
    W = 3
    rng = np.random.default_rng(3)
    grads = [[rng.standard_normal(N).astype(np.float32) for _ in range(W)] for _ in range(2)]
    results = []
    for mode in ("all", "calls", "all"):
        gpu, _ = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
        outs = []
        for step in range(2):
            dg = [H.to_dev(g) for g in grads[step]]
            out = H.dev_out(N)
            if mode == "all":
                gpu.step_all(dg, out)
            else:
                for w in (2, 0, 1):                      # any worker order
                    gpu.compress_step(w, dg[w], 0)
                gpu.aggregate(0)
                gpu.decompress(out)
            outs.append(out.cpu().numpy())
        results.append((outs, gpu.get_state().copy()))
        gpu.destroy()
    for outs, st in results[1:]:
        for a, b in zip(outs, results[0][0]):
            H.assert_bits_equal(a, b, "mean")
        assert np.array_equal(st, results[0][1])


def test_batched_and_call_by_call_steps_interleave():
    """The batched path leaves the residual to the next step's first pass; the call-by-call
    path writes it itself.  Any interleaving of the two, with workers compressed in any order,
    gives the oracle's payloads, means and (read once at the end) memory."""
    print("case mixed paths", flush=True)
    layers = wl.make_layers([(1, 2 * 8192 + 31, 0), (20, 900, 1), (1, 64, 0)])
    N = wl.total_params(layers)
    W = 3
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    rng = np.random.default_rng(21)
    out = H.dev_out(N)
    for step, mode in enumerate(["all", "calls", "all", "all", "calls", "calls", "all"]):
        if step % 2:
            grads = [(rng.integers(-3, 4, N) * 0.25).astype(np.float32) for _ in range(W)]
        else:
            grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        if mode == "all":
            _check_step(gpu, ora, grads, f"step {step} {mode}", check_state=False)
            continue
        out_ref = ora.step(grads)
        dg = [H.to_dev(g) for g in grads]
        for w in (1, 2, 0):
            gpu.compress_step(w, dg[w], 0)
        gpu.aggregate(0)
        gpu.decompress(out)
        H.assert_bits_equal(out.cpu().numpy(), out_ref, f"step {step} {mode}: mean")
        for w in range(W):
            for li in range(gpu.n_layers):
                idx, val = gpu.get_payload(w, li)
                assert np.array_equal(idx, ora.payload[(w, li)][0]), f"step {step}: indices"
                H.assert_bits_equal(val, ora.payload[(w, li)][1], f"step {step}: values")
    st = gpu.unpack_state(gpu.get_state())
    H.assert_bits_equal(st["e"], ora.e, "residual at the end")
    H.assert_bits_equal(st["A"], ora.A, "accumulator at the end")
    gpu.flush()                                             # nothing pending any more: a no-op
    assert np.array_equal(gpu.get_state(), gpu.pack_state(st["e"], st["A"], None, st["norm_old"],
                                                          st["has_old"], st["level"]))
    gpu.destroy()


def test_set_state_overrides_a_pending_residual():
    """Importing a state while the residual of the last batched step is still pending must take
    the imported memory as it is (nothing of the old step may be dropped from it)."""
    layers = wl.make_layers([(1, 8192 + 77, 0), (12, 50, 1)])
    N = wl.total_params(layers)
    W = 2
    gpu, ora = H.make_pair(B.ACC_TOPK, layers, W, 10, 1)
    rng = np.random.default_rng(33)
    for step in range(2):                                   # the second step leaves its residual pending
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        _check_step(gpu, ora, grads, f"step {step}", check_state=False)
    ora.e[:] = rng.standard_normal((W, N)).astype(np.float32)   # a memory from elsewhere
    ora.A[:] = 0
    gpu.set_state(H.oracle_state_blob(gpu, ora))
    for step in range(2):
        grads = [rng.standard_normal(N).astype(np.float32) for _ in range(W)]
        _check_step(gpu, ora, grads, f"after import, step {step}", check_state=(step == 1))
    gpu.destroy()


def test_state_machine_errors_come_from_the_host():
    layers = wl.make_layers([(4, 10, 1)])
    gpu, _ = H.make_pair(B.ACC_TOPK, layers, 2, 50, 10)
    g = H.to_dev(np.ones(40, np.float32))
    out = H.dev_out(40)
    with pytest.raises(B.AccordionError) as ei:
        gpu.aggregate(0)
    assert ei.value.status == B.ACC_ESTATE
    with pytest.raises(B.AccordionError):
        gpu.decompress(out)
    gpu.compress_step(0, g, 0)
    with pytest.raises(B.AccordionError) as ei:
        gpu.compress_step(0, g, 0)                       # same worker twice
    assert ei.value.status == B.ACC_ESTATE
    with pytest.raises(B.AccordionError) as ei:
        gpu.compress_step(2, g, 0)                       # worker out of range
    assert ei.value.status == B.ACC_EINVAL
    with pytest.raises(B.AccordionError) as ei:
        gpu.compress_step(1, g, 1)                       # TopK has no phase 1
    assert ei.value.status == B.ACC_EINVAL
    with pytest.raises(B.AccordionError) as ei:
        gpu.detect_regime(0.1, 0.1)                      # inside a step
    assert ei.value.status == B.ACC_ESTATE
    with pytest.raises(B.AccordionError):
        gpu.aggregate(0)                                 # worker 1 missing
    gpu.compress_step(1, g, 0)
    gpu.aggregate(0)
    gpu.decompress(out)
    assert np.all(out.cpu().numpy()[:20] == 1.0)         # k = 20 of 40 equal entries: first 20
    assert np.all(out.cpu().numpy()[20:] == 0.0)
    gpu.destroy()
