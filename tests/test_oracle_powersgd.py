"""Pins for the oracle's PowerSGD round (CPU only): library QR / SVD on tiny
matrices, exact-rank recovery, convergence to the truncated SVD, linearity over
workers and the error-feedback identity."""
import numpy as np
import pytest

from oracle import accordion_oracle as orc


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


@pytest.mark.parametrize("n,r", [(5, 1), (9, 2), (16, 4), (24, 3)])
def test_gram_schmidt_is_thin_qr_with_positive_diagonal(n, r):
    rng = np.random.default_rng([n, r])
    p = _rand(rng, n, r)
    q_lib, r_lib = np.linalg.qr(p.astype(np.float64))
    q_lib = q_lib * np.sign(np.diag(r_lib))           # make diag(R) positive
    got = orc.gram_schmidt(p)
    assert np.allclose(got, q_lib, atol=2e-6)
    assert np.allclose(got.T.astype(np.float64) @ got, np.eye(r), atol=1e-6)


def test_gram_schmidt_zero_column_stays_zero():
    p = np.array([[1, 2, 0], [0, 4, 0], [0, 6, 0]], np.float32)
    got = orc.gram_schmidt(p)
    assert np.all(got[:, 2] == 0)
    got = orc.gram_schmidt(np.array([[0, 1], [0, 0]], np.float32))
    assert got[:, 0].tolist() == [0, 0] and got[:, 1].tolist() == [1, 0]


@pytest.mark.parametrize("n,m,r", [(6, 11, 1), (16, 24, 2), (12, 7, 4), (3, 20, 3)])
def test_single_worker_is_projection_onto_span_of_MQ(n, m, r):
    rng = np.random.default_rng([n, m, r])
    M, Q = _rand(rng, n, m), _rand(rng, m, r)
    p_hat, q_bar, D = orc.powersgd_layer([M], Q)
    qf, _ = np.linalg.qr(M.astype(np.float64) @ Q.astype(np.float64))
    ref = qf @ (qf.T @ M.astype(np.float64))
    assert np.allclose(D, ref, atol=1e-5 * np.abs(ref).max())
    assert p_hat.shape == (n, r) and q_bar.shape == (m, r)
    # Q_bar = M^T P_hat  (a transposed operand would not even have this shape)
    assert np.allclose(q_bar, M.astype(np.float64).T @ p_hat.astype(np.float64), atol=1e-5)


def test_exact_rank_r_matrix_is_recovered():
    rng = np.random.default_rng(11)
    for r in (1, 2, 4):
        M = (_rand(rng, 14, r).astype(np.float64) @ _rand(rng, r, 22).astype(np.float64)).astype(np.float32)
        _, _, D = orc.powersgd_layer([M], _rand(rng, 22, r))
        assert np.allclose(D, M, atol=2e-5 * np.abs(M).max())


def test_iteration_converges_to_truncated_svd():
    rng = np.random.default_rng(12)
    n, m, r = 16, 24, 2
    U, _ = np.linalg.qr(rng.standard_normal((n, n)))
    V, _ = np.linalg.qr(rng.standard_normal((m, m)))
    s = np.array([10, 5, 1, .5, .2] + [0.05] * (n - 5))
    M = ((U * s) @ V[:, :n].T).astype(np.float32)
    Q = _rand(rng, m, r)
    for _ in range(50):
        _, Q, D = orc.powersgd_layer([M], Q)
    u, sv, vt = np.linalg.svd(M.astype(np.float64), full_matrices=False)
    best = (u[:, :r] * sv[:r]) @ vt[:r]
    assert np.allclose(D, best, atol=1e-4)
    assert np.allclose(np.linalg.svd(Q.astype(np.float64), compute_uv=False), sv[:r], rtol=1e-4)


def test_linearity_over_workers():
    rng = np.random.default_rng(13)
    n, m, r, W = 10, 18, 2, 4
    Ms = [_rand(rng, n, m) for _ in range(W)]
    Q = _rand(rng, m, r)
    _, _, D_w = orc.powersgd_layer(Ms, Q)
    mean = (sum(x.astype(np.float64) for x in Ms) / W)
    _, _, D_1 = orc.powersgd_layer([mean.astype(np.float32)], Q)
    assert np.allclose(D_w, D_1, atol=1e-5)


def test_state_machine_error_feedback_identity_and_vectors():
    rng = np.random.default_rng(14)
    layers = [(0, 6, 9, 1), (54, 1, 5, 0), (59, 4, 3, 1)]
    N, W, rmax = 71, 3, 2
    q0 = _rand(rng, 9 * rmax + 3 * rmax)
    o = orc.AccordionOracle(orc.POWERSGD, layers, W, 2, 1, 100, 0.5, 1, q0)
    e_prev = np.zeros((W, N), np.float32)
    g_sum0 = np.zeros(N, np.float32)
    for step in range(3):
        grads = [_rand(rng, N) for _ in range(W)]
        q_before = {li: q.copy() for li, q in o.Q.items()}
        D = o.step(grads)
        g_sum0 = g_sum0 + grads[0]
        for w in range(W):
            delta = grads[w] + e_prev[w]
            # compressed + residual = gradient + old residual on matrix layers
            for (off, r, c, is_m) in layers:
                sl = slice(off, off + r * c)
                if is_m:
                    ulp = np.spacing(np.maximum(np.abs(delta[sl]), np.abs(D[sl])))
                    assert np.all(np.abs((D[sl].astype(np.float64) + o.e[w, sl]) - delta[sl]) <= ulp)
                else:
                    assert np.all(o.e[w, sl] == 0)           # no memory on 1-D tensors
        # the vector layer is the plain mean of the raw gradients
        assert np.allclose(D[54:59], sum(g[54:59].astype(np.float64) for g in grads) / W, rtol=1e-6)
        # mean residual = mean delta - D
        mean_delta = sum((grads[w] + e_prev[w]).astype(np.float64) for w in range(W)) / W
        assert np.allclose(o.e.astype(np.float64).mean(0)[:54], mean_delta[:54] - D[:54], atol=1e-6)
        # layer 0 equals the standalone round on the same inputs
        d0 = [(grads[w] + e_prev[w])[:54].reshape(6, 9) for w in range(W)]
        _, qb, Dl = orc.powersgd_layer(d0, q_before[0][:, :2])
        assert np.array_equal(Dl.reshape(-1), D[:54]) and np.array_equal(qb, o.Q[0][:, :2])
        e_prev = o.e.copy()
        assert o.words_last == 2 * (6 + 9) + 5 + 2 * (4 + 3)
    assert np.array_equal(o.A, g_sum0)


def test_rank_switch_keeps_unused_columns():
    rng = np.random.default_rng(15)
    layers = [(0, 8, 12, 1)]
    q0 = _rand(rng, 12 * 2)
    o = orc.AccordionOracle(orc.POWERSGD, layers, 1, 2, 1, 100, 0.5, 0, q0)   # start non-critical: rank 1
    o.step([_rand(rng, 96)])
    assert np.array_equal(o.Q[0][:, 1], q0.reshape(12, 2)[:, 1])              # column 1 untouched
    assert not np.array_equal(o.Q[0][:, 0], q0.reshape(12, 2)[:, 0])
    assert o.P_hat[0].shape == (8, 1)
    o.level[0] = 1
    o.step([_rand(rng, 96)])
    assert o.P_hat[0].shape == (8, 2)


def test_rank_capped_by_shape():
    assert orc.effective_rank(4, 3, 20) == 3
    assert orc.effective_rank(4, 10, 512) == 4
    assert orc.effective_rank(2, 64, 1) == 1
