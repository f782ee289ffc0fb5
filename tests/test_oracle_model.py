"""Pins for the oracle's forward pass, loss multipliers, gradient and full epoch.

None of these checks re-types the oracle's own formula: each compares with the
pairwise definition (eq. fm_model), a hand-worked example, a closed form, a
library routine on a special case, or finite differences.
"""
import os

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import fm_oracle as O
from paper_2004_13940_amd.workloads import random_csr

HERE = os.path.dirname(os.path.abspath(__file__))


def _dense_to_matrix(Xd):
    Xs = sp.csr_matrix(Xd)
    Xs.sort_indices()
    return O.make_matrix(Xd.shape[0], Xd.shape[1], Xs.indptr.astype(np.int64), Xs.indices.astype(np.int32), Xs.data)


def _pairwise_score(Xd, w0, w, V):
    """eq. fm_model written out: O(K D^2) double loop over j < j'."""
    N, D = Xd.shape
    out = np.zeros(N)
    for i in range(N):
        f = w0
        for j in range(D):
            f += w[j] * Xd[i, j]
        for j in range(D):
            for jp in range(j + 1, D):
                f += float(np.dot(V[j], V[jp])) * Xd[i, j] * Xd[i, jp]
        out[i] = f
    return out


def test_hand_example_from_golden_file():
    rows = np.loadtxt(os.path.join(HERE, "golden", "fm_score_hand_example.txt"))
    Xd, want = rows[:, :3], rows[:, 3]
    w = np.array([0.1, -0.2, 0.3])
    V = np.array([[1.0, 0.0], [0.5, -1.0], [2.0, 1.0]])
    _, _, _, yhat = O.forward(_dense_to_matrix(Xd), 0.5, w, V)
    np.testing.assert_allclose(yhat, want, rtol=0, atol=1e-14)


@pytest.mark.parametrize("seed,N,D,K,density", [(0, 7, 12, 3, 1.0), (1, 9, 10, 5, 0.4), (2, 5, 8, 1, 0.6)])
def test_rewrite_equals_pairwise_definition(seed, N, D, K, density):
    rng = np.random.default_rng(seed)
    Xd = rng.standard_normal((N, D)) * (rng.random((N, D)) < density)
    w0, w, V = 0.3, rng.standard_normal(D), rng.standard_normal((D, K))
    _, _, _, yhat = O.forward(_dense_to_matrix(Xd), w0, w, V)
    np.testing.assert_allclose(yhat, _pairwise_score(Xd, w0, w, V), rtol=1e-12, atol=1e-12)


def test_all_ones_closed_form_and_two_feature_case():
    rng = np.random.default_rng(3)
    D, K = 9, 4
    w, V = rng.standard_normal(D), rng.standard_normal((D, K))
    _, _, _, yhat = O.forward(_dense_to_matrix(np.ones((2, D))), -0.7, w, V)
    want = -0.7 + w.sum() + 0.5 * (np.sum(V.sum(axis=0) ** 2) - np.sum(V ** 2))
    np.testing.assert_allclose(yhat, [want, want], rtol=1e-13)
    # D=2, K=1: the only pair term is v1 v2 x1 x2
    _, _, _, y2 = O.forward(_dense_to_matrix(np.array([[3.0, -2.0]])), 0.0, np.zeros(2), np.array([[0.5], [4.0]]))
    np.testing.assert_allclose(y2, [0.5 * 4.0 * 3.0 * -2.0], rtol=1e-14)


def test_aggregates_match_library_sparse_products():
    rng = np.random.default_rng(4)
    N, D, K = 40, 30, 6
    rowptr, col, val = random_csr(rng, N, D, 0.06)
    X = O.make_matrix(N, D, rowptr, col, val)
    Xs = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(N, D))
    w, V = rng.standard_normal(D), rng.standard_normal((D, K))
    a, G, q, yhat = O.forward(X, 0.25, w, V)
    np.testing.assert_allclose(a, Xs @ w, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(G, Xs @ V, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(q, Xs.multiply(Xs) @ (V * V).sum(axis=1), rtol=1e-12, atol=1e-13)
    # V = 0 reduces the score to a linear model
    _, G0, q0, y0 = O.forward(X, 0.25, w, np.zeros((D, K)))
    assert not G0.any() and not q0.any()
    np.testing.assert_allclose(y0, 0.25 + Xs @ w, rtol=1e-13, atol=1e-13)
    # rows with nothing stored predict the bias
    empty = np.diff(rowptr) == 0
    assert empty.any()
    np.testing.assert_array_equal(yhat[empty], 0.25)


def test_score_invariant_under_permuting_latent_columns_and_affine_in_one_coordinate():
    rng = np.random.default_rng(5)
    N, D, K = 12, 9, 5
    rowptr, col, val = random_csr(rng, N, D, 0.5)
    X = O.make_matrix(N, D, rowptr, col, val)
    w, V = rng.standard_normal(D), rng.standard_normal((D, K))
    _, _, _, y0 = O.forward(X, 0.1, w, V)
    _, _, _, y1 = O.forward(X, 0.1, w, V[:, rng.permutation(K)])
    np.testing.assert_allclose(y1, y0, rtol=1e-12, atol=1e-12)
    # the score is affine in a single v_jk: second difference vanishes
    Vp, Vm = V.copy(), V.copy()
    Vp[4, 2] += 0.5
    Vm[4, 2] -= 0.5
    _, _, _, yp = O.forward(X, 0.1, w, Vp)
    _, _, _, ym = O.forward(X, 0.1, w, Vm)
    np.testing.assert_allclose(yp + ym - 2 * y0, 0.0, atol=1e-12)


@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_multiplier_is_scaled_derivative_of_loss(loss):
    rng = np.random.default_rng(6)
    yh = rng.standard_normal(50) * 3
    y = np.where(rng.random(50) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(50)
    s, h = 0.37, 1e-6
    _, r = O.loss_multiplier(loss, s, yh, y)
    lp, _ = O.loss_multiplier(loss, s, yh + h, y)
    lm, _ = O.loss_multiplier(loss, s, yh - h, y)
    np.testing.assert_allclose(r, s * (lp - lm) / (2 * h), rtol=1e-6, atol=1e-9)


def test_loss_closed_values_and_extreme_margins():
    y = np.array([1.0, -1.0])
    l, r = O.loss_multiplier(O.LOSS_LOGISTIC, 2.0, np.zeros(2), y)
    np.testing.assert_allclose(l, np.log(2.0), rtol=1e-15)
    np.testing.assert_allclose(r, -2.0 * y / 2.0, rtol=1e-15)
    l, r = O.loss_multiplier(O.LOSS_SQUARED, 2.0, np.zeros(2), np.array([3.0, -0.5]))
    np.testing.assert_allclose(l, [4.5, 0.125], rtol=1e-15)
    np.testing.assert_allclose(r, [-6.0, 1.0], rtol=1e-15)
    m = np.array([-500.0, -50.0, -1.0, 0.0, 1.0, 50.0, 500.0])
    l, r = O.loss_multiplier(O.LOSS_LOGISTIC, 1.0, m, np.ones(7))
    assert np.all(np.isfinite(l)) and np.all(np.isfinite(r))
    assert np.all(np.diff(l) <= 0) and np.all(np.diff(r) >= 0)
    np.testing.assert_allclose(l[:2], [500.0, 50.0], rtol=1e-12)
    np.testing.assert_allclose(r[0], -1.0, rtol=1e-12)
    assert 0 < -r[-1] < 1e-200 and 0 < l[-1] < 1e-200


@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
@pytest.mark.parametrize("s_kind", ["one", "mean"])
def test_gradient_matches_finite_differences_of_objective(loss, s_kind):
    rng = np.random.default_rng(7)
    N, D, K = 25, 11, 3
    rowptr, col, val = random_csr(rng, N, D, 0.35)
    X = O.make_matrix(N, D, rowptr, col, val)
    y = np.where(rng.random(N) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(N)
    s = 1.0 if s_kind == "one" else 1.0 / N
    lw, lv = 0.03, 0.07
    w0, w, V = 0.2, rng.standard_normal(D) * 0.5, rng.standard_normal((D, K)) * 0.5

    def f(w0_, w_, V_):
        return sum(O.objective(loss, s, lw, lv, X, y, w0_, w_, V_))

    a, G, q, yhat = O.forward(X, w0, w, V)
    _, r = O.loss_multiplier(loss, s, yhat, y)
    gw0, gw, gV = O.gradient(X, r, G, w, V, lw, lv)
    h = 1e-6
    np.testing.assert_allclose(gw0, (f(w0 + h, w, V) - f(w0 - h, w, V)) / (2 * h), rtol=2e-6, atol=1e-9)
    for j in range(D):
        e = np.zeros(D)
        e[j] = h
        np.testing.assert_allclose(gw[j], (f(w0, w + e, V) - f(w0, w - e, V)) / (2 * h), rtol=2e-6, atol=1e-9)
        for k in range(K):
            E = np.zeros((D, K))
            E[j, k] = h
            np.testing.assert_allclose(gV[j, k], (f(w0, w, V + E) - f(w0, w, V - E)) / (2 * h),
                                       rtol=2e-6, atol=1e-9)


def test_zero_factors_reduce_to_linear_model_gradient():
    rng = np.random.default_rng(8)
    N, D, K = 60, 20, 4
    rowptr, col, val = random_csr(rng, N, D, 0.2)
    X = O.make_matrix(N, D, rowptr, col, val)
    Xs = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(N, D))
    y = np.where(rng.random(N) < 0.5, 1.0, -1.0)
    w = rng.standard_normal(D)
    V = np.zeros((D, K))
    a, G, q, yhat = O.forward(X, 0.0, w, V)
    _, r = O.loss_multiplier(O.LOSS_LOGISTIC, 1.0, yhat, y)
    gw0, gw, gV = O.gradient(X, r, G, w, V, 0.1, 0.2)
    assert not gV.any()
    # textbook logistic-regression gradient, via the library product
    sig = -y / (1.0 + np.exp(y * (Xs @ w)))
    np.testing.assert_allclose(gw, Xs.T @ sig + 0.1 * w, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(gw0, sig.sum(), rtol=1e-12)
    # V stays at its fixed point
    w0n, wn, Vn, _ = O.full_epoch(X, y, 0.0, w, V, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=0.1, lambda_v=0.2, eta=0.05)
    assert not Vn.any()
    # columns with nothing stored only feel the regulariser
    emptyc = np.diff(X.colptr) == 0
    if emptyc.any():
        np.testing.assert_allclose(gw[emptyc], 0.1 * w[emptyc], rtol=1e-15)


def test_first_logistic_epoch_from_zero_is_closed_form():
    rng = np.random.default_rng(9)
    N, D, K = 50, 15, 3
    rowptr, col, val = random_csr(rng, N, D, 0.3)
    X = O.make_matrix(N, D, rowptr, col, val)
    Xs = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(N, D))
    y = np.where(rng.random(N) < 0.5, 1.0, -1.0)
    eta, s = 0.1, 0.5
    w0n, wn, Vn, obj = O.full_epoch(X, y, 0.0, np.zeros(D), np.zeros((D, K)), loss=O.LOSS_LOGISTIC, s=s,
                                    lambda_w=1e-3, lambda_v=1e-3, eta=eta)
    np.testing.assert_allclose(wn, 0.5 * eta * s * (Xs.T @ y), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(w0n, 0.5 * eta * s * y.sum(), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(obj[0], s * N * np.log(2.0), rtol=1e-13)
    assert obj[1] == 0.0


def test_squared_loss_with_zero_factors_converges_to_ridge_solution():
    rng = np.random.default_rng(10)
    N, D, K = 80, 6, 2
    Xd = rng.standard_normal((N, D))
    X = _dense_to_matrix(Xd)
    y = Xd @ rng.standard_normal(D) + 0.1 * rng.standard_normal(N)
    s, lam = 1.0 / N, 0.05
    w, V, w0 = np.zeros(D), np.zeros((D, K)), 0.0
    H = s * Xd.T @ Xd + lam * np.eye(D)
    eta = 1.0 / np.linalg.eigvalsh(H)[-1]
    for _ in range(600):
        w0, w, V, _ = O.full_epoch(X, y, w0, w, V, loss=O.LOSS_SQUARED, s=s, lambda_w=lam, lambda_v=lam,
                                   eta=eta, update_w0=False)
    np.testing.assert_allclose(w, np.linalg.solve(H, s * Xd.T @ y), rtol=1e-8, atol=1e-10)
    assert w0 == 0.0 and not V.any()


def test_objective_decreases_for_small_step():
    rng = np.random.default_rng(11)
    N, D, K = 60, 25, 4
    rowptr, col, val = random_csr(rng, N, D, 0.25)
    X = O.make_matrix(N, D, rowptr, col, val)
    y = np.where(rng.random(N) < 0.5, 1.0, -1.0)
    w0, w, V = 0.0, np.zeros(D), rng.standard_normal((D, K)) * 0.1
    prev = np.inf
    for _ in range(15):
        w0, w, V, obj = O.full_epoch(X, y, w0, w, V, loss=O.LOSS_LOGISTIC, s=1.0 / N, lambda_w=1e-3,
                                     lambda_v=1e-3, eta=0.2)
        assert sum(obj) < prev
        prev = sum(obj)


def test_evaluate_against_hand_computed_scores():
    """V = 0 makes the score w0 + x.w: four rows whose scores are 1.5, -0.5, 0 and 2 by hand."""
    rowptr = np.array([0, 2, 3, 3, 5], np.int64)
    col = np.array([0, 1, 1, 0, 2], np.int32)
    val = np.array([1.0, 2.0, 1.0, 3.0, 1.0], np.float32)
    X = O.make_matrix(4, 3, rowptr, col, val)
    w = np.array([0.5, 0.5, 0.5])
    V = np.zeros((3, 2))
    # scores: 0 + (0.5 + 1.0) = 1.5 ; 0.5 ; 0 ; 1.5 + 0.5 = 2.0 -> shift by w0 = -1 for row 2: use w0 = 0
    y = np.array([1.0, -1.0, 1.0, -1.0])
    m = O.evaluate(X, y, 0.0, w, V, O.LOSS_SQUARED)
    scores = np.array([1.5, 0.5, 0.0, 2.0])
    assert abs(m["rmse"] - np.sqrt(((scores - y) ** 2).mean())) < 1e-15
    assert abs(m["rmse"] - np.sqrt((0.25 + 2.25 + 1.0 + 9.0) / 4)) < 1e-15
    assert m["accuracy"] == 0.5  # rows 0 and 2 (a score of 0 counts as +1) agree, rows 1 and 3 do not
    assert abs(m["mean_loss"] - 0.5 * (0.25 + 2.25 + 1.0 + 9.0) / 4) < 1e-15
    ml = O.evaluate(X, y, 0.0, w, V, O.LOSS_LOGISTIC)["mean_loss"]
    want = np.mean([np.log1p(np.exp(-1.5)), np.log1p(np.exp(0.5)), np.log(2.0), np.log1p(np.exp(2.0))])
    assert abs(ml - want) < 1e-14


def test_small_dense_workloads_have_the_stated_shapes_and_are_learnable():
    from paper_2004_13940_amd.workloads import make_small
    for name, (N, D) in (("regression_513x8", (513, 8)), ("regression_303x13", (303, 13))):
        tr, te = make_small(name)
        assert (tr.N, tr.D, tr.K) == (N, D, 4) and te.D == D and tr.nnz == N * D
        X, Xt = (O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val) for wl in (tr, te))
        w0, w, V = float(tr.w0), tr.w.astype(np.float64), tr.V.astype(np.float64)
        before = O.evaluate(Xt, te.y, w0, w, V, tr.loss)["rmse"]
        for _ in range(200):
            w0, w, V, _ = O.full_epoch(X, tr.y, w0, w, V, loss=tr.loss, s=tr.loss_scale, lambda_w=tr.lambda_w,
                                       lambda_v=tr.lambda_v, eta=tr.eta)
        after = O.evaluate(Xt, te.y, w0, w, V, tr.loss)["rmse"]
        assert after < 0.8 * before
