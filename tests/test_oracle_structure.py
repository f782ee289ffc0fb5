"""Pins for the oracle's integer structures (transpose, partition, per-stratum
matrices) and for its stratified epoch."""
import ctypes

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import fm_oracle as O
from paper_2004_13940_amd.workloads import random_csr


def _rand_problem(seed, N, D, K, density, loss=O.LOSS_LOGISTIC):
    rng = np.random.default_rng(seed)
    rowptr, col, val = random_csr(rng, N, D, density)
    X = O.make_matrix(N, D, rowptr, col, val)
    Xs = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(N, D))
    y = np.where(rng.random(N) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(N)
    w = rng.standard_normal(D) * 0.1
    V = rng.standard_normal((D, K)) * 0.1
    return rng, X, Xs, y, w, V


def test_transpose_matches_dense_and_round_trips():
    rng = np.random.default_rng(0)
    N, D = 23, 17
    rowptr, col, val = random_csr(rng, N, D, 0.3)
    Xd = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(N, D)).toarray()
    colptr, row, cval = O.csr_to_csc(N, D, rowptr, col, val)
    # brute force: walk the dense transpose
    want_row, want_val, want_ptr = [], [], [0]
    for j in range(D):
        for i in range(N):
            if Xd[i, j] != 0.0:
                want_row.append(i)
                want_val.append(Xd[i, j])
        want_ptr.append(len(want_row))
    np.testing.assert_array_equal(colptr, want_ptr)
    np.testing.assert_array_equal(row, want_row)
    np.testing.assert_array_equal(cval, want_val)
    # transposing twice gives the input back
    rp2, c2, v2 = O.csr_to_csc(D, N, colptr, row, cval)
    np.testing.assert_array_equal(rp2, rowptr)
    np.testing.assert_array_equal(c2, col)
    np.testing.assert_array_equal(v2, val.astype(np.float64))
    # rows ascend strictly inside every column
    for j in range(D):
        assert np.all(np.diff(row[colptr[j]:colptr[j + 1]]) > 0)


@pytest.mark.parametrize("n,P", [(10, 3), (7, 7), (5, 8), (1000, 64), (1, 1), (20_000_000, 128)])
def test_block_bounds_floor_split(n, P):
    b = O.block_bounds(n, P)
    assert b[0] == 0 and b[-1] == n and np.all(np.diff(b) >= 0)
    for k in range(P + 1):
        assert int(b[k]) == (k * n) // P  # python integers: exact at any size
    assert np.diff(b).max() - np.diff(b).min() <= 1


def test_block_bounds_do_not_overflow_64_bits():
    n, P = (1 << 62) + 12345, 1000
    lib = O._L()
    for k in (1, 499, 999, 1000):
        assert lib.oracle_block_bound(ctypes.c_int64(n), ctypes.c_int64(P), ctypes.c_int64(k)) == (k * n) // P


@pytest.mark.parametrize("N,D,P", [(30, 20, 4), (17, 9, 5), (6, 3, 8), (12, 12, 1)])
def test_cells_partition_every_entry_once_and_stratum_matrices(N, D, P):
    rng = np.random.default_rng(N * 100 + D)
    rowptr, col, val = random_csr(rng, N, D, 0.4)
    X = O.make_matrix(N, D, rowptr, col, val)
    Xd = sp.csr_matrix((val.astype(np.float64), col, rowptr), shape=(N, D)).toarray()
    stored = sp.csr_matrix((np.ones(len(col)), col, rowptr), shape=(N, D)).toarray() > 0
    rb, cb = [(k * N) // P for k in range(P + 1)], [(k * D) // P for k in range(P + 1)]
    # brute-force cell table from dense masks
    want = np.zeros((P, P), np.int64)
    for p in range(P):
        for q in range(P):
            want[p, q] = stored[rb[p]:rb[p + 1], cb[q]:cb[q + 1]].sum()
    got = O.cell_nnz(X, P)
    np.testing.assert_array_equal(got, want)
    assert got.sum() == len(col)
    total = np.zeros((N, D))
    count = np.zeros((N, D), np.int64)
    for s in range(P):
        mask = np.zeros((N, D), bool)
        for p, q in O.stratum_cells(P, s):
            mask[rb[p]:rb[p + 1], cb[q]:cb[q + 1]] = True
        rp, c, v = O.stratum_csr(X, P, s)
        S = sp.csr_matrix((v, c, rp), shape=(N, D))
        np.testing.assert_array_equal(S.toarray(), Xd * mask)
        assert len(c) == (stored & mask).sum()
        cp, r, cv = O.stratum_csc(X, P, s)
        T = sp.csc_matrix((cv, r, cp), shape=(N, D))
        np.testing.assert_array_equal(T.toarray(), Xd * mask)
        for j in range(D):
            assert np.all(np.diff(r[cp[j]:cp[j + 1]]) > 0)
        total += S.toarray()
        count += mask
    np.testing.assert_array_equal(total, Xd)
    assert np.all(count == 1)  # the P strata tile the whole grid exactly once


def test_ring_schedule_visits_each_cell_once_and_starts_on_diagonal():
    P = 5
    seen = set()
    for s in range(P):
        cells = O.stratum_cells(P, s)
        assert sorted(p for p, _ in cells) == list(range(P))
        assert sorted(q for _, q in cells) == list(range(P))  # disjoint rows and columns
        seen.update(cells)
    assert len(seen) == P * P
    assert O.stratum_cells(P, 0) == [(p, p) for p in range(P)]


@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_single_block_stratified_epoch_is_full_gradient_epoch(loss):
    rng, X, Xs, y, w, V = _rand_problem(21, 40, 18, 3, 0.3, loss)
    kw = dict(loss=loss, s=1.0 / X.N, lambda_w=0.01, lambda_v=0.02, eta=0.3)
    w0a, wa, Va, _ = O.full_epoch(X, y, 0.1, w, V, **kw)
    w0b, wb, Vb, _, aux = O.stratified_epoch(X, y, 0.1, w, V, P=1, **kw)
    np.testing.assert_allclose(wb, wa, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(Vb, Va, rtol=1e-13, atol=1e-15)
    # the bias step of the stratified epoch uses the refreshed aggregates, so compare
    # with the multiplier at the updated (w,V) and the old bias
    _, _, _, yh = O.forward(X, 0.1, wa, Va)
    _, r = O.loss_multiplier(loss, kw["s"], yh, y)
    np.testing.assert_allclose(w0b, 0.1 - kw["eta"] * r.sum(), rtol=1e-12)
    # with one block the refreshed aggregates are exact
    np.testing.assert_allclose(aux["G"], Xs @ Vb, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(aux["a"], Xs @ wb, rtol=1e-12, atol=1e-14)


def test_cell_order_inside_a_stratum_does_not_matter():
    rng, X, Xs, y, w, V = _rand_problem(22, 50, 24, 4, 0.3)
    P = 4
    kw = dict(P=P, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=1e-3, lambda_v=1e-3, eta=0.05)
    for all_rows in (False, True):
        base = O.stratified_epoch(X, y, 0.0, w, V, refresh_all_rows=all_rows, **kw)
        order = [list(rng.permutation(P)) for _ in range(P)]
        perm = O.stratified_epoch(X, y, 0.0, w, V, refresh_all_rows=all_rows, cell_order=order, **kw)
        assert base[0] == perm[0]
        np.testing.assert_array_equal(base[1], perm[1])
        np.testing.assert_array_equal(base[2], perm[2])
        for k in ("a", "G", "q"):
            np.testing.assert_array_equal(base[4][k], perm[4][k])


def test_exact_refresh_keeps_aggregates_equal_to_fresh_recomputation():
    rng, X, Xs, y, w, V = _rand_problem(23, 45, 20, 3, 0.35)
    X2 = Xs.multiply(Xs)
    checked = []

    def check(s, st):
        np.testing.assert_allclose(st["G"], Xs @ st["V"], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(st["a"], Xs @ st["w"], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(st["q"], X2 @ (st["V"] ** 2).sum(axis=1), rtol=1e-11, atol=1e-13)
        checked.append(s)

    O.stratified_epoch(X, y, 0.0, w, V, P=5, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=1e-3, lambda_v=1e-3,
                       eta=0.05, refresh_all_rows=True, on_stratum=check)
    assert checked == list(range(5))


def test_own_row_refresh_tracks_exactly_the_deltas_a_row_block_applied():
    """With the paper's local refresh a row block's aggregates hold the epoch-start
    parameters plus the changes that this row block itself made; changes made by
    other row blocks are missing until the next re-computation."""
    rng, X, Xs, y, w, V = _rand_problem(24, 48, 21, 3, 0.35)
    P, N, D = 4, X.N, X.D
    rb, cb = [(k * N) // P for k in range(P + 1)], [(k * D) // P for k in range(P + 1)]
    own_dV = [np.zeros_like(V) for _ in range(P)]
    own_dw = [np.zeros_like(w) for _ in range(P)]
    stale_seen = []

    def check(s, st):
        for p, q in st["cells"]:
            own_dV[p][cb[q]:cb[q + 1]] += st["dV"][cb[q]:cb[q + 1]]
            own_dw[p][cb[q]:cb[q + 1]] += st["dw"][cb[q]:cb[q + 1]]
        for p in range(P):
            I = slice(rb[p], rb[p + 1])
            np.testing.assert_allclose(st["G"][I], (Xs @ (V + own_dV[p]))[I], rtol=1e-11, atol=1e-13)
            np.testing.assert_allclose(st["a"][I], (Xs @ (w + own_dw[p]))[I], rtol=1e-11, atol=1e-13)
        stale_seen.append(np.abs(st["G"] - Xs @ st["V"]).max())

    out = O.stratified_epoch(X, y, 0.0, w, V, P=P, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=1e-3,
                             lambda_v=1e-3, eta=0.05, on_stratum=check)
    assert max(stale_seen) > 1e-6  # the staleness is real
    # every parameter moved by the sum of the deltas of the P row blocks
    np.testing.assert_allclose(out[2], V + sum(own_dV), rtol=1e-12, atol=1e-14)


def test_cell_gradients_sum_to_the_full_gradient_at_frozen_parameters():
    rng, X, Xs, y, w, V = _rand_problem(25, 36, 16, 3, 0.4)
    P, N, D, K = 4, X.N, X.D, V.shape[1]
    s, lw, lv = 0.5, 0.02, 0.03
    a, G, q, yhat = O.forward(X, 0.2, w, V)
    _, r = O.loss_multiplier(O.LOSS_LOGISTIC, s, yhat, y)
    gw0, gw, gV = O.gradient(X, r, G, w, V, lw, lv)
    rb, cb = O.block_bounds(N, P), O.block_bounds(D, P)
    acc_w, acc_V = np.zeros(D), np.zeros((D, K))
    L = O._L()
    f64, i64, i32, p_ = O._f64, O._i64, O._i32, O._p
    for p in range(P):
        for qb in range(P):
            wc, Vc, rc = w.copy(), V.copy(), np.zeros(N)
            dw, dV, dn = np.zeros(D), np.zeros((D, K)), np.zeros(D)
            rho = (rb[p + 1] - rb[p]) / N
            # eta = 1 at frozen copies: the recorded delta is minus the cell gradient
            L.oracle_cell_update(i32(K), i32(O.LOSS_LOGISTIC), f64(s), f64(1.0), f64(rho), f64(lw), f64(lv),
                                 i64(rb[p]), i64(rb[p + 1]), i64(cb[qb]), i64(cb[qb + 1]), p_(X.colptr),
                                 p_(X.row), p_(X.cval), p_(y), f64(0.2), p_(a), p_(G), p_(q), p_(rc),
                                 p_(wc), p_(Vc), p_(dw), p_(dV), p_(dn))
            acc_w -= dw
            acc_V -= dV
            np.testing.assert_allclose(dn[cb[qb]:cb[qb + 1]],
                                       (Vc ** 2).sum(1)[cb[qb]:cb[qb + 1]] - (V ** 2).sum(1)[cb[qb]:cb[qb + 1]],
                                       rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(acc_w, gw, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(acc_V, gV, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("all_rows", [False, True])
def test_stratified_objective_decreases_for_small_step(all_rows):
    rng, X, Xs, y, w, V = _rand_problem(26, 80, 30, 4, 0.25)
    w0, prev = 0.0, np.inf
    for _ in range(8):
        w0, w, V, obj, _ = O.stratified_epoch(X, y, w0, w, V, P=4, loss=O.LOSS_LOGISTIC, s=1.0 / X.N,
                                              lambda_w=1e-3, lambda_v=1e-3, eta=0.2,
                                              refresh_all_rows=all_rows)
        assert sum(obj) < prev
        prev = sum(obj)


def test_full_regulariser_per_cell_differs_only_by_the_regulariser_share():
    rng, X, Xs, y, w, V = _rand_problem(27, 40, 16, 2, 0.3)
    kw = dict(P=4, loss=O.LOSS_SQUARED, s=1.0 / X.N, eta=0.1)
    a = O.stratified_epoch(X, y, 0.0, w, V, lambda_w=0.0, lambda_v=0.0, reg_share=True, **kw)
    b = O.stratified_epoch(X, y, 0.0, w, V, lambda_w=0.0, lambda_v=0.0, reg_share=False, **kw)
    np.testing.assert_array_equal(a[1], b[1])  # no regulariser: identical
    c = O.stratified_epoch(X, y, 0.0, w, V, lambda_w=0.5, lambda_v=0.5, reg_share=False, **kw)
    d = O.stratified_epoch(X, y, 0.0, w, V, lambda_w=0.5, lambda_v=0.5, reg_share=True, **kw)
    assert np.linalg.norm(c[1]) < np.linalg.norm(d[1])  # full lambda per cell shrinks harder


@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_stale_aggregate_epoch_without_regulariser_is_the_full_gradient_epoch(loss):
    """Every cell step of a stale epoch reads the aggregates (hence the multipliers r) of the
    epoch's start, and every cell is visited once.  With lambda = 0 the steps on w and w0 add up
    to one full-gradient step at the starting point, whatever P is.  The gradient of v_j also
    holds v_j itself (the term -v_jk sum_i x_ij^2 r_i), which moves from one cell step to the
    next: V follows the affine maps v <- v - eta (gV_p - s2_p v) in the order of the ring, with
    gV_p, s2_p the sums over row block p at the frozen r and G (equal to the full step when P = 1)."""
    rng, X, Xs, y, w, V = _rand_problem(41, 60, 26, 4, 0.3)
    N, D = Xs.shape
    kw = dict(loss=loss, s=1.0 / 60, lambda_w=0.0, lambda_v=0.0, eta=0.07)
    w0a, wa, Va, _ = O.full_epoch(X, y, 0.2, w, V, **kw)
    _, G0, _, yh = O.forward(X, 0.2, w, V)
    _, r0 = O.loss_multiplier(loss, kw["s"], yh, y)
    for P in (1, 3, 7):
        w0b, wb, Vb, _, aux = O.stratified_epoch(X, y, 0.2, w, V, P=P, stale_aux=True, **kw)
        np.testing.assert_allclose(wb, wa, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(w0b, w0a, rtol=1e-12)
        rb, cb = O.block_bounds(N, P), O.block_bounds(D, P)
        want = V.copy()
        for q in range(P):
            J = slice(cb[q], cb[q + 1])
            for st in range(P):
                pb = (q - st) % P
                Xp = Xs[rb[pb]:rb[pb + 1], J]
                rp, Gp = r0[rb[pb]:rb[pb + 1]], G0[rb[pb]:rb[pb + 1]]
                gV = Xp.T @ (rp[:, None] * Gp)
                s2 = Xp.multiply(Xp).T @ rp
                want[J] = want[J] - kw["eta"] * (gV - s2[:, None] * want[J])
        np.testing.assert_allclose(Vb, want, rtol=1e-11, atol=1e-15)
        if P == 1:
            np.testing.assert_allclose(Vb, Va, rtol=1e-12, atol=1e-15)
        # the aggregates were never touched: still those of the starting point
        np.testing.assert_allclose(aux["G"], Xs @ V, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(aux["a"], Xs @ w, rtol=1e-12, atol=1e-14)


def test_stale_aggregate_epoch_with_regulariser_shrinks_each_column_by_its_shares():
    """With lambda > 0 and no data (y chosen so that r = 0: squared loss at y = yhat) a stale
    epoch multiplies every w_j by prod_p (1 - eta rho_p lambda), rho_p = |I_p|/N."""
    rng, X, Xs, y, w, V = _rand_problem(42, 50, 18, 3, 0.3)
    _, _, _, yh = O.forward(X, 0.0, w, V)
    P, eta, lw, lv = 4, 0.3, 0.2, 0.1
    _, wb, Vb, _, _ = O.stratified_epoch(X, yh, 0.0, w, V, P=P, stale_aux=True, loss=O.LOSS_SQUARED, s=1.0,
                                         lambda_w=lw, lambda_v=lv, eta=eta)
    rb = O.block_bounds(X.N, P)
    fw = np.prod([1 - eta * lw * (rb[p + 1] - rb[p]) / X.N for p in range(P)])
    fv = np.prod([1 - eta * lv * (rb[p + 1] - rb[p]) / X.N for p in range(P)])
    np.testing.assert_allclose(wb, w * fw, rtol=1e-12)
    np.testing.assert_allclose(Vb, V * fv, rtol=1e-12)


def test_stale_and_refreshed_epochs_differ_once_there_are_several_blocks():
    rng, X, Xs, y, w, V = _rand_problem(43, 60, 26, 4, 0.3)
    kw = dict(P=4, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=1e-3, lambda_v=1e-3, eta=0.05)
    a = O.stratified_epoch(X, y, 0.0, w, V, **kw)
    b = O.stratified_epoch(X, y, 0.0, w, V, stale_aux=True, **kw)
    assert np.abs(a[2] - b[2]).max() > 1e-6


@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_single_batch_minibatch_epoch_is_the_full_gradient_epoch(loss):
    rng, X, Xs, y, w, V = _rand_problem(51, 40, 18, 3, 0.3, loss)
    kw = dict(loss=loss, s=1.0 / 40, lambda_w=1e-2, lambda_v=2e-2, eta=0.1)
    w0a, wa, Va, _ = O.full_epoch(X, y, 0.3, w, V, **kw)
    w0b, wb, Vb, _ = O.minibatch_epoch(X, y, 0.3, w, V, B=1, **kw)
    np.testing.assert_allclose(w0b, w0a, rtol=1e-13)
    np.testing.assert_allclose(wb, wa, rtol=1e-13, atol=1e-16)
    np.testing.assert_allclose(Vb, Va, rtol=1e-13, atol=1e-16)


@pytest.mark.parametrize("loss,share", [(O.LOSS_SQUARED, True), (O.LOSS_LOGISTIC, True), (O.LOSS_LOGISTIC, False)])
def test_every_minibatch_step_is_a_gradient_step_on_the_batch_objective(loss, share):
    """The move of a batch step, divided by -eta, is the gradient of
    s sum_{i in batch} l_i + rho (lambda_w/2 |w|^2 + lambda_v/2 |V|^2) at the parameters the step
    started from: checked by central differences of the objective of the sub-matrix made of the
    batch's rows (an independent route: it never sees the other rows)."""
    N, D, K, B = 37, 15, 3, 4
    rng, X, Xs, y, w, V = _rand_problem(52, N, D, K, 0.35, loss)
    lw, lv, eta, s = 0.05, 0.08, 0.2, 1.0 / N
    rb = O.block_bounds(N, B)
    prev = dict(w0=0.1, w=w.copy(), V=V.copy())
    seen = []

    def check(b, st):
        lo, hi = st["rows"]
        assert (lo, hi) == (rb[b], rb[b + 1])
        sub = Xs[lo:hi].tocsr()
        sub.sort_indices()
        Xb = O.make_matrix(hi - lo, D, sub.indptr.astype(np.int64), sub.indices.astype(np.int32),
                           sub.data.astype(np.float32))
        rho = (hi - lo) / N if share else 1.0

        def F(w0_, w_, V_):
            o = O.objective(loss, s, rho * lw, rho * lv, Xb, y[lo:hi], w0_, w_, V_)
            return o[0] + o[1]

        h = 1e-6
        gw0 = (F(prev["w0"] + h, prev["w"], prev["V"]) - F(prev["w0"] - h, prev["w"], prev["V"])) / (2 * h)
        np.testing.assert_allclose((st["w0"] - prev["w0"]) / -eta, gw0, rtol=1e-6, atol=1e-9)
        for _ in range(6):
            j, k = int(rng.integers(D)), int(rng.integers(K))
            e = np.zeros(D); e[j] = h
            gw = (F(prev["w0"], prev["w"] + e, prev["V"]) - F(prev["w0"], prev["w"] - e, prev["V"])) / (2 * h)
            np.testing.assert_allclose((st["w"][j] - prev["w"][j]) / -eta, gw, rtol=1e-6, atol=1e-9)
            E = np.zeros((D, K)); E[j, k] = h
            gv = (F(prev["w0"], prev["w"], prev["V"] + E) - F(prev["w0"], prev["w"], prev["V"] - E)) / (2 * h)
            np.testing.assert_allclose((st["V"][j, k] - prev["V"][j, k]) / -eta, gv, rtol=1e-6, atol=1e-9)
        prev.update(w0=st["w0"], w=st["w"].copy(), V=st["V"].copy())
        seen.append(b)

    O.minibatch_epoch(X, y, 0.1, w, V, B=B, loss=loss, s=s, lambda_w=lw, lambda_v=lv, eta=eta, reg_share=share,
                      on_batch=check, final_objective=False)
    assert seen == list(range(B))


def test_batch_csc_keeps_each_entry_in_exactly_one_batch():
    rng, X, Xs, y, w, V = _rand_problem(53, 29, 13, 2, 0.3)
    B = 5
    dense = Xs.toarray()
    rb = O.block_bounds(29, B)
    total = 0
    for b in range(B):
        colptr, row, val = O.batch_csc(X, B, b)
        sub = np.zeros_like(dense)
        for j in range(13):
            for e in range(colptr[j], colptr[j + 1]):
                sub[row[e], j] = val[e]
            assert np.all(np.diff(row[colptr[j]:colptr[j + 1]]) > 0)
        want = np.zeros_like(dense)
        want[rb[b]:rb[b + 1]] = dense[rb[b]:rb[b + 1]]
        np.testing.assert_array_equal(sub, want)
        total += len(row)
    assert total == len(X.col)


# ---- Algorithm 1 with every column handed on individually (placed_epoch) ----

@pytest.mark.parametrize("stale", [True, False])
@pytest.mark.parametrize("P", [1, 3, 5])
def test_block_placement_reproduces_the_ring(P, stale):
    """With place[j] = column block of j the per-column schedule is the ring of stratified_epoch:
    same cells in the same rounds, so every number agrees bit for bit (stale and refreshed)."""
    rng, X, Xs, y, w, V = _rand_problem(51, 70, 23, 3, 0.3)
    kw = dict(P=P, loss=O.LOSS_LOGISTIC, s=1.0 / 70, lambda_w=2e-2, lambda_v=1e-2, eta=0.4)
    a = O.stratified_epoch(X, y, 0.1, w, V, stale_aux=stale, **kw)
    b = O.placed_epoch(X, y, 0.1, w, V, place=O.block_placement(X.D, P), stale_aux=stale, **kw)
    assert a[0] == b[0]
    np.testing.assert_array_equal(a[1], b[1])
    np.testing.assert_array_equal(a[2], b[2])
    for k in ("a", "G", "q", "r"):
        np.testing.assert_array_equal(a[4][k], b[4][k])


def test_every_column_meets_every_row_block_once_whatever_the_placement():
    rng, X, Xs, y, w, V = _rand_problem(52, 40, 17, 2, 0.3)
    P = 6
    place = rng.integers(0, P, X.D)
    seen = np.zeros((P, X.D), int)

    def on_round(t, st):
        held = st["held"]
        assert sorted(np.concatenate(held).tolist()) == list(range(X.D))  # every column is somewhere, once
        for p in range(P):
            seen[p, held[p]] += 1
        if t == 0:
            for p in range(P):
                assert set(held[p].tolist()) == set(np.flatnonzero(place == p).tolist())  # the initial placement

    O.placed_epoch(X, y, 0.0, w, V, P=P, place=place, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=0.0, lambda_v=0.0,
                   eta=0.1, on_round=on_round)
    assert (seen == 1).all()


@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_stale_placed_epoch_without_regulariser_matches_the_closed_form(loss):
    """lambda = 0, stale aggregates: the multipliers never change, so w and w0 take exactly one
    full-gradient step whatever the placement, and v_j follows the affine maps
    v <- v - eta (gV_p - s2_p v) over the row blocks in the order column j meets them,
    place[j], place[j]-1, ... (mod P), with gV_p, s2_p from the frozen r and G (dense products here)."""
    rng, X, Xs, y, w, V = _rand_problem(53, 60, 19, 4, 0.35)
    N, D = Xs.shape
    P = 5
    place = rng.integers(0, P, D)
    kw = dict(loss=loss, s=1.0 / N, lambda_w=0.0, lambda_v=0.0, eta=0.09)
    w0a, wa, _, _ = O.full_epoch(X, y, 0.2, w, V, **kw)
    _, G0, _, yh = O.forward(X, 0.2, w, V)
    _, r0 = O.loss_multiplier(loss, kw["s"], yh, y)
    w0b, wb, Vb, _, aux = O.placed_epoch(X, y, 0.2, w, V, P=P, place=place, stale_aux=True, **kw)
    np.testing.assert_allclose(wb, wa, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(w0b, w0a, rtol=1e-12)
    rb = O.block_bounds(N, P)
    Xd = Xs.toarray()
    want = V.copy()
    for j in range(D):
        for t in range(P):
            pb = (place[j] - t) % P
            I = slice(rb[pb], rb[pb + 1])
            x = Xd[I, j]
            gV = (x * r0[I]) @ G0[I]
            s2 = (x * x) @ r0[I]
            want[j] = want[j] - kw["eta"] * (gV - s2 * want[j])
    np.testing.assert_allclose(Vb, want, rtol=1e-11, atol=1e-15)
    np.testing.assert_allclose(aux["G"], Xs @ V, rtol=1e-12, atol=1e-14)  # never refreshed


def test_stale_placed_epoch_without_data_shrinks_every_column_by_all_shares():
    """r = 0 (squared loss at y = yhat): every column meets every row block once, so it is multiplied by
    prod_p (1 - eta rho_p lambda) whatever the placement."""
    rng, X, Xs, y, w, V = _rand_problem(54, 50, 18, 3, 0.3)
    _, _, _, yh = O.forward(X, 0.0, w, V)
    P, eta, lw, lv = 4, 0.3, 0.2, 0.1
    place = rng.integers(0, P, X.D)
    _, wb, Vb, _, _ = O.placed_epoch(X, yh, 0.0, w, V, P=P, place=place, stale_aux=True, loss=O.LOSS_SQUARED, s=1.0,
                                     lambda_w=lw, lambda_v=lv, eta=eta)
    rb = O.block_bounds(X.N, P)
    fw = np.prod([1 - eta * lw * (rb[p + 1] - rb[p]) / X.N for p in range(P)])
    fv = np.prod([1 - eta * lv * (rb[p + 1] - rb[p]) / X.N for p in range(P)])
    np.testing.assert_allclose(wb, w * fw, rtol=1e-12)
    np.testing.assert_allclose(Vb, V * fv, rtol=1e-12)


def test_refreshed_placed_epoch_keeps_own_deltas_and_differs_from_the_stale_one():
    """With the incremental refresh a worker's aggregates hold exactly the changes it applied itself:
    G_I = X_I V0 + sum over the rounds of X_{I,J_t} dV_{J_t}; and the result differs from the stale epoch."""
    rng, X, Xs, y, w, V = _rand_problem(55, 48, 20, 3, 0.3)
    P = 4
    place = rng.integers(0, P, X.D)
    kw = dict(P=P, place=place, loss=O.LOSS_LOGISTIC, s=1.0, lambda_w=1e-3, lambda_v=1e-3, eta=0.05)
    rb = O.block_bounds(X.N, P)
    Xd = Xs.toarray()
    want = Xd @ V
    prev = {"V": V.copy()}

    def on_round(t, st):
        dV = st["V"] - prev["V"]
        for p in range(P):
            I = slice(rb[p], rb[p + 1])
            J = st["held"][p]
            want[I] += Xd[I][:, J] @ dV[J]
        prev["V"] = st["V"].copy()
        np.testing.assert_allclose(st["G"], want, rtol=1e-11, atol=1e-13)

    a = O.placed_epoch(X, y, 0.0, w, V, stale_aux=False, on_round=on_round, **kw)
    b = O.placed_epoch(X, y, 0.0, w, V, stale_aux=True, **kw)
    assert np.abs(a[2] - b[2]).max() > 1e-6
