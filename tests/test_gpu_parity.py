"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle on the
same seeded inputs.  Integer structures must match bit for bit; fp32 outputs within
1e-4 relative (per array, see helpers.rel_err)."""
import numpy as np
import pytest

from oracle import fm_oracle as O
from paper_2004_13940_amd.workloads import make_config, random_csr

from helpers import REL_TOL, assert_close, dev_params, oracle_kw, to_dev
from helpers import run_full_epochs as _run_full_epochs, run_stratified_epochs as _run_stratified_epochs

pytestmark = pytest.mark.gpu


def _B():
    from paper_2004_13940_amd import binding
    return binding


def _say(*a):
    print(*a, flush=True)


def _problem(seed, N, D, K, density, loss, dense_cols=(), long_row=False):
    """Random CSR with optional dense columns (longer than one column segment) and
    one very long row; labels, parameters."""
    rng = np.random.default_rng(seed)
    mask = rng.random((N, D)) < density
    for c in dense_cols:
        mask[:, c] = True
    if long_row:
        mask[N // 2, :] = True
    rowptr = np.zeros(N + 1, np.int64)
    np.cumsum(mask.sum(axis=1), out=rowptr[1:])
    col = np.nonzero(mask)[1].astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    y = (np.where(rng.random(N) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(N)).astype(np.float32)
    w0 = np.float32(0.1)
    w = (rng.standard_normal(D) * 0.1).astype(np.float32)
    V = (rng.standard_normal((D, K)) * 0.1).astype(np.float32)
    return rowptr, col, val, y, w0, w, V


# ------------------------------------------------------------ structures ----

@pytest.mark.parametrize("N,D,density,dense", [(1, 1, 1.0, ()), (50, 40, 0.1, ()), (3000, 700, 0.02, (5, 699)),
                                               (257, 5000, 0.01, ()), (40, 30, 0.0, ())])
def test_csc_transpose_is_bit_exact(N, D, density, dense):
    B = _B()
    rowptr, col, val, *_ = _problem(N * 7 + D, N, D, 1, density, O.LOSS_SQUARED, dense)
    _say("transpose", N, D, len(col))
    m = B.Matrix(N, D, rowptr, col, val)
    m.fm_build_csc()
    colptr, row, cval = m.fm_get_csc()
    wp, wr, wv = O.csr_to_csc(N, D, rowptr, col, val)
    np.testing.assert_array_equal(colptr, wp)
    np.testing.assert_array_equal(row, wr)
    np.testing.assert_array_equal(cval, wv.astype(np.float32))
    m.close()


def test_csc_transpose_of_workloads_is_bit_exact():
    B = _B()
    for idx, scale in [(1, 1.0), (3, 0.2), (4, 0.002), (5, 0.002)]:
        wl = make_config(idx, scale=scale)
        _say("transpose workload", wl.name, wl.N, wl.D, wl.nnz)
        m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
        m.fm_build_csc()
        colptr, row, cval = m.fm_get_csc()
        wp, wr, wv = O.csr_to_csc(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
        np.testing.assert_array_equal(colptr, wp)
        np.testing.assert_array_equal(row, wr)
        np.testing.assert_array_equal(cval, wv.astype(np.float32))
        m.close()


@pytest.mark.parametrize("N,D,P,density", [(60, 40, 4, 0.2), (17, 9, 5, 0.4), (6, 3, 8, 0.6), (12, 12, 1, 0.3),
                                           (2500, 300, 7, 0.05), (100, 70, 64, 0.1)])
def test_partition_and_stratum_matrices_are_bit_exact(N, D, P, density):
    B = _B()
    rowptr, col, val, *_ = _problem(N + D + P, N, D, 1, density, O.LOSS_SQUARED, (0,) if N > 1000 else ())
    _say("partition", N, D, P, len(col))
    X = O.make_matrix(N, D, rowptr, col, val)
    m = B.Matrix(N, D, rowptr, col, val)
    m.fm_build_csc()
    m.fm_partition(P)
    rb, cb, cells = m.fm_get_block_index()
    np.testing.assert_array_equal(rb, O.block_bounds(N, P))
    np.testing.assert_array_equal(cb, O.block_bounds(D, P))
    np.testing.assert_array_equal(cells, O.cell_nnz(X, P))
    total = 0
    for s in range(P):
        rp, c, v = m.fm_get_stratum_csr(s)
        wrp, wc, wv = O.stratum_csr(X, P, s)
        np.testing.assert_array_equal(rp, wrp)
        np.testing.assert_array_equal(c, wc)
        np.testing.assert_array_equal(v, wv.astype(np.float32))
        cp, r, cv = m.fm_get_stratum_csc(s)
        wcp, wr, wcv = O.stratum_csc(X, P, s)
        np.testing.assert_array_equal(cp, wcp)
        np.testing.assert_array_equal(r, wr)
        np.testing.assert_array_equal(cv, wcv.astype(np.float32))
        total += len(c)
    assert total == len(col)
    m.close()


def test_partition_of_text_like_workload_is_bit_exact():
    B = _B()
    wl = make_config(3, scale=0.1)
    X = O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    m.fm_partition(wl.P)
    rb, cb, cells = m.fm_get_block_index()
    np.testing.assert_array_equal(cells, O.cell_nnz(X, wl.P))
    for s in (0, 1, wl.P - 1):
        rp, c, v = m.fm_get_stratum_csr(s)
        wrp, wc, wv = O.stratum_csr(X, wl.P, s)
        np.testing.assert_array_equal(rp, wrp)
        np.testing.assert_array_equal(c, wc)
        cp, r, cv = m.fm_get_stratum_csc(s)
        wcp, wr, wcv = O.stratum_csc(X, wl.P, s)
        np.testing.assert_array_equal(cp, wcp)
        np.testing.assert_array_equal(r, wr)
    m.close()


# --------------------------------------------------------- forward/gradient ----

def _forward_both(B, rowptr, col, val, y, w0, w, V, N, D, K, loss, s):
    import torch
    p = B.make_params(K, loss, 0.01, 0.02, 0.1, loss_scale=s)
    m = B.Matrix(N, D, rowptr, col, val)
    d_w0, d_w, d_V = dev_params(w0, w, V)
    d_y = to_dev(y)
    out = {k: torch.full((N * (K if k == "G" else 1),), float("nan"), device="cuda") for k in ("yhat", "a", "G", "q", "r")}
    loss_sum = m.fm_forward(p, d_y, d_w0, d_w, d_V, want_loss=True, **out)
    torch.cuda.synchronize()
    X = O.make_matrix(N, D, rowptr, col, val)
    a, G, q, yhat = O.forward(X, float(w0), w, V)
    l, r = O.loss_multiplier(loss, s, yhat, y)
    want = dict(yhat=yhat, a=a, G=G, q=q, r=r)
    return m, p, X, out, loss_sum, want, float(l.sum())


@pytest.mark.parametrize("K", [1, 2, 3, 6, 8, 16, 32, 64, 128])
@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_forward_matches_oracle_for_all_K(K, loss):
    B = _B()
    N, D = 333, 97  # ragged: not a multiple of any rows-per-block
    rowptr, col, val, y, w0, w, V = _problem(100 + K, N, D, K, 0.15, loss, long_row=True)
    _say("forward", K, loss, len(col))
    m, p, X, out, loss_sum, want, want_loss = _forward_both(B, rowptr, col, val, y, w0, w, V, N, D, K, loss, 0.5)
    for k in want:
        assert_close(out[k].cpu().numpy(), want[k], f"{k} K={K}")
    assert abs(loss_sum - want_loss) <= REL_TOL * abs(want_loss)
    m.close()


@pytest.mark.parametrize("K", [1, 3, 8, 16, 64])
@pytest.mark.parametrize("loss", [O.LOSS_SQUARED, O.LOSS_LOGISTIC])
def test_gradient_matches_oracle(K, loss):
    import torch
    B = _B()
    N, D = 2100, 130  # columns 3 and 129 are dense: 2100 entries > one 512-entry segment
    rowptr, col, val, y, w0, w, V = _problem(200 + K, N, D, K, 0.05, loss, dense_cols=(3, 129))
    _say("gradient", K, loss, len(col))
    m, p, X, out, _, want, _ = _forward_both(B, rowptr, col, val, y, w0, w, V, N, D, K, loss, 1.0 / N)
    m.fm_build_csc()
    d_w0, d_w, d_V = dev_params(w0, w, V)
    g0 = torch.zeros(1, device="cuda")
    gw = torch.full((D,), float("nan"), device="cuda")
    gV = torch.full((D * K,), float("nan"), device="cuda")
    m.fm_gradient(p, out["r"], out["G"], d_w, d_V, g0, gw, gV)
    torch.cuda.synchronize()
    # the oracle's gradient from ITS OWN r and G (the inputs differ only by fp32 rounding)
    wg0, wgw, wgV = O.gradient(X, want["r"], want["G"], w, V, p.lambda_w, p.lambda_v)
    assert abs(g0.item() - wg0) <= REL_TOL * max(abs(wg0), np.abs(want["r"]).sum() * 1e-3)
    assert_close(gw.cpu().numpy(), wgw, "grad_w")
    assert_close(gV.cpu().numpy(), wgV, "grad_V")
    # parameters untouched by fm_gradient
    np.testing.assert_array_equal(d_V.cpu().numpy().reshape(D, K), V)
    m.close()


def test_empty_rows_empty_columns_and_zero_entries():
    import torch
    B = _B()
    N, D, K = 40, 30, 8
    rowptr = np.zeros(N + 1, np.int64)  # nothing stored at all
    m = B.Matrix(N, D, rowptr, np.zeros(0, np.int32), np.zeros(0, np.float32))
    m.fm_build_csc()
    p = B.make_params(K, B.FM_LOSS_LOGISTIC, 0.5, 0.25, 0.1)
    rng = np.random.default_rng(0)
    w = rng.standard_normal(D).astype(np.float32)
    V = rng.standard_normal((D, K)).astype(np.float32)
    d_w0, d_w, d_V = dev_params(0.7, w, V)
    y = to_dev(np.ones(N))
    yhat, G, r = torch.empty(N, device="cuda"), torch.empty(N * K, device="cuda"), torch.empty(N, device="cuda")
    loss = m.fm_forward(p, y, d_w0, d_w, d_V, yhat=yhat, G=G, r=r, want_loss=True)
    np.testing.assert_array_equal(yhat.cpu().numpy(), np.float32(0.7))
    assert not G.cpu().numpy().any()
    assert abs(loss - N * np.log1p(np.exp(-0.7))) < 1e-4 * N
    gw, gV = torch.empty(D, device="cuda"), torch.empty(D * K, device="cuda")
    m.fm_gradient(p, r, G, d_w, d_V, None, gw, gV)
    np.testing.assert_allclose(gw.cpu().numpy(), 0.5 * w, rtol=1e-6)
    np.testing.assert_allclose(gV.cpu().numpy().reshape(D, K), 0.25 * V, rtol=1e-6)
    m.close()


# ------------------------------------------------------------ full epochs ----

def test_config1_ten_full_then_ten_stratified_epochs():
    B = _B()
    wl = make_config(1)
    _say("config 1", wl.N, wl.D, wl.nnz)
    m, p, X, dev, host = _run_full_epochs(B, wl, wl.epochs)
    m.fm_partition(wl.P)
    _run_stratified_epochs(B, wl, m, p, X, dev, host, wl.epochs)
    m.close()


def test_config1_stratified_from_the_initial_point_with_aggregates_checked_per_stratum():
    B = _B()
    wl = make_config(1)
    m, p, X, dev, host = _run_full_epochs(B, wl, 0)
    m.fm_partition(wl.P)
    _run_stratified_epochs(B, wl, m, p, X, dev, host, 2, check_strata=True)
    m.close()


@pytest.mark.parametrize("idx,scale,epochs", [(2, 0.004, 3), (3, 0.1, 3), (4, 0.001, 2), (5, 0.002, 2)])
def test_scaled_workloads_full_and_stratified_epochs(idx, scale, epochs):
    B = _B()
    wl = make_config(idx, scale=scale)
    _say("workload", wl.name, wl.N, wl.D, wl.nnz, "K", wl.K, "P", wl.P)
    m, p, X, dev, host = _run_full_epochs(B, wl, epochs)
    m.fm_partition(wl.P)
    _run_stratified_epochs(B, wl, m, p, X, dev, host, 2)
    m.close()


@pytest.mark.parametrize("P,flags", [(1, {}), (3, {}), (7, {"refresh_all_rows": True}),
                                     (5, {"reg_full_per_cell": True}), (64, {}),
                                     (4, {"refresh_all_rows": True, "reg_full_per_cell": True}),
                                     (6, {"stale_aux": True}), (200, {})])
def test_stratified_variants_with_per_stratum_checks(P, flags):
    """P not dividing N or D, P = 1, P > D (64, and 200: most column blocks empty, rows blocks of 11
    or 12 rows), exact refresh, full regulariser per cell; a dense column makes every stratum hold a
    column longer than one segment when P is small."""
    B = _B()
    N, D, K = 2300, 50, 8
    rowptr, col, val, y, w0, w, V = _problem(900 + P, N, D, K, 0.08, O.LOSS_LOGISTIC, dense_cols=(7,))
    from paper_2004_13940_amd.workloads import Workload
    wl = Workload("adhoc", N, D, K, rowptr, col, val, y, w0, w, V, O.LOSS_LOGISTIC, 1e-2, 2e-2, 0.5, 1.0 / N, 1, P, 1)
    _say("stratified variant", P, flags, len(col))
    m, p, X, dev, host = _run_full_epochs(B, wl, 0)
    m.fm_partition(P)
    _run_stratified_epochs(B, wl, m, p, X, dev, host, 2, check_strata=True, **flags)
    m.close()


def test_stale_aggregate_epochs_of_a_scaled_workload():
    """Algorithm 1's two phases (no refresh between strata) through fm_stratified_epoch, where the
    regulariser-only steps are postponed as well."""
    B = _B()
    wl = make_config(3, scale=0.1)
    m, p, X, dev, host = _run_full_epochs(B, wl, 1)
    m.fm_partition(wl.P)
    _run_stratified_epochs(B, wl, m, p, X, dev, host, 3, stale_aux=True)
    m.close()


@pytest.mark.parametrize("K", [5, 12, 20, 60, 252, 256])
def test_odd_and_large_latent_sizes_through_whole_epochs(K):
    """K that is odd (one float per lane), not a power of two, at the limit of the packed
    aggregate rows (252) and beyond it (256: planar rows, 64 lanes per group)."""
    B = _B()
    N, D = 700, 90
    rowptr, col, val, y, w0, w, V = _problem(300 + K, N, D, K, 0.1, O.LOSS_LOGISTIC, dense_cols=(11,))
    V *= np.float32(0.3)
    from paper_2004_13940_amd.workloads import Workload
    wl = Workload("ksize", N, D, K, rowptr, col, val, y, w0, w, V, O.LOSS_LOGISTIC, 1e-3, 1e-3, 0.2, 1.0 / N, 2, 3, 1)
    _say("latent size", K, len(col))
    m, p, X, dev, host = _run_full_epochs(B, wl, 2)
    m.fm_partition(3)
    _run_stratified_epochs(B, wl, m, p, X, dev, host, 1)
    m.close()


def test_single_block_stratified_epoch_equals_full_gradient_epoch_on_gpu():
    import torch
    B = _B()
    wl = make_config(1)
    wl.update_w0 = 0
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    m.fm_partition(1)
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, 0)
    y = to_dev(wl.y)
    a0, aw, aV = dev_params(wl.w0, wl.w, wl.V)
    b0, bw, bV = dev_params(wl.w0, wl.w, wl.V)
    m.fm_sgd_epoch(p, y, a0, aw, aV)
    m.fm_stratified_epoch(p, y, b0, bw, bV)
    torch.cuda.synchronize()
    # same kernels, same order of additions: identical bits
    assert torch.equal(aw, bw) and torch.equal(aV, bV)
    m.close()


@pytest.mark.parametrize("idx,scale,P,full_reg", [(3, 0.05, 8, False), (5, 0.002, 16, False), (5, 0.002, 5, True)])
def test_postponed_regulariser_steps_agree_with_immediate_ones(idx, scale, P, full_reg):
    """fm_stratified_epoch lets a column that is empty in its cell take its regulariser-only steps
    later, as one multiplication by their product (formed in fp64); fm_stratified_step takes every
    step at once, one rounded multiplication each.  They differ by the rounding of at most P - 1
    fp32 multiplications."""
    import torch
    B = _B()
    wl = make_config(idx, scale=scale)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    m.fm_partition(P)
    p = B.make_params(wl.K, wl.loss, 1e-2, 2e-2, wl.eta, wl.loss_scale, 1)
    p.reg_full_per_cell = int(full_reg)
    y = to_dev(wl.y)
    a0, aw, aV = dev_params(wl.w0, wl.w, wl.V)
    b0, bw, bV = dev_params(wl.w0, wl.w, wl.V)
    for _ in range(2):
        m.fm_stratified_epoch(p, y, a0, aw, aV)
        m.fm_stratified_begin(p, y, b0, bw, bV)
        for s in range(P):
            m.fm_stratified_step(p, s, y, b0, bw, bV)
        m.fm_stratified_end(p, b0)
        torch.cuda.synchronize()
        tol = 2.0 ** -23 * P
        for x, z in ((aw, bw), (aV, bV), (a0, b0)):
            x, z = x.cpu().numpy().astype(np.float64), z.cpu().numpy().astype(np.float64)
            assert np.abs(x - z).max() <= tol * max(np.abs(z).max(), 1e-30)
    assert not torch.equal(aw, to_dev(wl.w))
    m.close()


# ------------------------------------------------------- mini-batch epochs ----

@pytest.mark.parametrize("N,D,B,density", [(97, 31, 4, 0.2), (64, 50, 7, 0.1), (10, 40, 16, 0.3)])
def test_batch_csc_is_bit_exact(N, D, B, density):
    B_ = _B()
    rng = np.random.default_rng(77 + B)
    rowptr, col, val = random_csr(rng, N, D, density)
    X = O.make_matrix(N, D, rowptr, col, val)
    m = B_.Matrix(N, D, rowptr, col, val)
    m.fm_build_csc()
    m.fm_partition_batches(B)
    for b in range(B):
        colptr, row, v = m.fm_get_batch_csc(b)
        wc, wr, wv = O.batch_csc(X, B, b)
        np.testing.assert_array_equal(colptr, wc)
        np.testing.assert_array_equal(row, wr)
        np.testing.assert_array_equal(v, wv.astype(np.float32))
    m.close()


def _run_minibatch_epochs(Bm, wl, nb, epochs, full_reg=False, update_w0=True, setup=None):
    import torch
    X = O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m = Bm.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    if setup is not None:
        setup(m)
    m.fm_build_csc()
    m.fm_partition_batches(nb)
    p = Bm.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, int(update_w0),
                       reg_full_per_cell=int(full_reg))
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    w0, w, V = float(wl.w0), wl.w.astype(np.float64), wl.V.astype(np.float64)
    kw = oracle_kw(wl)
    for ep in range(epochs):
        obj = m.fm_minibatch_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        w0, w, V, wobj = O.minibatch_epoch(X, wl.y, w0, w, V, B=nb, update_w0=update_w0, reg_share=not full_reg, **kw)
        torch.cuda.synchronize()
        _say(f"  mini-batch epoch {ep}: objective gpu {obj[0] + obj[1]:.8f} oracle {wobj[0] + wobj[1]:.8f}")
        assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0])
        assert abs(obj[1] - wobj[1]) <= REL_TOL * abs(wobj[1]) + 1e-12
        assert_close(d_w.cpu().numpy(), w, f"w after mini-batch epoch {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after mini-batch epoch {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)
    return m, p, (d_w0, d_w, d_V, d_y)


@pytest.mark.parametrize("idx,scale,nb", [(1, 1.0, 5), (3, 0.1, 8), (4, 0.001, 10), (5, 0.002, 3), (2, 0.004, 4)])
def test_minibatch_epochs_of_the_workloads(idx, scale, nb):
    wl = make_config(idx, scale=scale)
    if idx == 1:
        wl.eta = 0.02  # a batch step with s = 1 still sees the curvature of 400 examples
    _say("mini-batch", wl.name, wl.N, wl.D, wl.nnz, "K", wl.K, "batches", nb)
    m, _, _ = _run_minibatch_epochs(_B(), wl, nb, 2, update_w0=bool(wl.update_w0))
    m.close()


@pytest.mark.parametrize("K,nb,full_reg", [(8, 1, False), (5, 6, False), (12, 9, True), (60, 4, False), (256, 3, False),
                                          (4, 2000, False)])
def test_minibatch_variants(K, nb, full_reg):
    """Batch counts that do not divide N, more batches than some columns have entries, the literal
    regulariser, one batch, more batches than rows (a quarter of them empty); a dense column is long
    in every batch that is large enough."""
    N, D = 1500, 70
    rowptr, col, val, y, w0, w, V = _problem(500 + K, N, D, K, 0.08, O.LOSS_LOGISTIC, dense_cols=(3,))
    V *= np.float32(0.3)
    from paper_2004_13940_amd.workloads import Workload
    wl = Workload("mb", N, D, K, rowptr, col, val, y, w0, w, V, O.LOSS_LOGISTIC, 1e-2, 2e-2, 0.3, 1.0 / N, 1, nb, 1)
    m, _, _ = _run_minibatch_epochs(_B(), wl, nb, 2, full_reg=full_reg)
    m.close()


def test_single_batch_epoch_equals_full_gradient_epoch_on_gpu():
    import torch
    B = _B()
    wl = make_config(3, scale=0.05)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    m.fm_partition_batches(1)
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, 1)
    y = to_dev(wl.y)
    a0, aw, aV = dev_params(wl.w0, wl.w, wl.V)
    b0, bw, bV = dev_params(wl.w0, wl.w, wl.V)
    m.fm_sgd_epoch(p, y, a0, aw, aV)
    m.fm_minibatch_epoch(p, y, b0, bw, bV)
    torch.cuda.synchronize()
    # the long columns are cut into items differently (panel order against fixed segments), so the
    # fp32 partial sums differ in the last bits: equal within rounding, not bit for bit
    np.testing.assert_allclose(bw.cpu().numpy(), aw.cpu().numpy(), rtol=2e-5, atol=1e-9)
    np.testing.assert_allclose(bV.cpu().numpy(), aV.cpu().numpy(), rtol=2e-5, atol=1e-9)
    assert abs(a0.item() - b0.item()) <= 1e-6 * max(1.0, abs(a0.item()))
    m.close()


def test_minibatch_needs_its_partition():
    B = _B()
    wl = make_config(1)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, 0)
    y = to_dev(wl.y)
    w0, w, V = dev_params(wl.w0, wl.w, wl.V)
    with pytest.raises(B.FMError):
        m.fm_minibatch_epoch(p, y, w0, w, V)
    with pytest.raises(B.FMError):
        m.fm_partition_batches(0)
    m.fm_partition_batches(3)
    with pytest.raises(B.FMError):
        m.fm_partition_batches(3)
    m.close()


# ------------------------------------------- small dense shapes, metrics ----

@pytest.mark.parametrize("name,mode", [("regression_513x8", "full"), ("regression_303x13", "stratified"),
                                       ("classification_49990x22", "minibatch")])
def test_small_dense_shapes_train_and_evaluate_like_the_oracle(name, mode):
    """The three small shapes of the paper's data set table (synthetic content): some epochs on the
    training rows, then mean loss, RMSE and accuracy on held-out rows, GPU against oracle."""
    import torch
    from paper_2004_13940_amd.workloads import make_small
    B = _B()
    tr, te = make_small(name)
    X, Xt = (O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val) for wl in (tr, te))
    m = B.Matrix(tr.N, tr.D, tr.rowptr, tr.col, tr.val)
    mt = B.Matrix(te.N, te.D, te.rowptr, te.col, te.val)
    m.fm_build_csc()
    p = B.make_params(tr.K, tr.loss, tr.lambda_w, tr.lambda_v, tr.eta, tr.loss_scale, 1)
    d_w0, d_w, d_V = dev_params(tr.w0, tr.w, tr.V)
    d_y, d_yt = to_dev(tr.y), to_dev(te.y)
    w0, w, V = float(tr.w0), tr.w.astype(np.float64), tr.V.astype(np.float64)
    kw = oracle_kw(tr)
    if mode == "stratified":
        m.fm_partition(tr.P)
    if mode == "minibatch":
        m.fm_partition_batches(10)
    first = None
    for ep in range(8):
        if mode == "full":
            m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V)
            w0, w, V, _ = O.full_epoch(X, tr.y, w0, w, V, **kw)
        elif mode == "stratified":
            m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V)
            w0, w, V, _, _ = O.stratified_epoch(X, tr.y, w0, w, V, P=tr.P, final_objective=False, **kw)
        else:
            m.fm_minibatch_epoch(p, d_y, d_w0, d_w, d_V)
            w0, w, V, _ = O.minibatch_epoch(X, tr.y, w0, w, V, B=10, final_objective=False, **kw)
        got = mt.fm_evaluate(p, d_yt, d_w0, d_w, d_V)
        want = O.evaluate(Xt, te.y, w0, w, V, tr.loss)
        first = first or want
        assert abs(got["mean_loss"] - want["mean_loss"]) <= REL_TOL * want["mean_loss"]
        assert abs(got["rmse"] - want["rmse"]) <= REL_TOL * want["rmse"]
        # a score within rounding of 0 may fall on either side
        assert abs(got["accuracy"] - want["accuracy"]) <= 2.0 / te.N
    _say(f"  {name} ({mode}): test metrics first {first} last {want}")
    assert want["mean_loss"] < first["mean_loss"]
    assert_close(d_V.cpu().numpy().reshape(tr.D, tr.K), V, "V")
    with pytest.raises(B.FMError):  # the evaluation used the aggregate storage of its handle
        mt.fm_get_aux(tr.K, r=torch.empty(te.N, device="cuda"))
    m.close()
    mt.close()


def test_results_are_bit_reproducible():
    import torch
    B = _B()
    wl = make_config(3, scale=0.05)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    m.fm_partition(8)
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, 1)
    y = to_dev(wl.y)
    outs = []
    for _ in range(2):
        w0, w, V = dev_params(wl.w0, wl.w, wl.V)
        m.fm_sgd_epoch(p, y, w0, w, V)
        m.fm_stratified_epoch(p, y, w0, w, V)
        torch.cuda.synchronize()
        outs.append((w0.clone(), w.clone(), V.clone()))
    for x, z in zip(*outs):
        assert torch.equal(x, z)
    m.close()


def test_heavy_columns_through_the_panel_order_and_workgroup_finish():
    """Small knobs force every code path of the column side at a size the oracle handles:
    columns cut at row-panel boundaries and handed out per XCD list, plain segments,
    short columns, and columns summed by a whole workgroup."""
    import torch
    B = _B()

    def small_knobs(m):
        m.fm_set_tuning(seg=16, panel=64, heavy_per_panel=2, vlong=8, min_panels=4)
        m.fm_set_tile_tuning(tile_rows=64, min_per_tile=12, tile_seg=16)

    if True:
        for K, loss in [(16, O.LOSS_LOGISTIC), (8, O.LOSS_SQUARED), (3, O.LOSS_LOGISTIC), (32, O.LOSS_SQUARED)]:
            N, D = 5000, 300
            rng = np.random.default_rng(40 + K)
            dens = np.concatenate([[1.0, 1.0, 0.5, 0.2, 0.1, 0.05], rng.random(D - 6) ** 6 * 0.05])
            mask = rng.random((N, D)) < dens[None, :]
            rowptr = np.zeros(N + 1, np.int64)
            np.cumsum(mask.sum(axis=1), out=rowptr[1:])
            col = np.nonzero(mask)[1].astype(np.int32)
            val = rng.standard_normal(len(col)).astype(np.float32)
            y = (np.where(rng.random(N) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(N)).astype(np.float32)
            w = (rng.standard_normal(D) * 0.1).astype(np.float32)
            V = (rng.standard_normal((D, K)) * 0.1).astype(np.float32)
            from paper_2004_13940_amd.workloads import Workload
            wl = Workload("panels", N, D, K, rowptr, col, val, y, np.float32(0.05), w, V, loss, 1e-3, 2e-3, 0.3,
                          1.0 / N, 3, 4, 1)
            _say("panel path", K, loss, len(col))
            m, p, X, dev, host = _run_full_epochs(B, wl, 3, setup=small_knobs)
            with pytest.raises(B.FMError) as e:  # the decomposition is fixed once the CSC is built
                m.fm_set_tuning(seg=32)
            assert e.value.code == -5
            m.close()


# ----------------------------------------- columns handed on one by one ----

def _run_placed_epochs(B, wl, P, place, epochs, stale):
    """fm_partition_placed + fm_stratified_epoch against the oracle's placed_epoch."""
    import torch
    m, p, X, dev, host = _run_full_epochs(B, wl, 0)
    m.fm_partition_placed(P, place)
    p.stale_aux = int(stale)
    d_w0, d_w, d_V, d_y = dev
    w0, w, V = host
    for ep in range(epochs):
        obj = m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        w0, w, V, wobj, _ = O.placed_epoch(X, wl.y, w0, w, V, P=P, place=place, stale_aux=stale,
                                           update_w0=bool(wl.update_w0), **oracle_kw(wl))
        torch.cuda.synchronize()
        _say(f"  placed epoch {ep} (stale={stale}): objective gpu {sum(obj):.8f} oracle {sum(wobj):.8f}")
        assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0])
        assert abs(obj[1] - wobj[1]) <= REL_TOL * abs(wobj[1]) + 1e-12
        assert_close(d_w.cpu().numpy(), w, f"w after placed epoch {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after placed epoch {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)
    return m, X


@pytest.mark.parametrize("stale", [True, False])
@pytest.mark.parametrize("N,D,P,K", [(300, 40, 4, 8), (97, 23, 7, 3), (2300, 50, 64, 16), (50, 9, 1, 4)])
def test_columns_placed_one_by_one_match_the_oracle(N, D, P, K, stale):
    """Algorithm 1's schedule with a seeded random initial placement of every column: structures bit for bit,
    then two epochs (update phase on stale aggregates, or with the own-row refresh) against the oracle."""
    from paper_2004_13940_amd.workloads import Workload, random_placement
    B = _B()
    rowptr, col, val, y, w0, w, V = _problem(1300 + P + K, N, D, K, 0.15, O.LOSS_LOGISTIC, dense_cols=(2,))
    wl = Workload("placed", N, D, K, rowptr, col, val, y, w0, w, V, O.LOSS_LOGISTIC, 1e-2, 2e-2, 0.5, 1.0 / N, 1, P, 1)
    place = random_placement(D, P, seed=77 + P)
    _say("placed", N, D, P, K, stale, len(col))
    m, X = _run_placed_epochs(B, wl, P, place, 2, stale)
    rb, cb, cells = m.fm_get_block_index()
    assert cb is None
    np.testing.assert_array_equal(rb, O.block_bounds(N, P))
    np.testing.assert_array_equal(cells, O.cell_nnz(X, P, place))
    for s in sorted({0, 1 % P, P - 1}):
        for got, want in ((m.fm_get_stratum_csr(s), O.stratum_csr(X, P, s, place)),
                          (m.fm_get_stratum_csc(s), O.stratum_csc(X, P, s, place))):
            np.testing.assert_array_equal(got[0], want[0])
            np.testing.assert_array_equal(got[1], want[1])
            np.testing.assert_array_equal(got[2], want[2].astype(np.float32))
    m.close()


def test_block_placement_is_the_ring_on_the_gpu_and_a_scaled_workload_runs_placed():
    """place[j] = column block of j must give bit for bit what fm_partition gives; then the text-like
    workload at a tenth of its size with a random placement on P = 32 workers, stale and refreshed."""
    import torch
    from paper_2004_13940_amd.workloads import random_placement
    B = _B()
    wl = make_config(3, scale=0.1)
    outs = []
    for placed in (False, True):
        m, p, X, dev, host = _run_full_epochs(B, wl, 0)
        if placed:
            m.fm_partition_placed(wl.P, O.block_placement(wl.D, wl.P))
        else:
            m.fm_partition(wl.P)
        d_w0, d_w, d_V, d_y = dev
        for stale in (1, 0):
            p.stale_aux = stale
            m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V)
        torch.cuda.synchronize()
        outs.append((d_w0.clone(), d_w.clone(), d_V.clone()))
        m.close()
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    place = random_placement(wl.D, wl.P, seed=5)
    for stale in (True, False):
        m, _ = _run_placed_epochs(B, wl, wl.P, place, 2, stale)
        m.close()
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    with pytest.raises(B.FMError) as e:
        m.fm_partition_placed(4, np.full(wl.D, 4, np.int32))  # worker 4 of 4 does not exist
    assert e.value.code == -4
    m.close()


# ------------------------------------------------------------ error paths ----

def test_state_and_argument_errors_are_reported():
    import torch
    B = _B()
    rowptr, col, val, y, w0, w, V = _problem(5, 20, 10, 4, 0.3, O.LOSS_SQUARED)
    m = B.Matrix(20, 10, rowptr, col, val)
    p = B.make_params(4, 0, 0.0, 0.0, 0.1)
    d_w0, d_w, d_V = dev_params(w0, w, V)
    d_y = to_dev(y)
    r, G = torch.zeros(20, device="cuda"), torch.zeros(80, device="cuda")
    with pytest.raises(B.FMError) as e:
        m.fm_gradient(p, r, G, d_w, d_V, None, torch.zeros(10, device="cuda"), None)
    assert e.value.code == -5
    with pytest.raises(B.FMError) as e:
        m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V)
    assert e.value.code == -5
    m.fm_build_csc()
    with pytest.raises(B.FMError) as e:
        m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V)
    assert e.value.code == -5
    with pytest.raises(B.FMError) as e:
        m.fm_partition(0)
    assert e.value.code == -1
    bad = B.make_params(65, 0, 0.0, 0.0, 0.1)  # K = 65 is neither <= 64 nor a multiple of 4
    with pytest.raises(B.FMError) as e:
        load = B.load()
        m._check(load.fm_forward(m._h, __import__("ctypes").byref(bad), None, B._vp(d_w0), B._vp(d_w), B._vp(d_V),
                                 None, None, None, None, None, None, None))
    assert e.value.code == -1
    m.fm_partition(2)
    with pytest.raises(B.FMError) as e:
        m.fm_stratified_step(p, 0, d_y, d_w0, d_w, d_V)  # no begin yet
    assert e.value.code == -5
    # arrays with K floats per row must be 16-byte aligned: a view that starts one float into a buffer is refused
    skew = torch.zeros(41, device="cuda")[1:]
    assert skew.data_ptr() % 16 == 4
    for call in (lambda: m.fm_forward(p, d_y, d_w0, d_w, skew),
                 lambda: m.fm_forward(p, d_y, d_w0, d_w, d_V, G=torch.zeros(81, device="cuda")[1:]),
                 lambda: m.fm_sgd_epoch(p, d_y, d_w0, d_w, skew),
                 lambda: m.fm_gradient(p, r, G, d_w, d_V, None, None, skew),
                 lambda: m.fm_forward_noalloc(p, d_y, d_w0, d_w, skew)):
        with pytest.raises(B.FMError) as e:
            call()
        assert e.value.code == B.FM_EINVAL and "aligned" in str(e.value)
    m.close()


def test_bench_probes_report_plausible_figures_and_reject_bad_arguments():
    """The calibration probes of bench.py live in a library of their own (not in the product ABI)."""
    import torch
    from paper_2004_13940_amd import bench_probe as P
    rate = P.gather_rate(64 << 20, 128)
    assert 1e9 < rate < 1e12
    with pytest.raises(RuntimeError):
        P.gather_rate(64 << 20, 96)
    with pytest.raises(RuntimeError):
        P.gather_rate(1000, 64)
    src = torch.arange(1 << 20, dtype=torch.float32, device="cuda")
    dst = torch.zeros_like(src)
    P.copy(src, dst, reps=2)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)
    assert not hasattr(_B().load(), "fm_probe_gather")


@pytest.mark.parametrize("options", [
    {"FM_OPT_AUX_PLANAR": 1},
    {"FM_OPT_SIDE_STREAMS": 0},
    {"FM_OPT_LAZY_REG": 0},
    {"FM_OPT_GRAPH": 2},
    {"FM_OPT_GRAPH": 0},
    {"FM_OPT_AUX_PLANAR": 1, "FM_OPT_SIDE_STREAMS": 0, "FM_OPT_LAZY_REG": 0, "FM_OPT_GRAPH": 2},
])
@pytest.mark.parametrize("idx,scale", [(3, 0.1), (4, 0.002)])
def test_every_option_gives_the_oracle_result(options, idx, scale):
    """Each per-handle switch (planar aggregates at K=16, one stream only, immediate regulariser steps,
    stratified epoch always or never from a graph) through full-gradient, stratified and mini-batch epochs."""
    B = _B()
    wl = make_config(idx, scale=scale)
    _say("options", options, wl.name, wl.N, wl.D, wl.nnz)

    def setup(m):
        for name, value in options.items():
            m.fm_set_option(getattr(B, name), value)

    m, p, X, dev, host = _run_full_epochs(B, wl, 2, setup=setup)
    m.fm_partition(wl.P)
    host = _run_stratified_epochs(B, wl, m, p, X, dev, host, 2)
    # switching the aggregate layout on a live handle: the next pass allocates the other layout
    if "FM_OPT_AUX_PLANAR" in options:
        m.fm_set_option(B.FM_OPT_AUX_PLANAR, 0)
        host = _run_stratified_epochs(B, wl, m, p, X, dev, host, 1)
    m.close()
    m2, _, _ = _run_minibatch_epochs(B, wl, 5, 1, update_w0=bool(wl.update_w0), setup=setup)
    m2.close()
    with pytest.raises(B.FMError):
        B.Matrix(1, 1, np.array([0, 0]), np.array([], np.int32), np.array([], np.float32)).fm_set_option(99, 1)


def test_random_shapes_through_every_epoch_kind():
    """Seeded sweep over shapes, latent sizes (every lane layout, packed and planar aggregates), losses,
    partitions and flags: one epoch of each kind against the oracle."""
    import torch
    from paper_2004_13940_amd.workloads import Workload
    B = _B()
    rng = np.random.default_rng(20241127)
    Ks = [1, 2, 3, 4, 6, 7, 8, 12, 16, 24, 28, 32, 36, 48, 64, 128]
    for case in range(32):
        K = int(Ks[case % len(Ks)])
        N = int(rng.integers(40, 900))
        D = int(rng.integers(5, 120))
        dens = float(rng.uniform(0.03, 0.5))
        loss = int(rng.integers(0, 2))
        P = int(rng.integers(1, 10))
        nb = int(rng.integers(1, 10))
        dense = tuple(int(c) for c in rng.choice(D, size=int(rng.integers(0, 3)), replace=False))
        rowptr, col, val, y, w0, w, V = _problem(7000 + case, N, D, K, dens, loss, dense_cols=dense)
        V *= np.float32(0.3)
        if loss == O.LOSS_SQUARED:
            y = (y * 0.5).astype(np.float32)
        wl = Workload("rnd", N, D, K, rowptr, col, val, y, w0, w, V, loss, float(rng.uniform(0, 0.05)),
                      float(rng.uniform(0, 0.05)), 0.1, 1.0 / N, 1, P, int(rng.integers(0, 2)))
        flags = {}
        if rng.random() < 0.3:
            flags["reg_full_per_cell"] = True
        mode = rng.integers(0, 3)
        if mode == 1:
            flags["refresh_all_rows"] = True
        elif mode == 2:
            flags["stale_aux"] = True
        _say(f"case {case}: N={N} D={D} K={K} nnz={len(col)} loss={loss} P={P} B={nb} dense={dense} flags={flags}")
        m, p, X, dev, host = _run_full_epochs(B, wl, 1)
        m.fm_partition(P)
        host = _run_stratified_epochs(B, wl, m, p, X, dev, host, 1, **flags)
        m.close()
        for k in flags:
            setattr(p, k, 0)
        m2, _, _ = _run_minibatch_epochs(B, wl, nb, 1, full_reg=bool(flags.get("reg_full_per_cell")),
                                         update_w0=bool(wl.update_w0))
        m2.close()
    torch.cuda.synchronize()


def test_replayed_stratified_epochs_stay_correct_between_other_work():
    """With P >= 16 and small strata fm_stratified_epoch is captured once per set of arguments and
    replayed; every replay is checked against the oracle, with other calls of the library (another
    handle's epoch, a forward of this handle, a synchronisation) between the replays."""
    import torch
    B = _B()
    wl = make_config(3, scale=0.1)
    other = make_config(1)
    mo = B.Matrix(other.N, other.D, other.rowptr, other.col, other.val)
    mo.fm_build_csc()
    po = B.make_params(other.K, other.loss, other.lambda_w, other.lambda_v, other.eta, other.loss_scale, 0)
    o0, ow, oV = dev_params(other.w0, other.w, other.V)
    oy = to_dev(other.y)
    X = O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    m.fm_partition(wl.P)
    assert wl.P >= 16
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, 1)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    yhat = torch.empty(wl.N, device="cuda")
    w0, w, V = float(wl.w0), wl.w.astype(np.float64), wl.V.astype(np.float64)
    kw = oracle_kw(wl)
    for ep in range(5):
        m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V)  # first call captures, the others replay
        w0, w, V, _, _ = O.stratified_epoch(X, wl.y, w0, w, V, P=wl.P, final_objective=False, **kw)
        mo.fm_sgd_epoch(po, oy, o0, ow, oV)
        m.fm_forward(p, d_y, d_w0, d_w, d_V, yhat=yhat)
        torch.cuda.synchronize()
        assert_close(d_w.cpu().numpy(), w, f"w after replay {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after replay {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)
        _, _, _, want = O.forward(X, w0, w, V)
        assert_close(yhat.cpu().numpy(), want, f"scores after replay {ep}")
    # new arrays: a new capture
    e_w0, e_w, e_V = dev_params(wl.w0, wl.w, wl.V)
    m.fm_stratified_epoch(p, d_y, e_w0, e_w, e_V)
    w0b, wb, Vb, _, _ = O.stratified_epoch(X, wl.y, float(wl.w0), wl.w, wl.V, P=wl.P, final_objective=False, **kw)
    assert_close(e_V.cpu().numpy().reshape(wl.D, wl.K), Vb, "V with new arrays")
    m.close()
    mo.close()


# ------------------------------------- half-precision copy of V for the gathers ----

def _round16(V):
    """What the library's copy holds: the fp32 factors rounded to IEEE half precision (nearest even)."""
    return np.asarray(V, np.float32).astype(np.float16).astype(np.float64)


@pytest.mark.parametrize("K,loss", [(4, O.LOSS_SQUARED), (16, O.LOSS_LOGISTIC), (64, O.LOSS_LOGISTIC), (128, O.LOSS_SQUARED)])
def test_half_gather_scores_the_model_with_rounded_factors(K, loss):
    """half_gather: the forward gathers V rows from a half-precision copy.  Both sides take the rounding in the
    same precision (binary16, nearest even), so the usual 1e-4 applies; the deviation from the unrounded model
    is printed for information.  The gradient and the step keep the fp32 factors."""
    import torch
    B = _B()
    N, D = 700, 90
    rowptr, col, val, y, w0, w, V = _problem(1700 + K, N, D, K, 0.15, loss, dense_cols=(1,))
    V = (V * (3 if K <= 16 else 0.5)).astype(np.float32)  # a spread of magnitudes, some below the smallest normal half
    V[::7] *= np.float32(1e-4)
    X = O.make_matrix(N, D, rowptr, col, val)
    m = B.Matrix(N, D, rowptr, col, val)
    m.fm_build_csc()
    s = 1.0 / N
    p = B.make_params(K, loss, 1e-2, 2e-2, 0.3, s, 1, half_gather=1)
    d_w0, d_w, d_V = dev_params(w0, w, V)
    d_y = to_dev(y)
    out = {k: torch.empty(n, device="cuda") for k, n in (("yhat", N), ("a", N), ("G", N * K), ("q", N), ("r", N))}
    got_loss = m.fm_forward(p, d_y, d_w0, d_w, d_V, want_loss=True, **out)
    a, G, q, yh = O.forward(X, float(w0), w, _round16(V))
    l, r = O.loss_multiplier(loss, s, yh, y)
    for k, want in (("yhat", yh), ("a", a), ("G", G), ("q", q), ("r", r)):
        assert_close(out[k].cpu().numpy().reshape(want.shape), want, f"{k} with rounded factors")
    assert abs(got_loss - l.sum()) <= REL_TOL * l.sum()
    _, _, _, yh_full = O.forward(X, float(w0), w, V)
    _say(f"  K={K}: yhat deviates from the unrounded model by {np.abs(yh - yh_full).max() / np.abs(yh_full).max():.2e} "
         f"of its largest entry")
    ev = m.fm_evaluate(p, d_y, d_w0, d_w, d_V)
    assert abs(ev["mean_loss"] - O.loss_multiplier(loss, 1.0, yh, y)[0].mean()) <= REL_TOL * abs(ev["mean_loss"]) + 1e-12
    # full-gradient epochs: forward on the rounded copy, gradient and step on the fp32 factors
    ow0, ow, oV = float(w0), w.astype(np.float64), V.astype(np.float64)
    for ep in range(3):
        obj = m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        a, G, q, yh = O.forward(X, ow0, ow, _round16(oV))
        l, r = O.loss_multiplier(loss, s, yh, y)
        gw0, gw, gV = O.gradient(X, r, G, ow, oV, 1e-2, 2e-2)
        assert abs(obj[0] - s * l.sum()) <= REL_TOL * s * l.sum()
        ow0, ow, oV = ow0 - 0.3 * gw0, ow - 0.3 * gw, oV - 0.3 * gV
        assert_close(d_w.cpu().numpy(), ow, f"w after epoch {ep} with half gathers")
        assert_close(d_V.cpu().numpy().reshape(D, K), oV, f"V after epoch {ep} with half gathers")
        assert abs(d_w0.item() - ow0) <= REL_TOL * max(abs(ow0), 1e-3)
    # mini-batch epoch: every batch scores its rows with the factors as they stand, rounded
    nb = 4
    m.fm_partition_batches(nb)
    m.fm_minibatch_epoch(p, d_y, d_w0, d_w, d_V)
    rb = O.block_bounds(N, nb)
    yd = y.astype(np.float64)
    rr = np.zeros(N)
    dw, dV, dn = np.zeros(D), np.zeros((D, K)), np.zeros(D)
    ow, oV = ow.copy(), oV.copy()
    for b in range(nb):
        lo, hi = int(rb[b]), int(rb[b + 1])
        a, G, q, _ = O.forward(X, ow0, ow, _round16(oV))
        O.cell_update(X, yd, ow0, ow, oV, a, G, q, rr, (lo, hi), (0, D), loss=loss, s=s, eta=0.3, rho=(hi - lo) / N,
                      lambda_w=1e-2, lambda_v=2e-2, dw=dw, dV=dV, dn=dn)
        ow0 = ow0 - 0.3 * float(rr[lo:hi].sum())
    assert_close(d_w.cpu().numpy(), ow, "w after a mini-batch epoch with half gathers")
    assert_close(d_V.cpu().numpy().reshape(D, K), oV, "V after a mini-batch epoch with half gathers")
    # where the mode does not apply
    m.fm_partition(2)
    with pytest.raises(B.FMError) as e:
        m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V)
    assert e.value.code == -1
    with pytest.raises(B.FMError) as e:
        m.fm_forward_noalloc(p, d_y, d_w0, d_w, d_V, yhat=out["yhat"])
    assert e.value.code == -1
    m.close()


def test_half_gather_needs_a_latent_size_that_is_a_multiple_of_four():
    B = _B()
    rowptr, col, val, y, w0, w, V = _problem(9, 30, 12, 6, 0.3, O.LOSS_SQUARED)
    m = B.Matrix(30, 12, rowptr, col, val)
    p = B.make_params(6, O.LOSS_SQUARED, 0.0, 0.0, 0.1, half_gather=1)
    d_w0, d_w, d_V = dev_params(w0, w, V)
    with pytest.raises(B.FMError) as e:
        m.fm_forward(p, to_dev(y), d_w0, d_w, d_V)
    assert e.value.code == -1
    m.close()


# ----------------------------------------------- many blocks, one example per step ----

@pytest.mark.parametrize("N,D,K,loss", [(1007, 64, 32, O.LOSS_SQUARED), (70, 32, 32, O.LOSS_LOGISTIC),
                                        (5003, 32, 64, O.LOSS_LOGISTIC), (9001, 64, 64, O.LOSS_SQUARED)])
def test_matrices_that_store_every_column_take_the_dense_kernels(N, D, K, loss):
    """Every row stores all D columns: forward, gradient and epochs run on the matrix cores by default
    and on the sparse kernels when the handle says so; both meet the oracle, and they are two paths
    (their results differ in the last bits)."""
    import torch
    from types import SimpleNamespace
    B = _B()
    rng = np.random.default_rng(4000 + N + D + K)
    val = (rng.standard_normal(N * D) * 0.5).astype(np.float32)
    val[rng.random(N * D) < 0.05] = 0.0  # stored zeros
    rowptr = np.arange(N + 1, dtype=np.int64) * D
    col = np.tile(np.arange(D, dtype=np.int32), N)
    y = (np.where(rng.random(N) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(N)).astype(np.float32)
    w0 = np.float32(0.3)
    w = (rng.standard_normal(D) * 0.1).astype(np.float32)
    V = (rng.standard_normal((D, K)) * 0.1).astype(np.float32)
    X = O.make_matrix(N, D, rowptr, col, val)
    s = 1.0 / N
    a, G, q, yhat = O.forward(X, float(w0), w, V)
    l, r = O.loss_multiplier(loss, s, yhat, y)
    want = dict(yhat=yhat, a=a, G=G, q=q, r=r)
    got_G = {}
    for dense in (1, 0):
        _say("dense rows", N, D, K, loss, "matrix cores" if dense else "sparse kernels")
        m = B.Matrix(N, D, rowptr, col, val)
        m.fm_set_option(B.FM_OPT_DENSE_ROWS, dense)
        p = B.make_params(K, loss, 0.01, 0.02, 0.1, loss_scale=s)
        d_w0, d_w, d_V = dev_params(w0, w, V)
        d_y = to_dev(y)
        out = {k: torch.full((N * (K if k == "G" else 1),), float("nan"), device="cuda") for k in want}
        loss_sum = m.fm_forward(p, d_y, d_w0, d_w, d_V, want_loss=True, **out)
        torch.cuda.synchronize()
        for k in want:
            assert_close(out[k].cpu().numpy(), want[k], f"{k} dense={dense}")
        assert abs(loss_sum - float(l.sum())) <= REL_TOL * abs(float(l.sum()))
        # (G itself can agree bit for bit: both paths add the products of a row in column order)
        got_G[dense] = np.concatenate([out[k].cpu().numpy() for k in ("a", "q", "yhat")])
        # the evaluation pass takes the same kernels
        met = m.fm_evaluate(p, d_y, d_w0, d_w, d_V)
        l1, _ = O.loss_multiplier(loss, 1.0, yhat, y)
        assert abs(met["mean_loss"] - l1.mean()) <= REL_TOL * l1.mean()
        assert abs(met["rmse"] - np.sqrt(np.mean((yhat - y) ** 2))) <= REL_TOL * np.sqrt(np.mean((yhat - y) ** 2))
        m.fm_build_csc()
        g0 = torch.zeros(1, device="cuda")
        gw = torch.full((D,), float("nan"), device="cuda")
        gV = torch.full((D * K,), float("nan"), device="cuda")
        m.fm_gradient(p, out["r"], out["G"], d_w, d_V, g0, gw, gV)
        torch.cuda.synchronize()
        wg0, wgw, wgV = O.gradient(X, r, G, w, V, p.lambda_w, p.lambda_v)
        assert_close(gw.cpu().numpy(), wgw, f"grad_w dense={dense}")
        assert_close(gV.cpu().numpy(), wgV, f"grad_V dense={dense}")
        wl = SimpleNamespace(N=N, D=D, K=K, rowptr=rowptr, col=col, val=val, y=y, w0=w0, w=w, V=V, loss=loss,
                             lambda_w=0.01, lambda_v=0.02, eta=0.1, loss_scale=s, update_w0=1)
        _run_full_epochs(B, wl, 3, m=m)
        m.close()
    assert not np.array_equal(got_G[0], got_G[1]), "the two settings ran the same kernels"


def test_per_example_steps_of_the_tiny_workload():
    """B = N: every step of the mini-batch epoch takes one example (Section 4.1's stochastic updates as printed),
    2,000 steps per epoch, against the oracle."""
    B = _B()
    wl = make_config(1)
    m, _, _ = _run_minibatch_epochs(B, wl, wl.N, 1, update_w0=bool(wl.update_w0))
    m.close()


def test_more_blocks_than_the_cell_table_holds():
    """P = 6,000 row and column blocks (most column blocks empty, one or two rows per row block): the structures
    add up, the cell table is refused, and an epoch on stale aggregates without regulariser moves w exactly as the
    full-gradient step does (the closed form that pins the oracle's stale epoch, whatever P is)."""
    import torch
    from paper_2004_13940_amd.workloads import Workload
    B = _B()
    N, D, K, P = 7000, 60, 4, 6000
    rowptr, col, val, y, w0, w, V = _problem(321, N, D, K, 0.1, O.LOSS_LOGISTIC)
    wl = Workload("manyblocks", N, D, K, rowptr, col, val, y, w0, w, V, O.LOSS_LOGISTIC, 0.0, 0.0, 0.3, 1.0 / N, 1, P, 1)
    m, p, X, dev, host = _run_full_epochs(B, wl, 0)
    m.fm_partition(P)
    rb, cb, _ = (np.empty(P + 1, np.int64), np.empty(P + 1, np.int64), None)
    m._check(B.load().fm_get_block_index(m._h, B._vp(rb), B._vp(cb), B._vp(None)))
    np.testing.assert_array_equal(rb, O.block_bounds(N, P))
    np.testing.assert_array_equal(cb, O.block_bounds(D, P))
    with pytest.raises(B.FMError) as e:
        m.fm_get_block_index()
    assert e.value.code == -5
    assert sum(m.fm_get_stratum_nnz(s) for s in range(0, P, 97)) <= len(col)
    got = m.fm_get_stratum_csc(0)
    want = O.stratum_csc(X, P, 0)
    for g, wv in zip(got, want):
        np.testing.assert_array_equal(g, wv.astype(g.dtype))
    d_w0, d_w, d_V, d_y = dev
    p.stale_aux = 1
    m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V)
    torch.cuda.synchronize()
    ow0, ow, _, _ = O.full_epoch(X, y, float(w0), w, V, update_w0=True, **oracle_kw(wl))
    assert_close(d_w.cpu().numpy(), ow, "w after a stale epoch over 6,000 strata")
    assert abs(d_w0.item() - ow0) <= REL_TOL * max(abs(ow0), 1e-3)
    m.close()
