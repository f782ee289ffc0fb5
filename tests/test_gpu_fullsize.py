"""Parity at the full size of the benchmarked workload (config 4: N=1e7, D=1e6, 39 nnz/row,
K=16), in the launch configuration bench.py times.  The C oracle is fast enough to redo a
whole full-gradient epoch at this size, so every output is compared; the stratified step
is compared on three sampled cells of stratum 0 plus an exactness property."""
import numpy as np
import pytest

from oracle import fm_oracle as O
from paper_2004_13940_amd.workloads import make_config

from helpers import REL_TOL, assert_close, dev_params, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]


def _say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module")
def full():
    import torch
    from paper_2004_13940_amd import binding as B
    wl = make_config(4)
    _say("generated", wl.name, wl.N, wl.D, wl.nnz)
    m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    m.fm_build_csc()
    X = O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    _say("oracle matrix ready")
    yield wl, m, X, B
    m.close()
    torch.cuda.empty_cache()


def test_full_size_forward_and_full_gradient_epoch(full):
    import torch
    wl, m, X, B = full
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    yhat = torch.empty(wl.N, device="cuda")
    loss = m.fm_forward(p, d_y, d_w0, d_w, d_V, yhat=yhat, want_loss=True)
    a, G, q, want_yhat = O.forward(X, float(wl.w0), wl.w, wl.V)
    l, r = O.loss_multiplier(wl.loss, wl.loss_scale, want_yhat, wl.y)
    assert_close(yhat.cpu().numpy(), want_yhat, "yhat at full size")
    assert abs(loss - l.sum()) <= REL_TOL * l.sum()
    del a, G, q, l, r
    w0, w, V = float(wl.w0), wl.w.astype(np.float64), wl.V.astype(np.float64)
    kw = dict(loss=wl.loss, s=wl.loss_scale, lambda_w=wl.lambda_w, lambda_v=wl.lambda_v, eta=wl.eta,
              update_w0=bool(wl.update_w0))
    for ep in range(2):
        obj = m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        w0, w, V, wobj = O.full_epoch(X, wl.y, w0, w, V, **kw)
        _say(f"full-size epoch {ep}: objective gpu {sum(obj):.8f} oracle {sum(wobj):.8f}")
        assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0])
        assert abs(obj[1] - wobj[1]) <= REL_TOL * abs(wobj[1]) + 1e-12
        assert_close(d_w.cpu().numpy(), w, f"w after full-size epoch {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after full-size epoch {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)


def test_full_size_stratum_on_sampled_cells(full):
    import torch
    wl, m, X, B = full
    P = wl.P
    m.fm_partition(P)
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    m.fm_stratified_begin(p, d_y, d_w0, d_w, d_V)
    m.fm_stratified_step(p, 0, d_y, d_w0, d_w, d_V)
    ga, gG, gq, gr = (torch.empty(n, device="cuda") for n in (wl.N, wl.N * wl.K, wl.N, wl.N))
    m.fm_get_aux(wl.K, ga, gG, gq, gr)
    torch.cuda.synchronize()
    rb, cb = O.block_bounds(wl.N, P), O.block_bounds(wl.D, P)
    y = wl.y.astype(np.float64)
    w, V = wl.w.astype(np.float64), wl.V.astype(np.float64)
    a, G, q, _ = O.forward(X, float(wl.w0), w, V)
    r = np.zeros(wl.N)
    dw, dV, dn = np.zeros(wl.D), np.zeros((wl.D, wl.K)), np.zeros(wl.D)
    gw, gV = d_w.cpu().numpy(), d_V.cpu().numpy().reshape(wl.D, wl.K)
    gG2 = gG.cpu().numpy().reshape(wl.N, wl.K)
    for c in (0, 1, 17, P - 1):  # stratum 0 holds the diagonal cells (c, c); cell 0 has the 13 dense columns
        rows, cols = (rb[c], rb[c + 1]), (cb[c], cb[c + 1])
        rho = (rows[1] - rows[0]) / wl.N
        O.cell_update(X, y, float(wl.w0), w, V, a, G, q, r, rows, cols, loss=wl.loss, s=wl.loss_scale, eta=wl.eta,
                      rho=rho, lambda_w=wl.lambda_w, lambda_v=wl.lambda_v, dw=dw, dV=dV, dn=dn)
        O.refresh(X, a, G, q, rows, cols, dw, dV, dn)
        I, J = slice(*rows), slice(*cols)
        _say("cell", c, "rows", rows, "cols", cols)
        assert_close(gw[J], w[J], f"w of column block {c}")
        assert_close(gV[J], V[J], f"V of column block {c}")
        assert_close(gG2[I], G[I], f"G of row block {c}")
        assert_close(ga.cpu().numpy()[I], a[I], f"a of row block {c}")
        assert_close(gq.cpu().numpy()[I], q[I], f"q of row block {c}")
        want_r = O.multiplier_from_aux(wl.loss, wl.loss_scale, float(wl.w0), a[I], G[I], q[I], y[I])
        assert_close(gr.cpu().numpy()[I], want_r, f"r of row block {c}")
    # property at any size: a whole stratified epoch followed by the objective pass leaves
    # aggregates that equal a fresh forward at the final parameters
    obj = m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
    m.fm_get_aux(wl.K, ga, gG, gq, gr)
    torch.cuda.synchronize()
    fa, fG, fq, fy = O.forward(X, d_w0.item(), d_w.cpu().numpy(), d_V.cpu().numpy().reshape(wl.D, wl.K))
    fl, _ = O.loss_multiplier(wl.loss, wl.loss_scale, fy, wl.y)
    assert_close(gG.cpu().numpy().reshape(wl.N, wl.K), fG, "G after the epoch")
    assert_close(ga.cpu().numpy(), fa, "a after the epoch")
    assert abs(obj[0] - wl.loss_scale * fl.sum()) <= REL_TOL * wl.loss_scale * fl.sum()
    assert np.isfinite(sum(obj)) and sum(obj) < np.log(2.0)  # the epoch made progress from the start value


def test_full_size_minibatch_epoch_and_gradient_entry_point(full):
    """Three row batches at full size: every output against the oracle; then fm_gradient (which packs
    the caller's r, G into aggregate rows first) on a sample of columns of each class."""
    import torch
    wl, m, X, B = full
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    nb = 3
    m.fm_partition_batches(nb)
    obj = m.fm_minibatch_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
    kw = dict(loss=wl.loss, s=wl.loss_scale, lambda_w=wl.lambda_w, lambda_v=wl.lambda_v, eta=wl.eta,
              update_w0=bool(wl.update_w0))
    w0, w, V, wobj = O.minibatch_epoch(X, wl.y, float(wl.w0), wl.w, wl.V, B=nb, **kw)
    _say(f"full-size mini-batch epoch: objective gpu {sum(obj):.8f} oracle {sum(wobj):.8f}")
    assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0])
    assert_close(d_w.cpu().numpy(), w, "w after the full-size mini-batch epoch")
    assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, "V after the full-size mini-batch epoch")
    assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)
    # gradient entry point at the new parameters
    a, G, q, yh = O.forward(X, w0, w, V)
    _, r = O.loss_multiplier(wl.loss, wl.loss_scale, yh, wl.y)
    r32, G32, w32, V32 = (x.astype(np.float32) for x in (r, G, w, V))  # the same inputs on both sides
    gw0, gw, gV = O.gradient(X, r32, G32, w32, V32, wl.lambda_w, wl.lambda_v)
    del a, q, yh, r, G
    o_w0, o_w, o_V = torch.empty(1, device="cuda"), torch.empty(wl.D, device="cuda"), torch.empty(wl.D * wl.K, device="cuda")
    m.fm_gradient(p, to_dev(r32), to_dev(G32.reshape(-1)), to_dev(w32), to_dev(V32.reshape(-1)), o_w0, o_w, o_V)
    assert_close(o_w.cpu().numpy(), gw, "grad_w at full size")
    assert_close(o_V.cpu().numpy().reshape(wl.D, wl.K), gV, "grad_V at full size")
    assert abs(o_w0.item() - gw0) <= REL_TOL * max(abs(gw0), 1e-6)
