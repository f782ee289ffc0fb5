"""Parity at the full shapes of the workloads, in the launch configuration bench.py times.

Config 4 (N=1e7, D=1e6, 39 entries per row, K=16: the benchmarked one), config 2 (dense, K=32), config 3
(text-like, K=16) and config 5 (N=2e6, D=2e7, K=64) all run at scale 1.0.  The C oracle is fast enough to
redo whole full-gradient epochs at these sizes, and whole stratified epochs for configs 2 and 3; for configs
4 and 5 a stratified step is compared on sampled cells of stratum 0, plus a property that holds at any size
(after an epoch with its objective pass the aggregates equal a fresh forward at the final parameters).

Besides the per-array figure (largest error over largest entry) the gradients and the first step are judged
element by element against what fp32 can resolve (helpers.assert_elementwise), so that the many short
columns, whose entries are orders of magnitude below the array's largest, count too."""
import time

import numpy as np
import pytest

from oracle import fm_oracle as O
from paper_2004_13940_amd.workloads import make_config

from helpers import (REL_TOL, assert_close, assert_elementwise, dev_params, gradient_term_sums, oracle_kw,
                     run_full_epochs, run_stratified_epochs, to_dev)

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]


def _say(*a):
    print(*a, flush=True)


def _host_ram_gib():
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable"):
                return int(line.split()[1]) / 2 ** 20
    except OSError:
        pass
    return float("nan")


def _params(B, wl):
    return B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)


def _check_gradient_entry_point(B, wl, m, X, w0, w, V):
    """fm_gradient on the same fp32 r, G, w, V on both sides: per array and element by element."""
    import torch
    p = _params(B, wl)
    a, G, q, yh = O.forward(X, w0, w, V)
    _, r = O.loss_multiplier(wl.loss, wl.loss_scale, yh, wl.y)
    r32, G32, w32, V32 = (np.asarray(x, np.float32) for x in (r, G, w, V))
    del a, q, yh, r, G
    gw0, gw, gV = O.gradient(X, r32, G32, w32, V32, wl.lambda_w, wl.lambda_v)
    tw, tV = gradient_term_sums(X, r32, G32, w32, V32, wl.lambda_w, wl.lambda_v)
    o_w0, o_w, o_V = (torch.empty(n, device="cuda") for n in (1, wl.D, wl.D * wl.K))
    m.fm_gradient(p, to_dev(r32), to_dev(G32.reshape(-1)), to_dev(w32), to_dev(V32.reshape(-1)), o_w0, o_w, o_V)
    torch.cuda.synchronize()
    assert_close(o_w.cpu().numpy(), gw, "grad_w at full size")
    assert_close(o_V.cpu().numpy().reshape(wl.D, wl.K), gV, "grad_V at full size")
    assert abs(o_w0.item() - gw0) <= REL_TOL * max(abs(gw0), float(np.abs(r32).sum()) * 1e-3, 1e-30)
    assert_elementwise(o_w.cpu().numpy(), gw, tw, "grad_w")
    assert_elementwise(o_V.cpu().numpy().reshape(wl.D, wl.K), gV, tV, "grad_V")


def _check_first_epoch_elementwise(B, wl, m, X):
    """One full-gradient epoch from the initial point on both sides; w and V element by element.  The step is
    eta times the gradient, so the part of the bound that fp32 sums cannot resolve is eta sum|terms|; twice
    ELEM_C there, because the multipliers and aggregates the library sums come from its own fp32 forward."""
    import torch
    from helpers import ELEM_C
    p = _params(B, wl)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V)
    torch.cuda.synchronize()
    a, G, q, yh = O.forward(X, float(wl.w0), wl.w, wl.V)
    _, r = O.loss_multiplier(wl.loss, wl.loss_scale, yh, wl.y)
    tw, tV = gradient_term_sums(X, r, G, wl.w, wl.V, wl.lambda_w, wl.lambda_v)
    del a, q, yh
    w0, w, V, _ = O.full_epoch(X, wl.y, float(wl.w0), wl.w, wl.V, update_w0=bool(wl.update_w0), **oracle_kw(wl))
    # (the rounding of the old value itself, 2^-24 of it, is far inside REL_TOL |want|)
    assert_elementwise(d_w.cpu().numpy(), w, wl.eta * tw, "w after one epoch", c=2 * ELEM_C)
    assert_elementwise(d_V.cpu().numpy().reshape(wl.D, wl.K), V, wl.eta * tV, "V after one epoch", c=2 * ELEM_C)


def _check_stratum0_cells(B, wl, m, X, cells):
    """fm_stratified_begin + step 0 on the library; the oracle takes the step of the sampled diagonal cells
    only (cells of a stratum touch disjoint rows and columns)."""
    import torch
    P = wl.P
    p = _params(B, wl)
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
    ha, hq, hr = ga.cpu().numpy(), gq.cpu().numpy(), gr.cpu().numpy()
    for c in cells:  # stratum 0 holds the diagonal cells (c, c)
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
        assert_close(ha[I], a[I], f"a of row block {c}")
        assert_close(hq[I], q[I], f"q of row block {c}")
        want_r = O.multiplier_from_aux(wl.loss, wl.loss_scale, float(wl.w0), a[I], G[I], q[I], y[I])
        assert_close(hr[I], want_r, f"r of row block {c}")
    return p, (d_w0, d_w, d_V, d_y), (ga, gG, gq, gr)


def _check_epoch_property(wl, m, X, p, dev, aux):
    """A whole stratified epoch followed by the objective pass leaves aggregates that equal a fresh forward at
    the final parameters, and the reported data term is the oracle's loss there."""
    import torch
    d_w0, d_w, d_V, d_y = dev
    ga, gG, gq, gr = aux
    obj = m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
    m.fm_get_aux(wl.K, ga, gG, gq, gr)
    torch.cuda.synchronize()
    fa, fG, fq, fy = O.forward(X, d_w0.item(), d_w.cpu().numpy(), d_V.cpu().numpy().reshape(wl.D, wl.K))
    fl, _ = O.loss_multiplier(wl.loss, wl.loss_scale, fy, wl.y)
    assert_close(gG.cpu().numpy().reshape(wl.N, wl.K), fG, "G after the epoch")
    assert_close(ga.cpu().numpy(), fa, "a after the epoch")
    assert_close(gq.cpu().numpy(), fq, "q after the epoch")
    assert abs(obj[0] - wl.loss_scale * fl.sum()) <= REL_TOL * wl.loss_scale * fl.sum()
    return obj


# ------------------------------------------------------------------ config 4 ----

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
    p = _params(B, wl)
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
    kw = dict(update_w0=bool(wl.update_w0), **oracle_kw(wl))
    for ep in range(2):
        obj = m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        w0, w, V, wobj = O.full_epoch(X, wl.y, w0, w, V, **kw)
        _say(f"full-size epoch {ep}: objective gpu {sum(obj):.8f} oracle {sum(wobj):.8f}")
        assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0])
        assert abs(obj[1] - wobj[1]) <= REL_TOL * abs(wobj[1]) + 1e-12
        assert_close(d_w.cpu().numpy(), w, f"w after full-size epoch {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after full-size epoch {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)


def test_full_size_epoch_with_half_precision_gathers(full):
    """half_gather at the benchmarked shape: the forward on V rounded to binary16 on both sides, gradient and step on
    the fp32 factors; the deviation of the scores from the unrounded model is printed for information."""
    import torch
    wl, m, X, B = full
    p = _params(B, wl)
    p.half_gather = 1
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    yhat = torch.empty(wl.N, device="cuda")
    m.fm_forward(p, d_y, d_w0, d_w, d_V, yhat=yhat)
    V16 = wl.V.astype(np.float16).astype(np.float64)
    a, G, q, yh = O.forward(X, float(wl.w0), wl.w, V16)
    assert_close(yhat.cpu().numpy(), yh, "yhat with rounded factors at full size")
    _, _, _, yh_full = O.forward(X, float(wl.w0), wl.w, wl.V)
    _say(f"scores deviate from the unrounded model by {np.abs(yh - yh_full).max() / np.abs(yh_full).max():.2e} of the largest")
    del a, q, yh_full
    l, r = O.loss_multiplier(wl.loss, wl.loss_scale, yh, wl.y)
    gw0, gw, gV = O.gradient(X, r, G, wl.w, wl.V, wl.lambda_w, wl.lambda_v)
    obj = m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
    assert abs(obj[0] - wl.loss_scale * l.sum()) <= REL_TOL * wl.loss_scale * l.sum()
    assert_close(d_w.cpu().numpy(), wl.w - wl.eta * gw, "w after an epoch with half gathers")
    assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), wl.V - wl.eta * gV, "V after an epoch with half gathers")


def test_full_size_first_step_element_by_element(full):
    wl, m, X, B = full
    _check_first_epoch_elementwise(B, wl, m, X)


def test_full_size_stratum_on_sampled_cells(full):
    wl, m, X, B = full
    m.fm_partition(wl.P)
    # cell 0 has the 13 always-present columns
    p, dev, aux = _check_stratum0_cells(B, wl, m, X, (0, 1, 17, wl.P - 1))
    obj = _check_epoch_property(wl, m, X, p, dev, aux)
    assert np.isfinite(sum(obj)) and sum(obj) < np.log(2.0)  # the epoch made progress from the start value


def test_full_size_minibatch_epoch_and_gradient_entry_point(full):
    """Three row batches at full size: every output against the oracle; then fm_gradient (which packs
    the caller's r, G into aggregate rows first) on every column, per array and element by element."""
    wl, m, X, B = full
    p = _params(B, wl)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    nb = 3
    m.fm_partition_batches(nb)
    obj = m.fm_minibatch_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
    kw = dict(update_w0=bool(wl.update_w0), **oracle_kw(wl))
    w0, w, V, wobj = O.minibatch_epoch(X, wl.y, float(wl.w0), wl.w, wl.V, B=nb, **kw)
    _say(f"full-size mini-batch epoch: objective gpu {sum(obj):.8f} oracle {sum(wobj):.8f}")
    assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0])
    assert_close(d_w.cpu().numpy(), w, "w after the full-size mini-batch epoch")
    assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, "V after the full-size mini-batch epoch")
    assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)
    _check_gradient_entry_point(B, wl, m, X, w0, w, V)  # at the new parameters


# ------------------------------------------------------- configs 2, 3 and 5 ----

@pytest.mark.parametrize("idx", [3, 2])
def test_full_shape_every_epoch_of_the_config(idx):
    """Configs 3 (text-like, 10 epochs, P=32: the stratified epochs are replayed from a graph) and 2 (every
    row stores all 64 columns: forward and gradient on the matrix cores, K=32 planar aggregates, 5 epochs,
    P=16) at their stated shapes: the stated
    number of full-gradient epochs, then as many stratified epochs from where those ended, every epoch's
    objective, w, V, w0 against the oracle; gradients and the first step element by element."""
    import torch
    from paper_2004_13940_amd import binding as B
    t0 = time.time()
    wl = make_config(idx)
    _say("workload", wl.name, wl.N, wl.D, wl.nnz, "K", wl.K, "P", wl.P, f"generated in {time.time() - t0:.1f}s")
    m, p, X, dev, host = run_full_epochs(B, wl, wl.epochs)
    _check_gradient_entry_point(B, wl, m, X, *host)
    _check_first_epoch_elementwise(B, wl, m, X)
    m.fm_partition(wl.P)
    run_stratified_epochs(B, wl, m, p, X, dev, host, wl.epochs)
    m.close()
    torch.cuda.empty_cache()
    _say(f"config {idx} done in {time.time() - t0:.1f}s")


def test_full_shape_config2_on_the_sparse_kernels():
    """Config 2 at its stated shape with the dense kernels switched off: the general sparse path (planar K=32
    aggregates through the LDS-staged column kernel with its real tile sizes), two epochs, the gradient entry
    point and the first step element by element."""
    import torch
    from paper_2004_13940_amd import binding as B
    t0 = time.time()
    wl = make_config(2)
    m, p, X, dev, host = run_full_epochs(B, wl, 2, setup=lambda h: h.fm_set_option(B.FM_OPT_DENSE_ROWS, 0))
    _check_gradient_entry_point(B, wl, m, X, *host)
    _check_first_epoch_elementwise(B, wl, m, X)
    m.close()
    torch.cuda.empty_cache()
    _say(f"config 2, sparse kernels, done in {time.time() - t0:.1f}s")


def test_full_shape_config5():
    """Config 5 at scale 1.0 (N=2e6, D=2e7, K=64, V = 5.1 GB; the oracle holds V, its gradient and its step in
    fp64: about 45 GB of host memory): one full-gradient epoch with every output compared, the gradient entry
    point and the first step element by element, stratum 0 of P=128 on sampled cells (cell 0 holds the head of
    the Zipf law, i.e. most of the stratum), and the any-size property of a whole stratified epoch."""
    import torch
    from paper_2004_13940_amd import binding as B
    t0 = time.time()
    _say(f"host memory available: {_host_ram_gib():.0f} GiB; config 5 runs at scale 1.0")
    wl = make_config(5)
    _say("workload", wl.name, wl.N, wl.D, wl.nnz, "K", wl.K, "P", wl.P, f"generated in {time.time() - t0:.1f}s")
    m, p, X, dev, host = run_full_epochs(B, wl, 1)
    _say(f"one full-gradient epoch compared at {time.time() - t0:.1f}s")
    del dev
    torch.cuda.empty_cache()
    _check_gradient_entry_point(B, wl, m, X, *host)
    del host
    _say(f"gradient entry point compared at {time.time() - t0:.1f}s")
    m.fm_partition(wl.P)
    p, dev, aux = _check_stratum0_cells(B, wl, m, X, (0, 1, 77, wl.P - 1))
    _say(f"stratum 0 compared at {time.time() - t0:.1f}s")
    _check_epoch_property(wl, m, X, p, dev, aux)
    m.close()
    torch.cuda.empty_cache()
    _say(f"config 5 done in {time.time() - t0:.1f}s")
