"""fm_forward_noalloc (the entry point for callers that cannot allocate device memory) against
fm_forward, through the C ABI: two calls in a row on the same GPU, the second with a smaller
input, so that the static scratch still holds the first call's partial sums when the second
runs.  Same kernels on both sides: the outputs must agree bit for bit, and both agree with the
fp64 oracle to the usual tolerance."""
import numpy as np
import pytest

from oracle import fm_oracle as O
from paper_2004_13940_amd.workloads import random_csr

from helpers import REL_TOL, assert_close, dev_params, to_dev

pytestmark = pytest.mark.gpu


def _case(seed, N, D, K, loss):
    rng = np.random.default_rng(seed)
    rowptr, col, val = random_csr(rng, N, D, 12.0 / D)
    y = (np.where(rng.random(N) < 0.5, 1.0, -1.0) if loss == O.LOSS_LOGISTIC else rng.standard_normal(N)).astype(np.float32)
    w = (rng.standard_normal(D) * 0.1).astype(np.float32)
    V = (rng.standard_normal((D, K)) * 0.1).astype(np.float32)
    return rowptr, col, val, y, np.float32(0.05), w, V


def test_noalloc_forward_matches_forward_on_two_calls_in_a_row():
    import torch
    from paper_2004_13940_amd import binding as B
    # the first input spans many workgroups and a ragged tail; the second is smaller and uses a
    # different latent size (other lane layout, other number of workgroups)
    for seed, N, D, K, loss in [(1, 70001, 900, 16, O.LOSS_LOGISTIC), (2, 1237, 300, 8, O.LOSS_SQUARED)]:
        rowptr, col, val, y, w0, w, V = _case(seed, N, D, K, loss)
        print("noalloc case", N, D, K, loss, len(col), flush=True)
        m = B.Matrix(N, D, rowptr, col, val)
        p = B.make_params(K, loss, 1e-4, 1e-4, 0.1, 0.5, 1)
        d_w0, d_w, d_V = dev_params(w0, w, V)
        d_y = to_dev(y)
        ref = {k: torch.empty(n, device="cuda") for k, n in (("yhat", N), ("a", N), ("G", N * K), ("q", N), ("r", N))}
        got = {k: torch.full_like(v, float("nan")) for k, v in ref.items()}
        sums = torch.full((2,), float("nan"), dtype=torch.float64, device="cuda")
        loss_ref = m.fm_forward(p, d_y, d_w0, d_w, d_V, want_loss=True, **ref)
        m.fm_forward_noalloc(p, d_y, d_w0, d_w, d_V, sums=sums, **got)
        torch.cuda.synchronize()
        for k in ref:
            np.testing.assert_array_equal(got[k].cpu().numpy(), ref[k].cpu().numpy(), err_msg=k)
        assert sums[0].item() == loss_ref
        r64 = ref["r"].double().cpu().numpy()
        assert abs(sums[1].item() - r64.sum()) <= 1e-6 * np.abs(r64).sum()
        X = O.make_matrix(N, D, rowptr, col, val)
        a, G, q, yh = O.forward(X, float(w0), w, V)
        l, r = O.loss_multiplier(loss, 0.5, yh, y)
        assert_close(got["yhat"].cpu().numpy(), yh, "yhat")
        assert_close(got["G"].cpu().numpy().reshape(N, K), G, "G")
        assert_close(got["r"].cpu().numpy(), r, "r")
        assert abs(sums[0].item() - l.sum()) <= REL_TOL * l.sum()
        assert abs(sums[1].item() - r.sum()) <= REL_TOL * np.abs(r).sum()
        # outputs are optional, as in fm_forward
        m.fm_forward_noalloc(p, None, d_w0, d_w, d_V, yhat=got["yhat"])
        torch.cuda.synchronize()
        np.testing.assert_array_equal(got["yhat"].cpu().numpy(), ref["yhat"].cpu().numpy())
        m.close()


def test_noalloc_forward_rejects_what_it_cannot_hold():
    import torch
    from paper_2004_13940_amd import binding as B
    rowptr, col, val, y, w0, w, V = _case(3, 50, 20, 4, O.LOSS_LOGISTIC)
    m = B.Matrix(50, 20, rowptr, col, val)
    p = B.make_params(4, O.LOSS_LOGISTIC, 0.0, 0.0, 0.1)
    d_w0, d_w, d_V = dev_params(w0, w, V)
    sums = torch.zeros(2, dtype=torch.float64, device="cuda")
    with pytest.raises(B.FMError) as e:  # sums need y
        m.fm_forward_noalloc(p, None, d_w0, d_w, d_V, sums=sums)
    assert e.value.code == -1
    m.fm_profile_enable(True)
    with pytest.raises(B.FMError) as e:
        m.fm_forward_noalloc(p, to_dev(y), d_w0, d_w, d_V, sums=sums)
    assert e.value.code == -5
    m.fm_profile_enable(False)
    m.close()
    # more workgroups than the static scratch has pairs for: an empty matrix of 2^24 + 64 rows at K = 16
    N = (1 << 24) + 64
    big = B.Matrix(N, 4, np.zeros(N + 1, np.int64), np.zeros(0, np.int32), np.zeros(0, np.float32))
    p16 = B.make_params(16, O.LOSS_LOGISTIC, 0.0, 0.0, 0.1)
    yb = torch.ones(N, device="cuda")
    Vb = torch.zeros(4 * 16, device="cuda")
    wb = torch.zeros(4, device="cuda")
    with pytest.raises(B.FMError) as e:
        big.fm_forward_noalloc(p16, yb, d_w0, wb, Vb, sums=sums)
    assert e.value.code == -4 and "workgroups" in str(e.value)
    yh = torch.empty(N, device="cuda")
    big.fm_forward_noalloc(p16, yb, d_w0, wb, Vb, yhat=yh)  # without sums any size runs
    torch.cuda.synchronize()
    assert float(yh.min()) == float(yh.max()) == float(d_w0.item())
    big.close()
