"""Shared helpers of the GPU parity tests: run the same seeded inputs through the
HIP library (via the C ABI binding) and through the fp64 oracle, and compare."""
import numpy as np

from oracle import fm_oracle as O

REL_TOL = 1e-4  # relative tolerance for fp32 outputs against the fp64 oracle


def rel_err(got, want):
    """max |got - want| / max |want|  (per array; sign-cancelling sums are judged
    against the largest entry of the array)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    assert got.shape == want.shape
    if want.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite GPU output"
    return float(np.max(np.abs(got - want)) / max(float(np.max(np.abs(want))), 1e-30))


def assert_close(got, want, what, tol=REL_TOL):
    e = rel_err(got, want)
    assert e <= tol, f"{what}: relative error {e:.3e} > {tol:.1e}"
    return e


def to_dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def dev_params(w0, w, V):
    import torch
    return (torch.tensor([float(w0)], dtype=torch.float32, device="cuda"), to_dev(w), to_dev(V))


def oracle_matrix(N, D, rowptr, col, val):
    return O.make_matrix(N, D, rowptr, col, val)


def oracle_kw(wl_or_params):
    p = wl_or_params
    return dict(loss=p.loss, s=p.loss_scale, lambda_w=p.lambda_w, lambda_v=p.lambda_v, eta=p.eta)
