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


# Element-wise bound for an fp32 result that is a sum of terms:  |got - want| <= REL_TOL |want| + ELEM_C sum|terms|.
# The second part is what fp32 arithmetic can resolve: every product is rounded (relative 2^-24) and the library
# adds them in fp32 inside work items of a few hundred entries (then in fp64): about sqrt(256) 2^-24 = 2^-20 of
# sum|terms| when the roundings are independent.  Observed worst cases stay below a third of this bound.
ELEM_C = 2.0 ** -20


def assert_elementwise(got, want, terms, what, rel=REL_TOL, c=ELEM_C):
    """Every element within rel |want| + c terms (terms = sum of the absolute values of the summands of that
    element).  Returns the largest |got - want| / (rel |want| + c terms).  Also prints, for information, the
    share of elements inside the tighter figure 1e-4 (|want| + 2^-20 terms)."""
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    terms = np.asarray(terms, dtype=np.float64).ravel()
    assert got.shape == want.shape == terms.shape
    if want.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), f"{what}: non-finite GPU output"
    err = np.abs(got - want)
    bound = rel * np.abs(want) + c * terms
    ratio = np.where(err > 0, err / np.maximum(bound, 1e-300), 0.0)
    worst = int(np.argmax(ratio))
    tight = float(np.mean(err <= 1e-4 * (np.abs(want) + terms * 2.0 ** -20)))
    print(f"  element-wise {what}: worst error/bound {ratio[worst]:.3f} at {worst} "
          f"(got {got[worst]:.6e} want {want[worst]:.6e} terms {terms[worst]:.3e}); "
          f"{100 * tight:.2f}% inside 1e-4 (|o| + 2^-20 sum|terms|)", flush=True)
    assert ratio[worst] <= 1.0, (f"{what}: element {worst}: |{got[worst]:.8e} - {want[worst]:.8e}| = {err[worst]:.3e} "
                                 f"> {bound[worst]:.3e}")
    return float(ratio[worst])


def gradient_term_sums(X, r, G, w, V, lambda_w, lambda_v):
    """sum of |summands| of every entry of grad_w and grad_V (eqs. updates_w, updates_v):
    sum_i |x_ij r_i| + lambda_w |w_j|   and   sum_i |x_ij r_i G_ik| + |v_jk| sum_i x_ij^2 |r_i| + lambda_v |v_jk|,
    from two oracle passes over the matrix of absolute values."""
    Xa = O.Matrix(X.N, X.D, X.rowptr, X.col, np.abs(X.val), X.colptr, X.row, np.abs(X.cval))
    ra, Ga = np.abs(np.asarray(r, np.float64)), np.abs(np.asarray(G, np.float64))
    w, V = np.asarray(w, np.float64), np.asarray(V, np.float64)
    D, K = V.shape
    _, tw, tV = O.gradient(Xa, ra, Ga, np.zeros(D), np.zeros((D, K)), 0.0, 0.0)
    # with G = 0 and V = -1 the same routine returns sum_i |r_i| x_ij^2
    _, _, s2 = O.gradient(Xa, ra, np.zeros((X.N, 1)), np.zeros(D), -np.ones((D, 1)), 0.0, 0.0)
    return tw + lambda_w * np.abs(w), tV + s2 * np.abs(V) + lambda_v * np.abs(V)


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


def _say(*a):
    print(*a, flush=True)


# ---- epoch runners shared by the parity tests: the library and the oracle side by side ----

def run_full_epochs(B, wl, epochs, m=None, setup=None):
    """epochs of fm_sgd_epoch vs the oracle's full_epoch; returns final states.  ``setup(m)`` runs on the
    new handle before its CSC is built (tuning and options)."""
    import torch
    X = O.make_matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
    if m is None:
        m = B.Matrix(wl.N, wl.D, wl.rowptr, wl.col, wl.val)
        if setup is not None:
            setup(m)
        m.fm_build_csc()
    p = B.make_params(wl.K, wl.loss, wl.lambda_w, wl.lambda_v, wl.eta, wl.loss_scale, wl.update_w0)
    d_w0, d_w, d_V = dev_params(wl.w0, wl.w, wl.V)
    d_y = to_dev(wl.y)
    w0, w, V = float(wl.w0), wl.w.astype(np.float64), wl.V.astype(np.float64)
    kw = oracle_kw(wl)
    for ep in range(epochs):
        obj = m.fm_sgd_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        w0, w, V, wobj = O.full_epoch(X, wl.y, w0, w, V, update_w0=bool(wl.update_w0), **kw)
        torch.cuda.synchronize()
        _say(f"  epoch {ep}: objective gpu {obj[0] + obj[1]:.8f} oracle {wobj[0] + wobj[1]:.8f}")
        assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0]), f"data term, epoch {ep}"
        assert abs(obj[1] - wobj[1]) <= REL_TOL * abs(wobj[1]) + 1e-12, f"regulariser, epoch {ep}"
        assert_close(d_w.cpu().numpy(), w, f"w after epoch {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after epoch {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3), f"w0 after epoch {ep}"
    return m, p, X, (d_w0, d_w, d_V, d_y), (w0, w, V)


def run_stratified_epochs(B, wl, m, p, X, dev, host, epochs, check_strata=False, **flags):
    import torch
    d_w0, d_w, d_V, d_y = dev
    w0, w, V = host
    for k, v in flags.items():
        setattr(p, k, int(v))
    kw = oracle_kw(wl)
    okw = dict(reg_share=not flags.get("reg_full_per_cell", False), refresh_all_rows=flags.get("refresh_all_rows", False),
               stale_aux=flags.get("stale_aux", False))
    for ep in range(epochs):
        if check_strata:
            # step through the strata on both sides and compare the live aggregates
            snaps = []
            O.stratified_epoch(X, wl.y, w0, w, V, P=m.P, update_w0=bool(wl.update_w0), final_objective=False,
                               on_stratum=lambda s, st: snaps.append({k: st[k].copy() for k in ("a", "G", "q", "r", "w", "V")}),
                               **kw, **okw)
            m.fm_stratified_begin(p, d_y, d_w0, d_w, d_V)
            a, G, q, r = (torch.empty(n, device="cuda") for n in (wl.N, wl.N * wl.K, wl.N, wl.N))
            for s in range(m.P):
                m.fm_stratified_step(p, s, d_y, d_w0, d_w, d_V)
                m.fm_get_aux(wl.K, a, G, q, r)
                torch.cuda.synchronize()
                for name, t in (("a", a), ("G", G), ("q", q), ("w", d_w), ("V", d_V)):
                    assert_close(t.cpu().numpy(), snaps[s][name], f"{name} after stratum {s} of epoch {ep}")
                # the library keeps r current with the refreshed aggregates; the oracle recomputes it
                # at the start of the next cell step: same function of the same aggregates
                want_r = O.multiplier_from_aux(wl.loss, wl.loss_scale, w0, snaps[s]["a"], snaps[s]["G"],
                                               snaps[s]["q"], wl.y)
                assert_close(r.cpu().numpy(), want_r, f"r after stratum {s} of epoch {ep}")
            m.fm_stratified_end(p, d_w0)
            obj = None
        else:
            obj = m.fm_stratified_epoch(p, d_y, d_w0, d_w, d_V, want_objective=True)
        w0, w, V, wobj, _ = O.stratified_epoch(X, wl.y, w0, w, V, P=m.P, update_w0=bool(wl.update_w0), **kw, **okw)
        torch.cuda.synchronize()
        if obj is not None:
            _say(f"  stratified epoch {ep}: objective gpu {obj[0] + obj[1]:.8f} oracle {wobj[0] + wobj[1]:.8f}")
            assert abs(obj[0] - wobj[0]) <= REL_TOL * abs(wobj[0]), f"data term, stratified epoch {ep}"
            assert abs(obj[1] - wobj[1]) <= REL_TOL * abs(wobj[1]) + 1e-12
        assert_close(d_w.cpu().numpy(), w, f"w after stratified epoch {ep}")
        assert_close(d_V.cpu().numpy().reshape(wl.D, wl.K), V, f"V after stratified epoch {ep}")
        assert abs(d_w0.item() - w0) <= REL_TOL * max(abs(w0), 1e-3)
    return (w0, w, V)
