"""fp64 CPU oracle for the FM pass -- TEST INFRASTRUCTURE ONLY.

Thin numpy front end over the plain C loops in ``fm_oracle.c`` plus the epoch
drivers (full-gradient epoch, stratified epoch, mini-batch epoch), written step by
step in the paper's order.  Nothing here imports, or is imported by, the HIP library;
only tests, the smoke check and the benchmark's ``cpu_baseline`` leg use it.

Pinned by tests/test_oracle_*.py against: the O(K D^2) pairwise definition
(eq. fm_model), a hand-computed example, closed forms, library sparse
products for V=0, central finite differences of the objective, the ridge
solution, dense transposes and brute-force cell masks.

Parity unpinned (conventions with no external check): the share ``rho`` of the
regulariser a cell step applies, the moment the bias is updated in a stratified
epoch, and the direction in which a column is handed from worker to worker.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fm_oracle.c")
_LIB = os.path.join(_HERE, "libfm_oracle.so")

LOSS_SQUARED = 0
LOSS_LOGISTIC = 1


def build(force: bool = False) -> str:
    """Compile the C loops with gcc (fp64, -O2, OpenMP over independent rows/columns)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_block_bound.restype = ctypes.c_int64
        _lib.oracle_block_bound.argtypes = [ctypes.c_int64] * 3
        _lib.oracle_threads.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(_L().oracle_threads())


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i64(x):
    return ctypes.c_int64(int(x))


def _i32(x):
    return ctypes.c_int32(int(x))


def _f64(x):
    return ctypes.c_double(float(x))


def _c(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


@dataclass
class Matrix:
    """The data matrix in both orientations, values widened to fp64."""
    N: int
    D: int
    rowptr: np.ndarray
    col: np.ndarray
    val: np.ndarray
    colptr: np.ndarray
    row: np.ndarray
    cval: np.ndarray


def csr_to_csc(N, D, rowptr, col, val):
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float64)
    nnz = int(rowptr[-1])
    colptr = np.empty(D + 1, np.int64)
    row = np.empty(nnz, np.int32)
    cval = np.empty(nnz, np.float64)
    _L().oracle_csr_to_csc(_i64(N), _i64(D), _p(rowptr), _p(col), _p(val), _p(colptr), _p(row), _p(cval))
    return colptr, row, cval


def make_matrix(N, D, rowptr, col, val) -> Matrix:
    rowptr, col, val = _c(rowptr, np.int64), _c(col, np.int32), _c(val, np.float64)
    colptr, row, cval = csr_to_csc(N, D, rowptr, col, val)
    return Matrix(int(N), int(D), rowptr, col, val, colptr, row, cval)


def forward(X: Matrix, w0, w, V):
    """a, G, q, yhat of every row (eq. fm_model2, eq. compute_a_jk)."""
    w, V = _c(w, np.float64), _c(V, np.float64)
    K = V.shape[1]
    a = np.empty(X.N)
    G = np.empty((X.N, K))
    q = np.empty(X.N)
    yhat = np.empty(X.N)
    _L().oracle_forward(_i64(X.N), _i32(K), _p(X.rowptr), _p(X.col), _p(X.val), _f64(w0),
                        _p(w), _p(V), _p(a), _p(G), _p(q), _p(yhat))
    return a, G, q, yhat


def loss_multiplier(loss, s, yhat, y):
    """Per-row loss l_i and multiplier r_i = s dl/dyhat."""
    yhat, y = _c(yhat, np.float64), _c(y, np.float64)
    l = np.empty_like(yhat)
    r = np.empty_like(yhat)
    _L().oracle_loss_multiplier(_i64(len(yhat)), _i32(loss), _f64(s), _p(yhat), _p(y), _p(l), _p(r))
    return l, r


def objective(loss, s, lambda_w, lambda_v, X: Matrix, y, w0, w, V):
    """(data term, regulariser) of eq. fm_obj with the data term scaled by s
    (s = 1/N is the printed objective; s = 1 matches the printed updates)."""
    _, _, _, yhat = forward(X, w0, w, V)
    l, _ = loss_multiplier(loss, s, yhat, y)
    w, V = _c(w, np.float64), _c(V, np.float64)
    return s * float(np.sum(l)), 0.5 * lambda_w * float(np.sum(w * w)) + 0.5 * lambda_v * float(np.sum(V * V))


def gradient(X: Matrix, r, G, w, V, lambda_w, lambda_v):
    """grad_w0, grad_w, grad_V (eqs. updates_w0, updates_w, updates_v)."""
    r, G, w, V = _c(r, np.float64), _c(G, np.float64), _c(w, np.float64), _c(V, np.float64)
    K = V.shape[1]
    gw0 = ctypes.c_double(0.0)
    gw = np.empty(X.D)
    gV = np.empty((X.D, K))
    _L().oracle_gradient(_i64(X.N), _i64(X.D), _i32(K), _p(X.colptr), _p(X.row), _p(X.cval), _p(r),
                         _p(G), _p(w), _p(V), _f64(lambda_w), _f64(lambda_v), ctypes.byref(gw0),
                         _p(gw), _p(gV))
    return gw0.value, gw, gV


def full_epoch(X: Matrix, y, w0, w, V, *, loss, s, lambda_w, lambda_v, eta, update_w0=True):
    """One full-gradient step: forward -> r -> gradient -> parameters -= eta * gradient.
    Returns new (w0, w, V) and the objective (data, reg) at the parameters the
    epoch started from."""
    w, V = _c(w, np.float64).copy(), _c(V, np.float64).copy()
    a, G, q, yhat = forward(X, w0, w, V)
    l, r = loss_multiplier(loss, s, yhat, y)
    obj = (s * float(np.sum(l)),
           0.5 * lambda_w * float(np.sum(w * w)) + 0.5 * lambda_v * float(np.sum(V * V)))
    gw0, gw, gV = gradient(X, r, G, w, V, lambda_w, lambda_v)
    if update_w0:
        w0 = float(w0) - eta * gw0
    w -= eta * gw
    V -= eta * gV
    return float(w0), w, V, obj


def multiplier_from_aux(loss, s, w0, a, G, q, y):
    """r for every row from stored aggregates (prediction by eq. fm_model2, no pass over X)."""
    a, G, q, y = _c(a, np.float64), _c(G, np.float64), _c(q, np.float64), _c(y, np.float64)
    r = np.empty(len(a))
    _L().oracle_multiplier_from_aux(_i64(len(a)), _i32(G.shape[1]), _i32(loss), _f64(s), _f64(w0), _p(a), _p(G),
                                    _p(q), _p(y), _p(r))
    return r


def block_bounds(n, P):
    """Boundaries of the contiguous floor split of n items into P blocks."""
    return np.array([_L().oracle_block_bound(_i64(n), _i64(P), _i64(b)) for b in range(P + 1)], np.int64)


def stratum_cells(P, s):
    """Cells (row block p, column block q) active in stratum s of the synchronous
    ring (Section 4.2; figure of the communication pattern: stratum 0 is the
    diagonal, column blocks then rotate by one)."""
    return [(p, (p + s) % P) for p in range(P)]


def cell_update(X: Matrix, y, w0, w, V, a, G, q, r, rows, cols, *, loss, s, eta, rho, lambda_w, lambda_v,
                dw, dV, dn):
    """Phase A of one cell step, in place on (w, V, r) with the deltas recorded in (dw, dV, dn):
    rows = (i_lo, i_hi), cols = (j_lo, j_hi).  All arrays fp64 and contiguous."""
    K = V.shape[1]
    _L().oracle_cell_update(_i32(K), _i32(loss), _f64(s), _f64(eta), _f64(rho), _f64(lambda_w), _f64(lambda_v),
                            _i64(rows[0]), _i64(rows[1]), _i64(cols[0]), _i64(cols[1]), _p(X.colptr), _p(X.row),
                            _p(X.cval), _p(y), _f64(w0), _p(a), _p(G), _p(q), _p(r), _p(w), _p(V), _p(dw), _p(dV),
                            _p(dn))


def refresh(X: Matrix, a, G, q, rows, cols, dw, dV, dn):
    """Phase B of one cell step, in place on (a, G, q)."""
    K = G.shape[1]
    _L().oracle_refresh(_i32(K), _i64(rows[0]), _i64(rows[1]), _i64(cols[0]), _i64(cols[1]), _p(X.rowptr), _p(X.col),
                        _p(X.val), _p(dw), _p(dV), _p(dn), _p(a), _p(G), _p(q))


def placed_epoch(X: Matrix, y, w0, w, V, *, P, place, loss, s, lambda_w, lambda_v, eta,
                 update_w0=True, reg_share=True, stale_aux=True, on_round=None, final_objective=True):
    """One epoch of the schedule of Algorithm 1 with every column handed on individually (Section 4.3).

    Worker p owns the rows of row block p for good.  Column j (its w_j and v_j) starts at worker
    ``place[j]`` (the paper places the parameters at random) and is handed on to the next worker after
    every round, against the numbering of the workers, so that in round t it is at worker
    (place[j] - t) mod P and after P rounds it has met every row block once; with
    place[j] = column block of j this is the ring of ``stratified_epoch``.

      aux (a,G,q) <- forward from scratch                        (the re-computation loop)
      for round t = 0..P-1, for every worker p with the columns J it holds in this round:
          r_I from aux; block gradient of the columns of J over the rows of p; step on w_J, V_J
          (``stale_aux``: nothing else, the update phase of Algorithm 1 reads stale aggregates;
           otherwise worker p refreshes its own rows with the changes of J, as in Section 4.2)
      bias step from the aux as it stands; objective from a fresh forward.

    ``on_round(t, state)`` is called after every round; state["held"][p] lists the columns worker p held.
    """
    y = _c(y, np.float64)
    w, V = _c(w, np.float64).copy(), _c(V, np.float64).copy()
    place = _c(place, np.int64)
    K = V.shape[1]
    N, D = X.N, X.D
    if place.shape != (D,) or (D and (place.min() < 0 or place.max() >= P)):
        raise ValueError("place must hold one worker in [0, P) per column")
    rb = block_bounds(N, P)
    a, G, q, _ = forward(X, w0, w, V)
    r = np.zeros(N)
    dw, dV, dn = np.zeros(D), np.zeros((D, K)), np.zeros(D)
    L = _L()
    for t in range(P):
        at = (place - t) % P  # the worker every column is at in this round
        held = [np.flatnonzero(at == p).astype(np.int32) for p in range(P)]
        for p in range(P):
            rho = (rb[p + 1] - rb[p]) / N if reg_share else 1.0
            L.oracle_cell_update_cols(_i32(K), _i32(loss), _f64(s), _f64(eta), _f64(rho), _f64(lambda_w),
                                      _f64(lambda_v), _i64(rb[p]), _i64(rb[p + 1]), _i64(len(held[p])),
                                      _p(held[p]), _p(X.colptr), _p(X.row), _p(X.cval), _p(y), _f64(w0), _p(a),
                                      _p(G), _p(q), _p(r), _p(w), _p(V), _p(dw), _p(dV), _p(dn))
        if not stale_aux:
            for p in range(P):
                inset = (at == p).astype(np.uint8)
                L.oracle_refresh_cols(_i32(K), _i64(rb[p]), _i64(rb[p + 1]), _p(inset), _p(X.rowptr), _p(X.col),
                                      _p(X.val), _p(dw), _p(dV), _p(dn), _p(a), _p(G), _p(q))
        if on_round is not None:
            on_round(t, dict(a=a, G=G, q=q, r=r, w=w, V=V, held=held))
    if update_w0:
        L.oracle_multiplier_from_aux(_i64(N), _i32(K), _i32(loss), _f64(s), _f64(w0), _p(a), _p(G),
                                     _p(q), _p(y), _p(r))
        w0 = float(w0) - eta * float(np.sum(r))
    obj = objective(loss, s, lambda_w, lambda_v, X, y, w0, w, V) if final_objective else None
    return float(w0), w, V, obj, dict(a=a, G=G, q=q, r=r)


def block_placement(D, P):
    """place[j] = column block of j in the contiguous floor split: the placement that turns
    ``placed_epoch`` into the ring of ``stratified_epoch``."""
    cb = block_bounds(D, P)
    return (np.searchsorted(cb, np.arange(D), side="right") - 1).astype(np.int32)


def stratified_epoch(X: Matrix, y, w0, w, V, *, P, loss, s, lambda_w, lambda_v, eta,
                     update_w0=True, reg_share=True, refresh_all_rows=False, stale_aux=False,
                     cell_order=None, on_stratum=None, final_objective=True):
    """One doubly-separable stratified epoch (Sections 4.2-4.3, synchronous ring reading).

      aux (a,G,q) <- forward from scratch            (the re-computation pass)
      for stratum s = 0..P-1, for its P disjoint cells (I_p, J_(p+s) mod P):
          phase A  r_I from aux; block gradient over the cell; step on w_J, V_J;
                   record the deltas
          phase B  refresh a_I, G_I, q_I with the deltas of J     (incremental sync)
      bias step from the aux as it stands; objective from a fresh forward.

    ``reg_share``: a cell step applies the share |I|/N of the regulariser (so that
    one epoch applies one epoch's worth and P=1 is the full-gradient epoch);
    False applies the full lambda in every cell step.
    ``refresh_all_rows``: phase B of a stratum refreshes every row with every
    column's delta (aggregates stay exact) instead of only each cell's own rows
    (aggregates of other row blocks go stale until the next re-computation, as
    the paper describes).
    ``stale_aux``: no phase B at all: every cell step of the epoch reads the
    aggregates computed at its start, and they are only recomputed by the next
    epoch's forward (the two phases of Algorithm 1: update with stale G and A,
    then re-computation).
    ``cell_order``: optional permutation of range(P) per stratum, to show that the
    result does not depend on the order of the cells.
    ``on_stratum(s, state)`` is called after every stratum with a dict of the live arrays.
    """
    y = _c(y, np.float64)
    w, V = _c(w, np.float64).copy(), _c(V, np.float64).copy()
    K = V.shape[1]
    N, D = X.N, X.D
    rb, cb = block_bounds(N, P), block_bounds(D, P)
    a, G, q, _ = forward(X, w0, w, V)
    r = np.zeros(N)
    dw, dV, dn = np.zeros(D), np.zeros((D, K)), np.zeros(D)
    L = _L()
    for st in range(P):
        cells = stratum_cells(P, st)
        if cell_order is not None:
            cells = [cells[t] for t in cell_order[st]]
        for (p, qb) in cells:  # phase A
            rho = (rb[p + 1] - rb[p]) / N if reg_share else 1.0
            L.oracle_cell_update(_i32(K), _i32(loss), _f64(s), _f64(eta), _f64(rho), _f64(lambda_w),
                                 _f64(lambda_v), _i64(rb[p]), _i64(rb[p + 1]), _i64(cb[qb]),
                                 _i64(cb[qb + 1]), _p(X.colptr), _p(X.row), _p(X.cval), _p(y),
                                 _f64(w0), _p(a), _p(G), _p(q), _p(r), _p(w), _p(V), _p(dw), _p(dV), _p(dn))
        if stale_aux:  # no phase B: the aggregates wait for the re-computation
            pass
        elif refresh_all_rows:  # phase B, exact: every column changed once in this stratum
            L.oracle_refresh(_i32(K), _i64(0), _i64(N), _i64(0), _i64(D), _p(X.rowptr), _p(X.col),
                             _p(X.val), _p(dw), _p(dV), _p(dn), _p(a), _p(G), _p(q))
        else:  # phase B, local: each cell refreshes its own rows with its own columns
            for (p, qb) in cells:
                L.oracle_refresh(_i32(K), _i64(rb[p]), _i64(rb[p + 1]), _i64(cb[qb]), _i64(cb[qb + 1]),
                                 _p(X.rowptr), _p(X.col), _p(X.val), _p(dw), _p(dV), _p(dn),
                                 _p(a), _p(G), _p(q))
        if on_stratum is not None:
            on_stratum(st, dict(a=a, G=G, q=q, r=r, w=w, V=V, dw=dw, dV=dV, dn=dn, cells=cells))
    if update_w0:
        L.oracle_multiplier_from_aux(_i64(N), _i32(K), _i32(loss), _f64(s), _f64(w0), _p(a), _p(G),
                                     _p(q), _p(y), _p(r))
        w0 = float(w0) - eta * float(np.sum(r))
    obj = objective(loss, s, lambda_w, lambda_v, X, y, w0, w, V) if final_objective else None
    return float(w0), w, V, obj, dict(a=a, G=G, q=q, r=r)


def evaluate(X: Matrix, y, w0, w, V, loss):
    """Predictive performance of the model on (X, y), as the paper's figures report it: mean loss,
    root mean squared error of the score (regression) and accuracy of its sign (classification,
    labels in {-1,+1}; a score of exactly 0 counts as +1).  Plain definitions on the scores."""
    y = _c(y, np.float64)
    _, _, _, yhat = forward(X, w0, w, V)
    l, _ = loss_multiplier(loss, 1.0, yhat, y)
    n = max(len(y), 1)
    pred = np.where(yhat >= 0.0, 1.0, -1.0)
    return dict(mean_loss=float(np.sum(l)) / n, rmse=float(np.sqrt(np.sum((yhat - y) ** 2) / n)),
                accuracy=float(np.sum(pred == y)) / n)


def minibatch_epoch(X: Matrix, y, w0, w, V, *, B, loss, s, lambda_w, lambda_v, eta,
                    update_w0=True, reg_share=True, on_batch=None, final_objective=True):
    """One pass of mini-batch gradient descent over B contiguous row batches, in order
    (Section 4.1: the stochastic updates, eqs. sgd updates of w_j and v_jk, taken a batch of
    examples at a time instead of one; the batches are the floor-split row blocks).

      for batch b = 0..B-1, rows I_b:
          score the rows of I_b at the current parameters; multipliers r_i, i in I_b
          gradient of  s * sum_{i in I_b} l_i  +  rho_b (lambda_w/2 |w|^2 + lambda_v/2 |V|^2)
          step on w0, w, V with it                      (rho_b = |I_b|/N, or 1 if not reg_share)

    With B = 1 this is the full-gradient epoch.  ``on_batch(b, state)`` is called after every step.
    """
    y = _c(y, np.float64)
    w, V = _c(w, np.float64).copy(), _c(V, np.float64).copy()
    w0 = float(w0)
    K = V.shape[1]
    N, D = X.N, X.D
    rb = block_bounds(N, B)
    r = np.zeros(N)
    dw, dV, dn = np.zeros(D), np.zeros((D, K)), np.zeros(D)
    for b in range(B):
        lo, hi = int(rb[b]), int(rb[b + 1])
        a, G, q, _ = forward(X, w0, w, V)  # only the rows of the batch are used
        rho = (hi - lo) / N if reg_share else 1.0
        cell_update(X, y, w0, w, V, a, G, q, r, (lo, hi), (0, D), loss=loss, s=s, eta=eta, rho=rho,
                    lambda_w=lambda_w, lambda_v=lambda_v, dw=dw, dV=dV, dn=dn)
        if update_w0:
            w0 = w0 - eta * float(np.sum(r[lo:hi]))
        if on_batch is not None:
            on_batch(b, dict(w0=w0, w=w, V=V, r=r, rows=(lo, hi)))
    obj = objective(loss, s, lambda_w, lambda_v, X, y, w0, w, V) if final_objective else None
    return w0, w, V, obj


# ---- integer structures the library must reproduce bit for bit -------------

def batch_csc(X: Matrix, B, b):
    """CSC (colptr over all D columns, row, val) of the matrix that keeps only the rows of
    batch b of B (global row numbers)."""
    rb = block_bounds(X.N, B)
    cols = np.repeat(np.arange(X.D, dtype=np.int64), np.diff(X.colptr))
    keep = (X.row >= rb[b]) & (X.row < rb[b + 1])
    colptr = np.zeros(X.D + 1, np.int64)
    np.cumsum(np.bincount(cols[keep], minlength=X.D), out=colptr[1:])
    return colptr, X.row[keep], X.cval[keep]


def stratum_of_entries(N, D, P, rows, cols, place=None):
    """Stratum (q - p) mod P of entries given by their row and column indices; q is the column block,
    or place[column] when the columns are placed one by one (then the stratum is the round)."""
    rb, cb = block_bounds(N, P), block_bounds(D, P)
    p = np.searchsorted(rb, rows, side="right") - 1
    # empty blocks repeat a boundary: searchsorted(right)-1 lands on the last of
    # the repeated boundaries, which is the one non-empty block holding the index
    q = np.searchsorted(cb, cols, side="right") - 1 if place is None else np.asarray(place, np.int64)[cols]
    return ((q - p) % P).astype(np.int64), p, q


def cell_nnz(X: Matrix, P, place=None):
    """P x P table of stored entries per cell."""
    rows = np.repeat(np.arange(X.N, dtype=np.int64), np.diff(X.rowptr))
    _, p, q = stratum_of_entries(X.N, X.D, P, rows, X.col.astype(np.int64), place)
    out = np.zeros((P, P), np.int64)
    np.add.at(out, (p, q), 1)
    return out


def stratum_csr(X: Matrix, P, s, place=None):
    """CSR (rowptr over all N rows, col, val) of the matrix that keeps only the
    entries lying in the cells of stratum s."""
    rows = np.repeat(np.arange(X.N, dtype=np.int64), np.diff(X.rowptr))
    st, _, _ = stratum_of_entries(X.N, X.D, P, rows, X.col.astype(np.int64), place)
    keep = st == s
    rowptr = np.zeros(X.N + 1, np.int64)
    np.cumsum(np.bincount(rows[keep], minlength=X.N), out=rowptr[1:])
    return rowptr, X.col[keep], X.val[keep]


def stratum_csc(X: Matrix, P, s, place=None):
    """CSC (colptr over all D columns, row, val) of the same per-stratum matrix."""
    cols = np.repeat(np.arange(X.D, dtype=np.int64), np.diff(X.colptr))
    st, _, _ = stratum_of_entries(X.N, X.D, P, X.row.astype(np.int64), cols, place)
    keep = st == s
    colptr = np.zeros(X.D + 1, np.int64)
    np.cumsum(np.bincount(cols[keep], minlength=X.D), out=colptr[1:])
    return colptr, X.row[keep], X.cval[keep]
