"""Seeded synthetic workloads for the factorization-machine pass.

This module only *synthesises inputs* (a CSR matrix, labels, initial
parameters, hyper-parameters).  It is shared by the tests, the benchmark and
the smoke run, and is imported by neither the CPU oracle nor the HIP library.
The five recipes stand in for the data sets the paper measures on (small dense
regression/classification tables, a text-like matrix of real-sim's shape, and
click logs of Criteo's structure; Section 5, Table "Dataset Characteristics",
and the sizing argument in the abstract): those data sets are not available
here and nothing of them is reproduced.

Labels come from a *planted teacher*: a random factorization machine whose
score is evaluated here with scipy.sparse products, then thresholded (or
perturbed with noise for regression).  This is input synthesis; neither the
oracle nor the HIP path calls it to produce any output.

Every array is a deterministic function of ``(config index, seed, scale)``:
``numpy.random.Generator(PCG64)`` streams spawned from
``SeedSequence(13940 + index)`` (or the given seed).  Columns inside a row are
distinct and ascending.
"""
from __future__ import annotations

import hashlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np
import scipy.sparse as sp

LOSS_SQUARED = 0
LOSS_LOGISTIC = 1


@dataclass
class Workload:
    name: str
    N: int
    D: int
    K: int
    rowptr: np.ndarray  # int64 [N+1]
    col: np.ndarray  # int32 [nnz], ascending and distinct inside a row
    val: np.ndarray  # float32 [nnz]
    y: np.ndarray  # float32 [N]
    w0: np.float32
    w: np.ndarray  # float32 [D]
    V: np.ndarray  # float32 [D, K] row-major
    loss: int
    lambda_w: float
    lambda_v: float
    eta: float
    loss_scale: float
    epochs: int
    P: int
    update_w0: int = 1
    notes: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def sha256(self) -> str:
        h = hashlib.sha256()
        for arr in (self.rowptr, self.col, self.val, self.y):
            h.update(np.ascontiguousarray(arr).view(np.uint8))
        return h.hexdigest()


# --------------------------------------------------------------------------
# helpers (sampling only)
# --------------------------------------------------------------------------

def _zipf_cdf(n: int, s: float) -> np.ndarray:
    """CDF of the Zipf law with exponent ``s`` truncated to ranks 1..n."""
    p = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(p)
    c /= c[-1]
    return c


def _zipf_draw(rng: np.random.Generator, cdf: np.ndarray, size: int) -> np.ndarray:
    """0-based ranks drawn by inverse CDF."""
    u = rng.random(size)
    r = np.searchsorted(cdf, u, side="right")
    np.minimum(r, len(cdf) - 1, out=r)
    return r


_CHUNKS = 64    # fixed, so that the arrays do not depend on the number of threads
_THREADS = 16


def _row_chunks(N: int) -> list[tuple[int, int]]:
    return [((c * N) // _CHUNKS, ((c + 1) * N) // _CHUNKS) for c in range(_CHUNKS) if (c * N) // _CHUNKS < ((c + 1) * N) // _CHUNKS]


def _distinct_zipf_rows(rng, lengths: np.ndarray, cdf: np.ndarray,
                        rank_to_col: np.ndarray | None) -> tuple[np.ndarray, np.ndarray]:
    """Draw ``lengths[i]`` distinct Zipf columns for every row (collisions are
    redrawn) and return (rowptr, sorted columns).  Rows are handled in fixed chunks, each with
    its own child stream of ``rng``, by a pool of threads."""
    N = len(lengths)
    rowptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(lengths, out=rowptr[1:])
    cols = np.empty(int(rowptr[-1]), dtype=np.int32)
    Dn = len(cdf)
    chunks = _row_chunks(N)
    streams = rng.spawn(len(chunks))

    def work(t):
        (lo, hi), g = chunks[t], streams[t]
        n = int(rowptr[hi] - rowptr[lo])
        rows = np.repeat(np.arange(lo, hi, dtype=np.int64), lengths[lo:hi])
        # keys (row, column) kept sorted: duplicates are then neighbours, and since every row keeps
        # its length the sorted keys line up with `rows` again after every round
        key = rows * Dn + _zipf_draw(g, cdf, n)
        for _ in range(10_000):
            key.sort()
            dup = np.flatnonzero(key[1:] == key[:-1]) + 1
            if len(dup) == 0:
                break
            key[dup] = rows[dup] * Dn + _zipf_draw(g, cdf, len(dup))
        else:  # pragma: no cover
            raise RuntimeError("could not make columns distinct")
        if rank_to_col is not None:
            key = rows * Dn + rank_to_col[key - rows * Dn]
            key.sort()
        cols[rowptr[lo]:rowptr[hi]] = key - rows * Dn

    with ThreadPoolExecutor(max_workers=_THREADS) as ex:
        list(ex.map(work, range(len(chunks))))
    return rowptr, cols


def _teacher_score(rowptr, col, val, N, D, w_star, V_star) -> np.ndarray:
    """Score of the planted teacher on every row (label synthesis only)."""
    n2 = (V_star ** 2).sum(axis=1)
    out = np.empty(N)

    def work(ch):
        lo, hi = ch
        e0, e1 = int(rowptr[lo]), int(rowptr[hi])
        X = sp.csr_matrix((val[e0:e1].astype(np.float64), col[e0:e1], rowptr[lo:hi + 1] - e0), shape=(hi - lo, D))
        G = X @ V_star
        X2 = X.copy()
        X2.data **= 2
        out[lo:hi] = X @ w_star + 0.5 * ((G ** 2).sum(axis=1) - X2 @ n2)

    with ThreadPoolExecutor(max_workers=_THREADS) as ex:
        list(ex.map(work, _row_chunks(N)))
    return out


def _init_params(rng, D, K):
    w0 = np.float32(0.0)
    w = np.zeros(D, dtype=np.float32)
    V = np.empty((D, K), dtype=np.float32)
    chunks = _row_chunks(D)
    streams = rng.spawn(len(chunks))

    def work(t):
        (a, b), g = chunks[t], streams[t]
        step = max(1, (1 << 22) // max(K, 1))
        for c in range(a, b, step):  # chunked: V can be several GB
            d = min(b, c + step)
            V[c:d] = g.standard_normal((d - c, K), dtype=np.float32) * np.float32(0.01)

    with ThreadPoolExecutor(max_workers=_THREADS) as ex:
        list(ex.map(work, range(len(chunks))))
    return w0, w, V


def _scaled(n: int, scale: float, lo: int = 1) -> int:
    return max(lo, int(round(n * scale)))


# --------------------------------------------------------------------------
# the five recipes
# --------------------------------------------------------------------------

def _cfg1(ss, scale):
    rng_x, rng_t, rng_p = (np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(3))
    N, D, K, nz = _scaled(2000, scale, 8), 1000, 8, 10
    pick = np.argpartition(rng_x.random((N, D)), nz, axis=1)[:, :nz]
    pick.sort(axis=1)
    col = pick.astype(np.int32).ravel()
    rowptr = np.arange(N + 1, dtype=np.int64) * nz
    val = rng_x.random(N * nz, dtype=np.float32)
    w_star = rng_t.standard_normal(D)
    V_star = rng_t.standard_normal((D, 8)) * 0.3
    sc = _teacher_score(rowptr, col, val, N, D, w_star, V_star)
    y = np.where(sc >= 0, 1.0, -1.0)
    flip = rng_t.random(N) < 0.05
    y[flip] = -y[flip]
    w0, w, V = _init_params(rng_p, D, K)
    return Workload("cfg1_tiny_binary", N, D, K, rowptr, col, val, y.astype(np.float32), w0, w, V,
                    LOSS_LOGISTIC, 1e-4, 1e-4, 0.1, 1.0, 10, 4, 0,
                    {"teacher_K": 8, "flip": 0.05})


def _cfg2(ss, scale):
    rng_x, rng_t, rng_p = (np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(3))
    N, D, K = _scaled(1_000_000, scale, 64), 64, 32
    col = np.tile(np.arange(D, dtype=np.int32), N)
    rowptr = np.arange(N + 1, dtype=np.int64) * D
    val = rng_x.standard_normal(N * D, dtype=np.float32)
    w_star = rng_t.standard_normal(D) / np.sqrt(D)
    V_star = rng_t.standard_normal((D, 32)) * 0.3 / np.sqrt(D)
    sc = _teacher_score(rowptr, col, val, N, D, w_star, V_star)
    y = sc + 0.1 * rng_t.standard_normal(N)
    w0, w, V = _init_params(rng_p, D, K)
    return Workload("cfg2_dense_regression", N, D, K, rowptr, col, val, y.astype(np.float32), w0, w, V,
                    LOSS_SQUARED, 1e-5, 1e-5, 0.05, 1.0 / N, 5, 16, 1,
                    {"teacher_K": 32, "noise_std": 0.1})


def _cfg3(ss, scale):
    rng_x, rng_t, rng_p = (np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(3))
    N, D, K = _scaled(50_000, scale, 64), 20_000, 16
    lengths = np.clip(rng_x.poisson(50, N), 1, D).astype(np.int64)
    perm = rng_x.permutation(D).astype(np.int64)
    rowptr, col = _distinct_zipf_rows(rng_x, lengths, _zipf_cdf(D, 1.0), perm)
    nnz = int(rowptr[-1])
    val = rng_x.lognormal(0.0, 1.0, nnz)
    sq = np.add.reduceat(val * val, rowptr[:-1])
    val = (val / np.sqrt(np.repeat(sq, lengths))).astype(np.float32)
    w_star = rng_t.standard_normal(D)
    V_star = rng_t.standard_normal((D, 16)) * 0.3
    sc = _teacher_score(rowptr, col, val, N, D, w_star, V_star)
    y = np.where(sc >= np.median(sc), 1.0, -1.0)
    w0, w, V = _init_params(rng_p, D, K)
    return Workload("cfg3_textlike_sparse", N, D, K, rowptr, col, val, y.astype(np.float32), w0, w, V,
                    LOSS_LOGISTIC, 1e-4, 1e-4, 4.0, 1.0 / N, 10, 32, 1,
                    {"teacher_K": 16, "zipf_s": 1.0})


def _cfg4(ss, scale, threads=8):
    N, D, K = _scaled(10_000_000, scale, 64), 1_000_000, 16
    ND, NF, nz = 13, 26, 39
    seeds = ss.spawn(NF + 3)
    rng_d = np.random.Generator(np.random.PCG64(seeds[NF]))
    rng_t = np.random.Generator(np.random.PCG64(seeds[NF + 1]))
    rng_p = np.random.Generator(np.random.PCG64(seeds[NF + 2]))
    col = np.empty((N, nz), dtype=np.int32)
    val = np.ones((N, nz), dtype=np.float32)
    col[:, :ND] = np.arange(ND, dtype=np.int32)
    val[:, :ND] = np.log1p(rng_d.poisson(3.0, (N, ND))).astype(np.float32)
    span = D - ND
    starts = [ND + (f * span) // NF for f in range(NF + 1)]

    def fill(f):
        rng = np.random.Generator(np.random.PCG64(seeds[f]))
        width = starts[f + 1] - starts[f]
        col[:, ND + f] = starts[f] + _zipf_draw(rng, _zipf_cdf(width, 1.1), N)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(fill, range(NF)))
    rowptr = np.arange(N + 1, dtype=np.int64) * nz
    col = col.ravel()
    val = val.ravel()
    w_star = rng_t.standard_normal(D)
    V_star = rng_t.standard_normal((D, 8)) * 0.3
    sc = _teacher_score(rowptr, col, val, N, D, w_star, V_star)
    thr = np.quantile(sc, 0.97)
    y = np.where(sc > thr, 1.0, -1.0)
    w0, w, V = _init_params(rng_p, D, K)
    return Workload("cfg4_click_onehot", N, D, K, rowptr, col, val, y.astype(np.float32), w0, w, V,
                    LOSS_LOGISTIC, 1e-6, 1e-6, 0.02, 1.0 / N, 3, 64, 1,
                    {"teacher_K": 8, "positive_rate": 0.03, "zipf_s": 1.1})


def _cfg5(ss, scale):
    rng_x, rng_t, rng_p = (np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(3))
    N, D, K = _scaled(2_000_000, scale, 64), 20_000_000, 64
    if scale < 1.0:  # keep V proportionally small for reduced runs
        D = max(4096, int(round(D * scale)))
    lengths = rng_x.integers(50, 151, N).astype(np.int64)
    rowptr, col = _distinct_zipf_rows(rng_x, lengths, _zipf_cdf(D, 1.05), None)
    val = np.ones(int(rowptr[-1]), dtype=np.float32)
    w_star = rng_t.standard_normal(D) * 0.3
    V_star = rng_t.standard_normal((D, 8)) * 0.1
    sc = _teacher_score(rowptr, col, val, N, D, w_star, V_star)
    y = np.where(sc >= np.median(sc), 1.0, -1.0)
    w0, w, V = _init_params(rng_p, D, K)
    return Workload("cfg5_hashed_stress", N, D, K, rowptr, col, val, y.astype(np.float32), w0, w, V,
                    LOSS_LOGISTIC, 1e-6, 1e-6, 0.05, 1.0 / N, 2, 128, 1,
                    {"teacher_K": 8, "zipf_s": 1.05})


# --------------------------------------------------------------------------
# small dense shapes (stand-ins for the three small data sets of the paper's
# table of data set characteristics: same N, D, K and task; synthetic content)
# --------------------------------------------------------------------------

_SMALL = {"regression_513x8": (513, 8, 4, LOSS_SQUARED), "regression_303x13": (303, 13, 4, LOSS_SQUARED),
          "classification_49990x22": (49_990, 22, 4, LOSS_LOGISTIC)}


def make_small(name: str, seed: int | None = None, test_fraction: float = 0.25):
    """(train, test) workloads of one of the small dense shapes: every feature stored in every row,
    standard normal features, targets from a planted FM plus noise (regression) or the sign of the
    planted score with 5 % flipped (classification).  The test rows are drawn from the same law."""
    if name not in _SMALL:
        raise ValueError("small workload must be one of " + ", ".join(_SMALL))
    N, D, K, loss = _SMALL[name]
    ss = np.random.SeedSequence(13940 + 100 + sorted(_SMALL).index(name) if seed is None else seed)
    rng_x, rng_t, rng_p = (np.random.Generator(np.random.PCG64(q)) for q in ss.spawn(3))
    Nt = max(1, int(round(N * test_fraction)))
    w_star = rng_t.standard_normal(D) / np.sqrt(D)
    V_star = rng_t.standard_normal((D, K)) * 0.5 / np.sqrt(D)
    w0, w, V = _init_params(rng_p, D, K)
    out = []
    for n, tag in ((N, "train"), (Nt, "test")):
        col = np.tile(np.arange(D, dtype=np.int32), n)
        rowptr = np.arange(n + 1, dtype=np.int64) * D
        val = rng_x.standard_normal(n * D, dtype=np.float32)
        sc = _teacher_score(rowptr, col, val, n, D, w_star, V_star)
        if loss == LOSS_SQUARED:
            y = sc + 0.1 * rng_t.standard_normal(n)
        else:
            y = np.where(sc >= 0.0, 1.0, -1.0)
            flip = rng_t.random(n) < 0.05
            y = np.where(flip, -y, y)
        out.append(Workload(f"{name}_{tag}", n, D, K, rowptr, col, val, y.astype(np.float32), w0, w.copy(), V.copy(),
                            loss, 1e-3, 1e-3, 0.1 if loss == LOSS_SQUARED else 0.5, 1.0 / N, 20, 2, 1,
                            {"teacher_K": K, "split": tag}))
    return out[0], out[1]


_RECIPES = {1: _cfg1, 2: _cfg2, 3: _cfg3, 4: _cfg4, 5: _cfg5}


def make_config(index: int, seed: int | None = None, scale: float = 1.0) -> Workload:
    """Build workload ``index`` (1..5).  ``scale`` shrinks the row count (and,
    for workload 5, the column count) for quick checks; 1.0 is the full shape."""
    if index not in _RECIPES:
        raise ValueError("workload index must be 1..5")
    ss = np.random.SeedSequence(13940 + index if seed is None else seed)
    wl = _RECIPES[index](ss, float(scale))
    wl.notes["scale"] = float(scale)
    return wl


def random_placement(D: int, P: int, seed: int) -> np.ndarray:
    """Seeded initial placement of the D columns on P workers, uniform at random (Algorithm 1 places
    the parameters at random before the first round)."""
    return np.random.Generator(np.random.PCG64(seed)).integers(0, P, D).astype(np.int32)


def random_csr(rng: np.random.Generator, N: int, D: int, density: float,
               empty_rows: bool = True) -> tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Small random CSR matrix with N(0,1) values for unit tests (rows may be
    empty, columns may be empty)."""
    mask = rng.random((N, D)) < density
    if not empty_rows:
        mask[np.arange(N), rng.integers(0, D, N)] = True
    rowptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(mask.sum(axis=1), out=rowptr[1:])
    col = np.nonzero(mask)[1].astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    return rowptr, col, val
