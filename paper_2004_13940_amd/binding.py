"""ctypes binding of libfm_mi355x.so: same names as the C ABI (include/fm.h),
argument marshalling only.  PyTorch tensors are used as device buffers; every
step of the pass runs in the library's HIP kernels.  There is no fallback: if the
library is missing, or there is no GPU, calls raise."""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfm_mi355x.so")

FM_OK = 0
FM_LOSS_SQUARED = 0
FM_LOSS_LOGISTIC = 1
FM_EINVAL, FM_ENOMEM, FM_EUNSORTED, FM_ERANGE, FM_ESTATE, FM_EHIP = -1, -2, -3, -4, -5, -6
STATUS_NAMES = {FM_OK: "FM_OK", FM_EINVAL: "FM_EINVAL", FM_ENOMEM: "FM_ENOMEM", FM_EUNSORTED: "FM_EUNSORTED",
                FM_ERANGE: "FM_ERANGE", FM_ESTATE: "FM_ESTATE", FM_EHIP: "FM_EHIP"}


class fm_params(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int32), ("loss", ctypes.c_int32),
                ("lambda_w", ctypes.c_float), ("lambda_v", ctypes.c_float),
                ("eta", ctypes.c_float), ("loss_scale", ctypes.c_float),
                ("update_w0", ctypes.c_int32), ("reg_full_per_cell", ctypes.c_int32),
                ("refresh_all_rows", ctypes.c_int32), ("stale_aux", ctypes.c_int32),
                ("half_gather", ctypes.c_int32)]


class FMError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{STATUS_NAMES.get(code, code)}: {msg}")
        self.code = code


EXPORTS = ["fm_build_csr", "fm_build_csc", "fm_partition", "fm_partition_placed", "fm_get_csc", "fm_get_block_index",
           "fm_get_stratum_nnz", "fm_get_stratum_csr", "fm_get_stratum_csc", "fm_partition_batches",
           "fm_get_batch_csc", "fm_forward", "fm_forward_noalloc", "fm_evaluate", "fm_gradient",
           "fm_sgd_epoch", "fm_minibatch_epoch", "fm_stratified_epoch", "fm_stratified_begin", "fm_stratified_step",
           "fm_stratified_end", "fm_get_aux", "fm_profile_enable", "fm_profile_kernels",
           "fm_profile_kernel_name", "fm_profile_read", "fm_set_option", "fm_set_tuning", "fm_set_tile_tuning", "fm_destroy",
           "fm_last_error"]
FM_OPT_AUX_PLANAR, FM_OPT_SIDE_STREAMS, FM_OPT_LAZY_REG, FM_OPT_GRAPH, FM_OPT_DENSE_ROWS = 0, 1, 2, 3, 4

_lib = None


def load() -> ctypes.CDLL:
    """Load the shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2004_13940_amd.build` "
                                    "(there is no CPU fallback)")
        # PyTorch ships its own HIP runtime under the same soname; it must be the one this
        # library binds to, so that streams and device pointers of torch tensors are valid here
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name).restype = ctypes.c_int
        lib.fm_last_error.restype = ctypes.c_char_p
        lib.fm_last_error.argtypes = [ctypes.c_void_p]
        lib.fm_profile_kernel_name.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _vp(x):
    """void* of a torch tensor (device), a numpy array (host) or None."""
    if x is None:
        return ctypes.c_void_p(None)
    if isinstance(x, np.ndarray):
        return ctypes.c_void_p(x.ctypes.data)
    return ctypes.c_void_p(x.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev(t, n, what):
    import torch
    if t is None:
        return
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError(f"{what} must be a contiguous float32 CUDA tensor")
    if t.numel() != n:
        raise ValueError(f"{what} has {t.numel()} elements, expected {n}")


def make_params(K, loss, lambda_w, lambda_v, eta, loss_scale=1.0, update_w0=1, reg_full_per_cell=0,
                refresh_all_rows=0, stale_aux=0, half_gather=0) -> fm_params:
    return fm_params(int(K), int(loss), float(lambda_w), float(lambda_v), float(eta), float(loss_scale),
                     int(update_w0), int(reg_full_per_cell), int(refresh_all_rows), int(stale_aux), int(half_gather))


class Matrix:
    """Owner of an ``fm_matrix`` handle; methods mirror the C entry points."""

    def __init__(self, N, D, rowptr, col, val, stream=None):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the FM pass only runs on the HIP library")
        lib = load()
        self.N, self.D = int(N), int(D)
        rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
        col = np.ascontiguousarray(col, dtype=np.int32)
        val = np.ascontiguousarray(val, dtype=np.float32)
        if rowptr.shape != (self.N + 1,):
            raise ValueError("rowptr must have N+1 entries")
        self.nnz = int(rowptr[-1]) if len(rowptr) else 0
        if len(col) != self.nnz or len(val) != self.nnz:
            raise ValueError("col/val length must equal rowptr[N]")
        self.P = 0
        self._h = ctypes.c_void_p(None)
        rc = lib.fm_build_csr(ctypes.c_int64(self.N), ctypes.c_int64(self.D), ctypes.c_int64(self.nnz),
                              _vp(rowptr), _vp(col), _vp(val), _stream(stream), ctypes.byref(self._h))
        if rc != FM_OK:
            raise FMError(rc, (lib.fm_last_error(None) or b"").decode())

    def _check(self, rc):
        if rc != FM_OK:
            raise FMError(rc, (load().fm_last_error(self._h) or b"").decode())

    def close(self):
        if self._h:
            load().fm_destroy(self._h)
            self._h = ctypes.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- settings
    def fm_set_option(self, option, value):
        self._check(load().fm_set_option(self._h, ctypes.c_int32(int(option)), ctypes.c_int32(int(value))))

    def fm_set_tuning(self, seg=0, panel=0, heavy_per_panel=0, vlong=0, min_panels=0):
        self._check(load().fm_set_tuning(self._h, *(ctypes.c_int32(int(v)) for v in (seg, panel, heavy_per_panel, vlong,
                                                                                     min_panels))))

    def fm_set_tile_tuning(self, tile_rows=0, min_per_tile=-1, tile_seg=0):
        self._check(load().fm_set_tile_tuning(self._h, *(ctypes.c_int32(int(v)) for v in (tile_rows, min_per_tile,
                                                                                          tile_seg))))

    # -- structures
    def fm_build_csc(self, stream=None):
        self._check(load().fm_build_csc(self._h, _stream(stream)))

    def fm_partition(self, P, stream=None):
        self._check(load().fm_partition(self._h, ctypes.c_int32(P), _stream(stream)))
        self.P = int(P)

    def fm_partition_placed(self, P, place, stream=None):
        place = np.ascontiguousarray(place, dtype=np.int32)
        if place.shape != (self.D,):
            raise ValueError("place must have D entries")
        self._check(load().fm_partition_placed(self._h, ctypes.c_int32(P), _vp(place), _stream(stream)))
        self.P = int(P)
        self.placed = True

    def fm_get_csc(self):
        colptr = np.empty(self.D + 1, np.int64)
        row = np.empty(self.nnz, np.int32)
        val = np.empty(self.nnz, np.float32)
        self._check(load().fm_get_csc(self._h, _vp(colptr), _vp(row), _vp(val)))
        return colptr, row, val

    def fm_get_block_index(self):
        rb = np.empty(self.P + 1, np.int64)
        cb = None if getattr(self, "placed", False) else np.empty(self.P + 1, np.int64)
        cells = np.empty((self.P, self.P), np.int64)
        self._check(load().fm_get_block_index(self._h, _vp(rb), _vp(cb), _vp(cells)))
        return rb, cb, cells

    def fm_get_stratum_nnz(self, s):
        n = ctypes.c_int64(0)
        self._check(load().fm_get_stratum_nnz(self._h, ctypes.c_int32(s), ctypes.byref(n)))
        return n.value

    def _get_stratum(self, fn, s, nmaj):
        n = self.fm_get_stratum_nnz(s)
        ptr = np.empty(nmaj + 1, np.int64)
        ind = np.empty(n, np.int32)
        val = np.empty(n, np.float32)
        self._check(fn(self._h, ctypes.c_int32(s), _vp(ptr), _vp(ind), _vp(val)))
        return ptr, ind, val

    def fm_get_stratum_csr(self, s):
        return self._get_stratum(load().fm_get_stratum_csr, s, self.N)

    def fm_get_stratum_csc(self, s):
        return self._get_stratum(load().fm_get_stratum_csc, s, self.D)

    def fm_partition_batches(self, B, stream=None):
        self._check(load().fm_partition_batches(self._h, ctypes.c_int32(B), _stream(stream)))
        self.B = int(B)

    def fm_get_batch_csc(self, b):
        colptr = np.empty(self.D + 1, np.int64)
        self._check(load().fm_get_batch_csc(self._h, ctypes.c_int32(b), _vp(colptr), _vp(None), _vp(None)))
        n = int(colptr[-1])
        row = np.empty(n, np.int32)
        val = np.empty(n, np.float32)
        self._check(load().fm_get_batch_csc(self._h, ctypes.c_int32(b), _vp(None), _vp(row), _vp(val)))
        return colptr, row, val

    # -- the pass
    def fm_forward(self, p: fm_params, y, w0, w, V, yhat=None, a=None, G=None, q=None, r=None,
                   want_loss=False, stream=None):
        N, D, K = self.N, self.D, p.K
        _dev(y, N, "y"); _dev(w0, 1, "w0"); _dev(w, D, "w"); _dev(V, D * K, "V")
        _dev(yhat, N, "yhat"); _dev(a, N, "a"); _dev(G, N * K, "G"); _dev(q, N, "q"); _dev(r, N, "r")
        loss = ctypes.c_double(0.0)
        self._check(load().fm_forward(self._h, ctypes.byref(p), _vp(y), _vp(w0), _vp(w), _vp(V), _vp(yhat),
                                      _vp(a), _vp(G), _vp(q), _vp(r),
                                      ctypes.byref(loss) if want_loss else ctypes.c_void_p(None), _stream(stream)))
        return loss.value if want_loss else None

    def fm_forward_noalloc(self, p: fm_params, y, w0, w, V, yhat=None, a=None, G=None, q=None, r=None,
                           sums=None, stream=None):
        """sums: float64 CUDA tensor of 2 elements (sum of losses, sum of multipliers) or None."""
        import torch
        N, D, K = self.N, self.D, p.K
        _dev(y, N, "y"); _dev(w0, 1, "w0"); _dev(w, D, "w"); _dev(V, D * K, "V")
        _dev(yhat, N, "yhat"); _dev(a, N, "a"); _dev(G, N * K, "G"); _dev(q, N, "q"); _dev(r, N, "r")
        if sums is not None and not (isinstance(sums, torch.Tensor) and sums.is_cuda and sums.dtype == torch.float64
                                     and sums.is_contiguous() and sums.numel() == 2):
            raise TypeError("sums must be a contiguous float64 CUDA tensor of 2 elements")
        self._check(load().fm_forward_noalloc(self._h, ctypes.byref(p), _vp(y), _vp(w0), _vp(w), _vp(V), _vp(yhat),
                                              _vp(a), _vp(G), _vp(q), _vp(r), _vp(sums), _stream(stream)))

    def fm_gradient(self, p: fm_params, r, G, w, V, grad_w0=None, grad_w=None, grad_V=None, stream=None):
        N, D, K = self.N, self.D, p.K
        _dev(r, N, "r"); _dev(G, N * K, "G"); _dev(w, D, "w"); _dev(V, D * K, "V")
        _dev(grad_w0, 1, "grad_w0"); _dev(grad_w, D, "grad_w"); _dev(grad_V, D * K, "grad_V")
        self._check(load().fm_gradient(self._h, ctypes.byref(p), _vp(r), _vp(G), _vp(w), _vp(V), _vp(grad_w0),
                                       _vp(grad_w), _vp(grad_V), _stream(stream)))

    def _epoch(self, fn, p, y, w0, w, V, want_objective, stream):
        N, D, K = self.N, self.D, p.K
        _dev(y, N, "y"); _dev(w0, 1, "w0"); _dev(w, D, "w"); _dev(V, D * K, "V")
        obj = (ctypes.c_double * 2)(0.0, 0.0)
        self._check(fn(self._h, ctypes.byref(p), _vp(y), _vp(w0), _vp(w), _vp(V),
                       obj if want_objective else ctypes.c_void_p(None), _stream(stream)))
        return (obj[0], obj[1]) if want_objective else None

    def fm_sgd_epoch(self, p, y, w0, w, V, want_objective=False, stream=None):
        return self._epoch(load().fm_sgd_epoch, p, y, w0, w, V, want_objective, stream)

    def fm_evaluate(self, p, y, w0, w, V, stream=None):
        _dev(y, self.N, "y"); _dev(w0, 1, "w0"); _dev(w, self.D, "w"); _dev(V, self.D * p.K, "V")
        out = (ctypes.c_double * 3)()
        self._check(load().fm_evaluate(self._h, ctypes.byref(p), _vp(y), _vp(w0), _vp(w), _vp(V), out,
                                       _stream(stream)))
        return dict(mean_loss=out[0], rmse=out[1], accuracy=out[2])

    def fm_minibatch_epoch(self, p, y, w0, w, V, want_objective=False, stream=None):
        return self._epoch(load().fm_minibatch_epoch, p, y, w0, w, V, want_objective, stream)

    def fm_stratified_epoch(self, p, y, w0, w, V, want_objective=False, stream=None):
        return self._epoch(load().fm_stratified_epoch, p, y, w0, w, V, want_objective, stream)

    def fm_stratified_begin(self, p, y, w0, w, V, stream=None):
        _dev(y, self.N, "y"); _dev(w0, 1, "w0"); _dev(w, self.D, "w"); _dev(V, self.D * p.K, "V")
        self._check(load().fm_stratified_begin(self._h, ctypes.byref(p), _vp(y), _vp(w0), _vp(w), _vp(V),
                                               _stream(stream)))

    def fm_stratified_step(self, p, s, y, w0, w, V, stream=None):
        _dev(y, self.N, "y"); _dev(w0, 1, "w0"); _dev(w, self.D, "w"); _dev(V, self.D * p.K, "V")
        self._check(load().fm_stratified_step(self._h, ctypes.byref(p), ctypes.c_int32(s), _vp(y), _vp(w0),
                                              _vp(w), _vp(V), _stream(stream)))

    def fm_stratified_end(self, p, w0, stream=None):
        _dev(w0, 1, "w0")
        self._check(load().fm_stratified_end(self._h, ctypes.byref(p), _vp(w0), _stream(stream)))

    def fm_get_aux(self, K, a=None, G=None, q=None, r=None, stream=None):
        _dev(a, self.N, "a"); _dev(G, self.N * K, "G"); _dev(q, self.N, "q"); _dev(r, self.N, "r")
        self._check(load().fm_get_aux(self._h, _vp(a), _vp(G), _vp(q), _vp(r), _stream(stream)))

    # -- per-kernel timing
    def fm_profile_enable(self, on=True):
        self._check(load().fm_profile_enable(self._h, ctypes.c_int32(1 if on else 0)))

    def fm_profile_read(self):
        lib = load()
        nk = lib.fm_profile_kernels()
        launches = np.zeros(nk, np.int64)
        ms = np.zeros(nk, np.float64)
        self._check(lib.fm_profile_read(self._h, _vp(launches), _vp(ms)))
        return {lib.fm_profile_kernel_name(ctypes.c_int32(k)).decode(): (int(launches[k]), float(ms[k]))
                for k in range(nk)}
