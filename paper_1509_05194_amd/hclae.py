"""ctypes binding of libhclae.so -- argument marshalling only.

Function names and argument order are those of ``include/hclae.h``; tensors are PyTorch CUDA
(ROCm) tensors used purely as device buffers, their ``data_ptr()`` is what crosses the ABI.
Every step of the method runs inside the library's HIP kernels; there is no fallback: if the
library is missing or fails to load, importing a symbol from it raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhclae.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE = 0, -1, -2, -3, -4
_ERRNAME = {0: "HCLAE_OK", -1: "HCLAE_EINVAL", -2: "HCLAE_ENOMEM", -3: "HCLAE_EHIP", -4: "HCLAE_ESTATE"}

EXPORTS = (
    "hclae_check_shape", "hclae_create", "hclae_destroy", "hclae_last_error",
    "hclae_encode", "hclae_anneal_stage", "hclae_sweep", "hclae_anneal", "hclae_quant_error", "hclae_quant_error_noalloc",
    "hclae_heat", "hclae_cool", "hclae_assign", "hclae_update", "hclae_last_refined", "hclae_work_counters",
    "hclae_timing_enable", "hclae_timing_read", "hclae_online_begin", "hclae_online_chunk",
    "hclae_online_export", "hclae_online_import",
    "hclae_covariance", "hclae_pca_axes", "hclae_symmetric_eigen", "hclae_rotate", "hclae_assign_prefix", "hclae_anneal_stage_pca", "hclae_dimension_schedule", "hclae_set_cooldown",
    "hclae_reorder_by_variance", "hclae_code_stats",
    "hclae_beam_step", "hclae_encode_beam", "hclae_set_beam_width", "hclae_set_contraction", "hclae_set_pruning",
)

KERNEL_CLASSES = ("heat", "cool", "assign", "refine", "accumulate", "merge", "norms", "error", "transition",
                  "rotate", "moments", "beam_score", "beam_expand", "accumulate_moved",
                  "assign_active", "bounds")


class KernelTimes(ctypes.Structure):
    _fields_ = [("ms", ctypes.c_double * len(KERNEL_CLASSES)),
                ("launches", ctypes.c_int64 * len(KERNEL_CLASSES))]


class StageStats(ctypes.Structure):
    _fields_ = [("err_before", ctypes.c_double), ("err_after", ctypes.c_double),
                ("codes_changed", ctypes.c_int64), ("refined", ctypes.c_int64),
                ("empty_clusters", ctypes.c_int32), ("iters_run", ctypes.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class HclaeError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("%s (%d): %s" % (_ERRNAME.get(code, "?"), code, text))
        self.code = code


_lib = None


def lib():
    """The loaded library.  Raises if libhclae.so has not been built (see build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libhclae.so is not built: run `python -m paper_1509_05194_amd.build`")
    # PyTorch ships its own HIP runtime (same soname).  Loading it first makes libhclae bind to
    # that one, so the process holds a single runtime and both see the same device and streams.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    L.hclae_check_shape.argtypes = [i64, i32, i32, i32]
    L.hclae_create.argtypes = [ctypes.POINTER(vp), i64, i32, i32, i32, vp]
    L.hclae_destroy.argtypes = [vp]
    L.hclae_last_error.argtypes = [vp]
    L.hclae_last_error.restype = ctypes.c_char_p
    L.hclae_encode.argtypes = [vp, vp, i64, i32, vp, i32, i32, vp, vp]
    L.hclae_anneal_stage.argtypes = [vp, i32, i64, i32, vp, i32, i32, vp, vp, i32, vp, ctypes.POINTER(StageStats)]
    L.hclae_sweep.argtypes = [vp, vp, i64, i32, vp, i32, i32, vp, vp, i32, i32, vp, vp]
    L.hclae_anneal.argtypes = [vp, i64, i32, vp, i32, i32, vp, vp, i32, i32, vp, vp]
    L.hclae_quant_error.argtypes = [vp, vp, i64, i32, ctypes.POINTER(ctypes.c_double)]
    L.hclae_quant_error_noalloc.argtypes = [vp, i64, i32, vp, vp]
    L.hclae_heat.argtypes = [vp, i32, i64, i32, vp, i32, i32, vp, vp]
    L.hclae_cool.argtypes = [vp, i32, i64, i32, vp, i32, i32, vp, vp]
    L.hclae_assign.argtypes = [vp, i32, i64, i32, vp, vp, i32, i32, vp, vp]
    L.hclae_update.argtypes = [vp, i32, i64, i32, vp, vp, i32, i32, vp, vp]
    L.hclae_last_refined.argtypes = [vp, ctypes.POINTER(i64)]
    L.hclae_work_counters.argtypes = [vp, ctypes.POINTER(i64), i32]
    L.hclae_online_begin.argtypes = [vp, vp, i32, i32, i32, vp]
    L.hclae_online_chunk.argtypes = [vp, vp, i64, i32, vp, i32, i32, vp, vp, vp, ctypes.POINTER(ctypes.c_double)]
    L.hclae_online_export.argtypes = [vp, vp, vp]
    L.hclae_online_import.argtypes = [vp, vp, vp]
    L.hclae_covariance.argtypes = [vp, vp, i64, i32, vp, vp]
    L.hclae_pca_axes.argtypes = [vp, vp, i64, i32, vp, vp]
    L.hclae_symmetric_eigen.argtypes = [vp, i32, vp, vp]
    L.hclae_rotate.argtypes = [vp, vp, i64, i32, vp, i32, vp]
    L.hclae_assign_prefix.argtypes = [vp, i32, i64, i32, vp, vp, i32, i32, i32, vp]
    L.hclae_anneal_stage_pca.argtypes = [vp, i32, i64, i32, vp, i32, i32, vp, vp, vp, vp, i32, i32, vp, vp,
                                         ctypes.POINTER(StageStats)]
    L.hclae_dimension_schedule.argtypes = [i32, i32, vp, vp]
    L.hclae_set_cooldown.argtypes = [vp, i32, i32]
    L.hclae_reorder_by_variance.argtypes = [vp, i64, i32, vp, i32, i32, vp, vp, vp]
    L.hclae_code_stats.argtypes = [vp, vp, i64, i32, i32, vp, i32, i32, vp]
    L.hclae_beam_step.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i32, vp, vp, vp, vp]
    L.hclae_encode_beam.argtypes = [vp, vp, i64, i32, vp, i32, i32, i32, vp, vp, vp]
    L.hclae_set_beam_width.argtypes = [vp, i32]
    L.hclae_set_contraction.argtypes = [vp, i32]
    L.hclae_set_pruning.argtypes = [vp, i32]
    L.hclae_timing_enable.argtypes = [vp, ctypes.c_uint32]
    L.hclae_timing_read.argtypes = [vp, ctypes.POINTER(KernelTimes)]
    for name in EXPORTS:
        if name != "hclae_last_error":
            getattr(L, name).restype = i32
    _lib = L
    return L


def check_shape(N, D, M, K):
    return lib().hclae_check_shape(N, D, M, K)


def quant_error_noalloc(residue, out, stream=None):
    """hclae_quant_error_noalloc: residue CUDA float32 [N][D], out CUDA float64 tensor of one element (written on
    `stream`, default torch's current stream; no synchronisation)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    N, D = residue.shape
    rc = lib().hclae_quant_error_noalloc(_ptr(residue, "f32"), N, D, _ptr(out, "f64", (1,)), ctypes.c_void_p(stream))
    if rc != OK:
        raise HclaeError(rc, lib().hclae_last_error(None).decode())


def dimension_schedule(D, phases=10):
    """The prefixes d_i = ceil(D^(i/phases)) of the improved k-means (Sec. 3.2), equal values once, the last one D."""
    dims = np.zeros(phases, np.int32)
    n = ctypes.c_int()
    rc = lib().hclae_dimension_schedule(D, phases, dims.ctypes.data_as(ctypes.c_void_p), ctypes.byref(n))
    if rc != OK:
        raise HclaeError(rc, "hclae_dimension_schedule")
    return dims[:n.value].copy()


def symmetric_eigen(A):
    """(w float64 [n] descending, Vt float64 [n][n], rows = eigenvectors) of a symmetric host matrix; no device."""
    A = np.ascontiguousarray(A, np.float64)
    n = A.shape[0]
    assert A.shape == (n, n)
    w = np.zeros(n, np.float64)
    Vt = np.zeros((n, n), np.float64)
    rc = lib().hclae_symmetric_eigen(A.ctypes.data_as(ctypes.c_void_p), n, w.ctypes.data_as(ctypes.c_void_p),
                                     Vt.ctypes.data_as(ctypes.c_void_p))
    if rc != OK:
        raise HclaeError(rc, "hclae_symmetric_eigen")
    return w, Vt


def _ptr(t, dtype_name, shape=None):
    """Device pointer of a contiguous CUDA tensor of the expected dtype (None -> NULL)."""
    if t is None:
        return None
    import torch
    want = {"f32": torch.float32, "u8": torch.uint8, "i32": torch.int32, "f64": torch.float64}[dtype_name]
    if not (t.is_cuda and t.dtype == want and t.is_contiguous()):
        raise TypeError("expected a contiguous CUDA %s tensor" % dtype_name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("tensor shape %s, expected %s" % (tuple(t.shape), tuple(shape)))
    return ctypes.c_void_p(t.data_ptr())


class Context:
    """An hclae_ctx bound to one HIP stream (default: torch's current stream)."""

    def __init__(self, N_max, D, M, K, stream=None):
        import torch
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.N_max, self.D, self.M, self.K = int(N_max), int(D), int(M), int(K)
        self._h = ctypes.c_void_p()
        rc = lib().hclae_create(ctypes.byref(self._h), self.N_max, self.D, self.M, self.K, ctypes.c_void_p(stream))
        if rc != OK:
            raise HclaeError(rc, lib().hclae_last_error(None).decode())

    def close(self):
        if self._h:
            lib().hclae_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc):
        if rc != OK:
            raise HclaeError(rc, lib().hclae_last_error(self._h).decode())

    def _shapes(self, N, C=None, codes=None, res=None):
        D, M, K = self.D, self.M, self.K
        return (_ptr(C, "f32", (M, K, D)) if C is not None else None,
                _ptr(codes, "u8", (N, M)) if codes is not None else None,
                _ptr(res, "f32", (N, D)) if res is not None else None)

    # ---- the four calls of the method -------------------------------------------------
    def encode(self, X, C, codes, residue):
        N = X.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        self._chk(lib().hclae_encode(self._h, _ptr(X, "f32", (N, self.D)), N, self.D, pC, self.M, self.K, pcodes, pres))

    def beam_step(self, rows, err, Cm, L, rows_next, err_next=None, parent=None, code=None):
        """One dictionary of the multi-path encoding: rows f32 [N][Lc][D], err f64 [N][Lc] or None."""
        N, Lc = rows.shape[0], rows.shape[1]
        Ln = min(L, self.K * Lc)
        self._chk(lib().hclae_beam_step(
            self._h, _ptr(rows, "f32", (N, Lc, self.D)), _ptr(err, "f64", (N, Lc)), _ptr(Cm, "f32", (self.K, self.D)),
            N, self.D, self.K, Lc, L, _ptr(rows_next, "f32", (N, Ln, self.D)), _ptr(err_next, "f64", (N, Ln)),
            _ptr(parent, "u8", (N, Ln)), _ptr(code, "u8", (N, Ln))))

    def encode_beam(self, X, C, L, codes, residue, err=None):
        N = X.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        self._chk(lib().hclae_encode_beam(self._h, _ptr(X, "f32", (N, self.D)), N, self.D, pC, self.M, self.K, L,
                                          pcodes, pres, _ptr(err, "f64", (N,))))

    def set_pruning(self, on):
        """Exact pruning of the Lloyd iterations of a stage (default on; same results either way)."""
        self._chk(lib().hclae_set_pruning(self._h, 1 if on else 0))

    def set_cooldown(self, improved, phases=10):
        """The k-means that cools a dictionary in anneal_stage / sweep: plain Lloyd, or the improved one of Sec. 3.2."""
        self._chk(lib().hclae_set_cooldown(self._h, 1 if improved else 0, phases))

    def set_contraction(self, mode):
        """0: fp32 MFMA; 1: split-bf16 MFMA (same results, see hclae_set_contraction)."""
        self._chk(lib().hclae_set_contraction(self._h, mode))

    def set_beam_width(self, L):
        self._chk(lib().hclae_set_beam_width(self._h, L))

    def anneal_stage(self, m, C, codes, residue, iters, init_idx=None, want_stats=True):
        N = residue.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        idx = None
        if init_idx is not None:
            idx = np.ascontiguousarray(init_idx, np.int64)
            assert idx.shape == (self.K,)
        stats = StageStats() if want_stats else None
        self._chk(lib().hclae_anneal_stage(self._h, m, N, self.D, pC, self.M, self.K, pcodes, pres, iters,
                                           idx.ctypes.data_as(ctypes.c_void_p) if idx is not None else None,
                                           ctypes.byref(stats) if want_stats else None))
        return stats.as_dict() if want_stats else None

    def sweep(self, C, codes, residue, iters, X=None, reencode_mode=0, init_idx=None, want_err=True):
        N = residue.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        idx = None
        if init_idx is not None:
            idx = np.ascontiguousarray(init_idx, np.int64)
            assert idx.shape == (self.M, self.K)
        err = np.zeros(self.M, np.float64) if want_err else None
        self._chk(lib().hclae_sweep(self._h, _ptr(X, "f32", (N, self.D)), N, self.D, pC, self.M, self.K, pcodes, pres,
                                    iters, reencode_mode,
                                    idx.ctypes.data_as(ctypes.c_void_p) if idx is not None else None,
                                    err.ctypes.data_as(ctypes.c_void_p) if want_err else None))
        return err

    def anneal(self, C, codes, residue, iters, n_sweeps, init_idx=None, want_err=True):
        N = residue.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        idx = None
        if init_idx is not None:
            idx = np.ascontiguousarray(init_idx, np.int64)
            assert idx.shape == (self.M, self.K)
        err = np.zeros((n_sweeps, self.M), np.float64) if want_err else None
        self._chk(lib().hclae_anneal(self._h, N, self.D, pC, self.M, self.K, pcodes, pres, iters, n_sweeps,
                                     idx.ctypes.data_as(ctypes.c_void_p) if idx is not None else None,
                                     err.ctypes.data_as(ctypes.c_void_p) if want_err else None))
        return err

    def quant_error(self, residue):
        N = residue.shape[0]
        out = ctypes.c_double()
        self._chk(lib().hclae_quant_error(self._h, _ptr(residue, "f32", (N, self.D)), N, self.D, ctypes.byref(out)))
        return out.value

    # ---- single steps -------------------------------------------------------------------
    def heat(self, m, C, codes, residue):
        N = residue.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        self._chk(lib().hclae_heat(self._h, m, N, self.D, pC, self.M, self.K, pcodes, pres))

    def cool(self, m, C, codes, xp):
        N = xp.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, xp)
        self._chk(lib().hclae_cool(self._h, m, N, self.D, pC, self.M, self.K, pcodes, pres))

    def assign(self, m, xp, C, codes, dmin=None):
        N = xp.shape[0]
        pC, pcodes, pxp = self._shapes(N, C, codes, xp)
        self._chk(lib().hclae_assign(self._h, m, N, self.D, pxp, pC, self.M, self.K, pcodes, _ptr(dmin, "f32", (N,))))

    def update(self, m, xp, C, codes, counts=None):
        N = xp.shape[0]
        pC, pcodes, pxp = self._shapes(N, C, codes, xp)
        self._chk(lib().hclae_update(self._h, m, N, self.D, pxp, pC, self.M, self.K, pcodes, _ptr(counts, "i32", (self.K,))))

    def last_refined(self):
        out = ctypes.c_int64()
        self._chk(lib().hclae_last_refined(self._h, ctypes.byref(out)))
        return out.value

    def work_counters(self, reset=False):
        """(assignments run, vectors they recomputed, vectors decided by the fp64 re-check) since the last reset."""
        out = (ctypes.c_int64 * 3)()
        self._chk(lib().hclae_work_counters(self._h, out, 1 if reset else 0))
        return int(out[0]), int(out[1]), int(out[2])

    # ---- online learning -----------------------------------------------------------------
    def online_begin(self, C, n0=None):
        pC, _, _ = self._shapes(0, C)
        w = None
        if n0 is not None:
            w = np.ascontiguousarray(n0, np.int64)
            assert w.shape == (self.M, self.K)
        self._chk(lib().hclae_online_begin(self._h, pC, self.M, self.K, self.D,
                                           w.ctypes.data_as(ctypes.c_void_p) if w is not None else None))

    def online_export(self):
        S = np.empty((self.M, self.K, self.D), np.float64)
        cnt = np.empty((self.M, self.K), np.int64)
        self._chk(lib().hclae_online_export(self._h, S.ctypes.data_as(ctypes.c_void_p), cnt.ctypes.data_as(ctypes.c_void_p)))
        return S, cnt

    def online_import(self, S, cnt):
        S = np.ascontiguousarray(S, np.float64)
        cnt = np.ascontiguousarray(cnt, np.int64)
        assert S.shape == (self.M, self.K, self.D) and cnt.shape == (self.M, self.K)
        self._chk(lib().hclae_online_import(self._h, S.ctypes.data_as(ctypes.c_void_p), cnt.ctypes.data_as(ctypes.c_void_p)))

    def online_chunk(self, Xu8, C, codes, residue, want_err=False, codes_first=None):
        n = Xu8.shape[0]
        if not (Xu8.is_cuda and Xu8.is_contiguous() and tuple(Xu8.shape) == (n, self.D) and str(Xu8.dtype) == "torch.uint8"):
            raise TypeError("expected a contiguous CUDA uint8 tensor [n][D]")
        pC, pcodes, pres = self._shapes(n, C, codes, residue)
        err = ctypes.c_double()
        self._chk(lib().hclae_online_chunk(self._h, ctypes.c_void_p(Xu8.data_ptr()), n, self.D, pC, self.M, self.K,
                                           pcodes, pres, _ptr(codes_first, "u8", (n, self.M)),
                                           ctypes.byref(err) if want_err else None))
        return err.value if want_err else None

    # ---- improved k-means (Sec. 3.2) -----------------------------------------------------
    def covariance(self, xp):
        """(mean float64 [D], cov float64 [D][D]) of the rows of xp, as CUDA tensors."""
        import torch
        N = xp.shape[0]
        mean = torch.empty(self.D, dtype=torch.float64, device=xp.device)
        cov = torch.empty((self.D, self.D), dtype=torch.float64, device=xp.device)
        self._chk(lib().hclae_covariance(self._h, _ptr(xp, "f32", (N, self.D)), N, self.D,
                                         ctypes.c_void_p(mean.data_ptr()), ctypes.c_void_p(cov.data_ptr())))
        return mean, cov

    def pca_axes(self, xp):
        """(R float32 [D][D] CUDA tensor, rows = principal axes; eigenvalues float64 [D] NumPy, descending)."""
        import torch
        N = xp.shape[0]
        R = torch.empty((self.D, self.D), dtype=torch.float32, device=xp.device)
        w = np.zeros(self.D, np.float64)
        self._chk(lib().hclae_pca_axes(self._h, _ptr(xp, "f32", (N, self.D)), N, self.D, _ptr(R, "f32"),
                                       w.ctypes.data_as(ctypes.c_void_p)))
        return R, w

    def rotate(self, x, R, out, transpose=False):
        N = x.shape[0]
        self._chk(lib().hclae_rotate(self._h, _ptr(x, "f32", (N, self.D)), N, self.D, _ptr(R, "f32", (self.D, self.D)),
                                     1 if transpose else 0, _ptr(out, "f32", (N, self.D))))

    def assign_prefix(self, m, xp, C, codes, dact):
        N = xp.shape[0]
        pC, pcodes, pxp = self._shapes(N, C, codes, xp)
        self._chk(lib().hclae_assign_prefix(self._h, m, N, self.D, pxp, pC, self.M, self.K, int(dact), pcodes))

    def anneal_stage_pca(self, m, C, codes, residue, R, dims, iters_per_dim, xr, init_idx=None, want_stats=True):
        N = residue.shape[0]
        pC, pcodes, pres = self._shapes(N, C, codes, residue)
        dims = np.ascontiguousarray(dims, np.int32)
        idx = None
        if init_idx is not None:
            idx = np.ascontiguousarray(init_idx, np.int64)
            assert idx.shape == (self.K,)
        stats = StageStats() if want_stats else None
        self._chk(lib().hclae_anneal_stage_pca(
            self._h, m, N, self.D, pC, self.M, self.K, pcodes, pres,
            _ptr(R, "f32", (self.D, self.D)) if R is not None else None,
            dims.ctypes.data_as(ctypes.c_void_p), len(dims), iters_per_dim, _ptr(xr, "f32", (N, self.D)),
            idx.ctypes.data_as(ctypes.c_void_p) if idx is not None else None,
            ctypes.byref(stats) if want_stats else None))
        return stats.as_dict() if want_stats else None

    # ---- dictionary order and code statistics ---------------------------------------------
    def reorder_by_variance(self, C, codes):
        """Permutes C and the code columns in place; returns (variances in the old order, order)."""
        N = codes.shape[0]
        pC, pcodes, _ = self._shapes(N, C, codes)
        var = np.zeros(self.M, np.float64)
        order = np.zeros(self.M, np.int32)
        self._chk(lib().hclae_reorder_by_variance(self._h, N, self.D, pC, self.M, self.K, pcodes,
                                                  var.ctypes.data_as(ctypes.c_void_p), order.ctypes.data_as(ctypes.c_void_p)))
        return var, order

    def code_stats(self, codes, pair=None):
        """hist int64 [M][K] and, for pair=(a, b), the joint counts int64 [K][K] (else None)."""
        N = codes.shape[0]
        _, pcodes, _ = self._shapes(N, None, codes)
        hist = np.zeros((self.M, self.K), np.int64)
        joint = np.zeros((self.K, self.K), np.int64) if pair is not None else None
        a, b = pair if pair is not None else (0, 0)
        self._chk(lib().hclae_code_stats(self._h, pcodes, N, self.M, self.K, hist.ctypes.data_as(ctypes.c_void_p), a, b,
                                         joint.ctypes.data_as(ctypes.c_void_p) if joint is not None else None))
        return hist, joint

    def timing_enable(self, classes):
        """classes: iterable of names from KERNEL_CLASSES (empty = off)."""
        mask = 0
        for c in classes:
            mask |= 1 << KERNEL_CLASSES.index(c)
        self._chk(lib().hclae_timing_enable(self._h, mask))

    def timing_read(self):
        """{class: (total ms, launches)} since the last read."""
        kt = KernelTimes()
        self._chk(lib().hclae_timing_read(self._h, ctypes.byref(kt)))
        return {c: (kt.ms[i], kt.launches[i]) for i, c in enumerate(KERNEL_CLASSES)}
