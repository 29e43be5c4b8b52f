"""ctypes front-end of the plain CPU oracle of Dictionary Annealing (``da_oracle.c``).

TEST INFRASTRUCTURE ONLY: the product path never imports this package.  Callers are the
tests, the smoke check and the benchmark's ``cpu_baseline`` leg.

State is kept in float64 NumPy arrays (``C[M][K][D]``, ``r[N][D]``) and uint8 codes
``[N][M]``; every function mutates its arrays in place like the C routines do.  See the
header of ``da_oracle.c`` for the passages of the paper (arXiv 1509.05194, Sec. 3.1-3.3)
each routine follows.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "da_oracle.c")
_LIB = os.path.join(_HERE, "libda_oracle.so")
# The mutation tests (tests/test_oracle_mutations.py) point this at a copy of da_oracle.c with one planted
# mistake and check that the pins notice it.
if os.environ.get("DA_ORACLE_SRC"):
    _SRC = os.environ["DA_ORACLE_SRC"]
    _LIB = _SRC + ".so"
_lib = None


def build(force=True):
    """Compile the oracle with gcc: -O2, OpenMP, no fast-math, no FP contraction."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
           "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_f64p = ctypes.POINTER(ctypes.c_double)
_f32p = ctypes.POINTER(ctypes.c_float)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_i64 = ctypes.c_int64
_int = ctypes.c_int


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    lib.da_oracle_threads.restype = _int
    lib.da_oracle_set_threads.argtypes = [_int]
    lib.da_heat.argtypes = [_f64p, _u8p, _f64p, _i64, _int, _int, _int, _int]
    lib.da_cool.argtypes = [_f64p, _u8p, _f64p, _i64, _int, _int, _int, _int]
    lib.da_assign.argtypes = [_f64p, _f64p, _i64, _int, _int, _int, _int, _u8p, _f64p, _f64p, _i32p]
    lib.da_beam_step.argtypes = [_f32p, _f64p, _i64, _int, _int, _int, _int, _f64p, _u8p, _u8p, _f64p,
                                 _f64p, _f64p]
    lib.da_encode_beam.argtypes = [_f32p, _f64p, _i64, _int, _int, _int, _int, _u8p, _f64p, _f64p, _f64p]
    lib.da_dist_to.argtypes = [_f64p, _f64p, _i64, _int, _int, _int, _int]
    lib.da_dist_to.restype = ctypes.c_double
    lib.da_update.argtypes = [_f64p, _u8p, _f64p, _i64, _int, _int, _int, _int, _i64p]
    lib.da_update.restype = _int
    lib.da_quant_error.argtypes = [_f64p, _i64, _int]
    lib.da_quant_error.restype = ctypes.c_double
    lib.da_encode.argtypes = [_f32p, _f64p, _i64, _int, _int, _int, _u8p, _f64p]
    lib.da_anneal_stage.argtypes = [_int, _f64p, _u8p, _f64p, _i64, _int, _int, _int, _int, _i64p, _f64p]
    lib.da_anneal_stage.restype = ctypes.c_double
    lib.da_sweep.argtypes = [_f64p, _u8p, _f64p, _i64, _int, _int, _int, _int, _i64p, _f64p]
    lib.da_reconstruct.argtypes = [_f64p, _u8p, _i64, _int, _int, _int, _f64p]
    lib.da_rotate.argtypes = [_f64p, _i64, _int, _f64p, _int, _f64p]
    lib.da_anneal_stage_pca.argtypes = [_int, _f64p, _u8p, _f64p, _i64, _int, _int, _int, _f64p,
                                        ctypes.POINTER(ctypes.c_int), _int, _int, _i64p]
    lib.da_anneal_stage_pca.restype = ctypes.c_double
    lib.da_online_chunk.argtypes = [_u8p, _i64, _int, _int, _int, _f64p, _f64p, _i64p, _u8p, _f64p]
    lib.da_online_chunk.restype = ctypes.c_double
    _lib = lib
    return lib


def _chk(a, dtype, shape=None):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], \
        "expected a C-contiguous %s array" % np.dtype(dtype).name
    if shape is not None:
        assert tuple(a.shape) == tuple(shape), "shape %s, expected %s" % (a.shape, shape)
    return a


def _p(a, ptype):
    return None if a is None else a.ctypes.data_as(ptype)


def _dims(C, codes, r):
    M, K, D = C.shape
    N = r.shape[0]
    _chk(C, np.float64)
    _chk(codes, np.uint8, (N, M))
    _chk(r, np.float64, (N, D))
    return N, D, M, K


def threads():
    return _load().da_oracle_threads()


def set_threads(t):
    _load().da_oracle_set_threads(int(t))


def heat(r, codes, C, m):
    N, D, M, K = _dims(C, codes, r)
    _load().da_heat(_p(r, _f64p), _p(codes, _u8p), _p(C, _f64p), N, D, M, K, m)


def cool(xp, codes, C, m):
    N, D, M, K = _dims(C, codes, xp)
    _load().da_cool(_p(xp, _f64p), _p(codes, _u8p), _p(C, _f64p), N, D, M, K, m)


def assign(xp, C, codes, m, top2=False):
    """Nearest codeword of dictionary m; writes codes[:, m].
    With top2=True also returns (d1, d2, i2): best / second-best squared distance and the
    index of the second best."""
    N, D, M, K = _dims(C, codes, xp)
    if top2:
        d1 = np.empty(N, np.float64)
        d2 = np.empty(N, np.float64)
        i2 = np.empty(N, np.int32)
    else:
        d1 = d2 = i2 = None
    _load().da_assign(_p(xp, _f64p), _p(C, _f64p), N, D, M, K, m, _p(codes, _u8p),
                      _p(d1, _f64p), _p(d2, _f64p), _p(i2, _i32p))
    return (d1, d2, i2) if top2 else None


def dist_to(xp, C, n, m, k):
    M, K, D = C.shape
    return _load().da_dist_to(_p(xp, _f64p), _p(C, _f64p), int(n), D, K, m, int(k))


def update(xp, codes, C, m):
    """Centroid update of dictionary m in place; returns (counts[K] int64, n_empty)."""
    N, D, M, K = _dims(C, codes, xp)
    counts = np.zeros(K, np.int64)
    empty = _load().da_update(_p(xp, _f64p), _p(codes, _u8p), _p(C, _f64p), N, D, M, K, m,
                              _p(counts, _i64p))
    return counts, empty


def quant_error(r):
    _chk(r, np.float64)
    N, D = r.shape
    return _load().da_quant_error(_p(r, _f64p), N, D)


def encode(X, C):
    """Greedy (single-path) residual encoding.  Returns (codes uint8 [N][M], r float64 [N][D])."""
    _chk(X, np.float32)
    _chk(C, np.float64)
    N, D = X.shape
    M, K, D2 = C.shape
    assert D == D2
    codes = np.zeros((N, M), np.uint8)
    r = np.empty((N, D), np.float64)
    _load().da_encode(_p(X, _f32p), _p(C, _f64p), N, D, M, K, _p(codes, _u8p), _p(r, _f64p))
    return codes, r


def beam_step(X, Cm, A, L):
    """One dictionary of the multi-path encoding (Sec. 3.3): A float64 [N][Lc][D] are the kept
    sums so far.  Returns (parent uint8 [N][Ln], code uint8 [N][Ln], err float64 [N][Ln],
    A_next float64 [N][Ln][D], gap float64 [N]) with Ln = min(L, K * Lc)."""
    _chk(X, np.float32)
    _chk(Cm, np.float64)
    _chk(A, np.float64)
    N, D = X.shape
    K = Cm.shape[0]
    Lc = A.shape[1]
    assert Cm.shape == (K, D) and A.shape == (N, Lc, D) and L >= 1
    Ln = min(L, K * Lc)
    parent = np.zeros((N, Ln), np.uint8)
    code = np.zeros((N, Ln), np.uint8)
    err = np.zeros((N, Ln), np.float64)
    A_next = np.zeros((N, Ln, D), np.float64)
    gap = np.zeros(N, np.float64)
    _load().da_beam_step(_p(X, _f32p), _p(Cm, _f64p), N, D, K, Lc, L, _p(A, _f64p), _p(parent, _u8p),
                         _p(code, _u8p), _p(err, _f64p), _p(A_next, _f64p), _p(gap, _f64p))
    return parent, code, err, A_next, gap


def encode_beam(X, C, L):
    """Multi-path encoding with L paths (Sec. 3.3).  Returns (codes uint8 [N][M], r float64
    [N][D], err float64 [N], gap float64 [N])."""
    _chk(X, np.float32)
    _chk(C, np.float64)
    N, D = X.shape
    M, K, D2 = C.shape
    assert D == D2 and L >= 1
    codes = np.zeros((N, M), np.uint8)
    r = np.empty((N, D), np.float64)
    err = np.zeros(N, np.float64)
    gap = np.zeros(N, np.float64)
    _load().da_encode_beam(_p(X, _f32p), _p(C, _f64p), N, D, M, K, L, _p(codes, _u8p), _p(r, _f64p),
                           _p(err, _f64p), _p(gap, _f64p))
    return codes, r, err, gap


def anneal_stage(m, C, codes, r, T, init_idx=None, trace=False):
    """One DA iteration on dictionary m, in place.  Returns E after the stage, or (E, J)
    with the 2T+2 objective values when trace=True."""
    N, D, M, K = _dims(C, codes, r)
    if init_idx is not None:
        init_idx = np.ascontiguousarray(init_idx, np.int64)
        assert init_idx.shape == (K,) and init_idx.min() >= 0 and init_idx.max() < N
    J = np.zeros(2 * T + 2, np.float64) if trace else None
    E = _load().da_anneal_stage(m, _p(C, _f64p), _p(codes, _u8p), _p(r, _f64p), N, D, M, K, T,
                                _p(init_idx, _i64p), _p(J, _f64p))
    return (E, J) if trace else E


def sweep(C, codes, r, T, init_idx=None):
    """Stages m = 0..M-1 in order, in place.  Returns E after each stage (float64[M])."""
    N, D, M, K = _dims(C, codes, r)
    if init_idx is not None:
        init_idx = np.ascontiguousarray(init_idx, np.int64)
        assert init_idx.shape == (M, K) and init_idx.min() >= 0 and init_idx.max() < N
    err = np.zeros(M, np.float64)
    _load().da_sweep(_p(C, _f64p), _p(codes, _u8p), _p(r, _f64p), N, D, M, K, T,
                     _p(init_idx, _i64p), _p(err, _f64p))
    return err


def reconstruct(C, codes):
    _chk(C, np.float64)
    M, K, D = C.shape
    N = codes.shape[0]
    _chk(codes, np.uint8, (N, M))
    xhat = np.empty((N, D), np.float64)
    _load().da_reconstruct(_p(C, _f64p), _p(codes, _u8p), N, D, M, K, _p(xhat, _f64p))
    return xhat


def online_chunk(X_u8, C, S, cnt):
    """One online chunk (uint8 [n][D]) against running sums S float64 [M][K][D] and counts
    int64 [M][K], all updated in place together with C.  Returns (codes, residue, E)."""
    _chk(X_u8, np.uint8)
    _chk(C, np.float64)
    M, K, D = C.shape
    n = X_u8.shape[0]
    assert X_u8.shape == (n, D)
    _chk(S, np.float64, (M, K, D))
    _chk(cnt, np.int64, (M, K))
    codes = np.zeros((n, M), np.uint8)
    r = np.empty((n, D), np.float64)
    E = _load().da_online_chunk(_p(X_u8, _u8p), n, D, M, K, _p(C, _f64p), _p(S, _f64p), _p(cnt, _i64p),
                                _p(codes, _u8p), _p(r, _f64p))
    return codes, r, E


def rotate(x, R, transpose=False):
    """y_n = R x_n (or R^T x_n); x float64 [N][D], R float64 [D][D] with the axes as rows."""
    _chk(x, np.float64)
    N, D = x.shape
    _chk(R, np.float64, (D, D))
    y = np.empty_like(x)
    _load().da_rotate(_p(x, _f64p), N, D, _p(R, _f64p), 1 if transpose else 0, _p(y, _f64p))
    return y


def dimension_schedule(D, I=10):
    """d_i = ceil(D^(i/I)), i = 1..I, duplicates removed (Sec. 3.2: d_i = d^(i/I), I = 10)."""
    out = []
    for i in range(1, I + 1):
        d = int(np.ceil(D ** (i / I) - 1e-9))
        d = max(1, min(D, d))
        if not out or d > out[-1]:
            out.append(d)
    out[-1] = D
    return np.array(out, np.int32)


def anneal_stage_pca(m, C, codes, r, R, dims, T, init_idx=None):
    """One DA iteration on dictionary m with the improved k-means of Sec. 3.2 as cool-down."""
    N, D, M, K = _dims(C, codes, r)
    _chk(R, np.float64, (D, D))
    dims = np.ascontiguousarray(dims, np.int32)
    assert dims[-1] == D and np.all(np.diff(dims) > 0) and dims[0] >= 1
    if init_idx is not None:
        init_idx = np.ascontiguousarray(init_idx, np.int64)
        assert init_idx.shape == (K,)
    return _load().da_anneal_stage_pca(m, _p(C, _f64p), _p(codes, _u8p), _p(r, _f64p), N, D, M, K, _p(R, _f64p),
                                       dims.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), len(dims), T,
                                       _p(init_idx, _i64p))


def pca_axes(xp):
    """Principal axes of {x'} as rows of R (most variance first): eigenvectors of the centred
    covariance, LAPACK via NumPy; each axis is signed so that its largest-magnitude entry is positive."""
    x = np.asarray(xp, np.float64)
    cov = np.cov(x, rowvar=False, bias=True)
    w, V = np.linalg.eigh(cov)
    order = np.argsort(-w, kind="stable")
    R = V[:, order].T.copy()
    for i in range(R.shape[0]):
        j = np.argmax(np.abs(R[i]))
        if R[i, j] < 0:
            R[i] = -R[i]
    return np.ascontiguousarray(R)


# ---- dictionary order and code statistics (Sec. 3.3, Sec. 2.2): plain NumPy definitions ----------
def dictionary_variances(C):
    """var_m = (1/K) sum_k ||c_m(k) - mean_k c_m||^2 (the reading taken of "variance of a dictionary's elements")."""
    C = np.asarray(C, np.float64)
    return ((C - C.mean(axis=1, keepdims=True)) ** 2).sum(axis=2).mean(axis=1)


def variance_order(C):
    """Dictionaries in descending variance; ties keep the lower index.  order[j] = old index at new position j."""
    v = dictionary_variances(C)
    return np.array(sorted(range(len(v)), key=lambda j: (-v[j], j)), np.int32)


def code_histogram(codes, K):
    return np.stack([np.bincount(codes[:, m], minlength=K) for m in range(codes.shape[1])]).astype(np.int64)


def joint_histogram(codes, a, b, K):
    J = np.zeros((K, K), np.int64)
    np.add.at(J, (codes[:, a].astype(np.int64), codes[:, b].astype(np.int64)), 1)
    return J


def entropy_bits(counts):
    """Plug-in entropy of a count table, in bits (Sec. 2.2: self-information of a code part)."""
    c = np.asarray(counts, np.float64).reshape(-1)
    p = c[c > 0] / c.sum()
    return float(-(p * np.log2(p)).sum())


def mutual_information_bits(joint):
    """I(A;B) = H(A) + H(B) - H(A,B) from the joint count table."""
    J = np.asarray(joint, np.float64)
    return entropy_bits(J.sum(1)) + entropy_bits(J.sum(0)) - entropy_bits(J)
