"""Seeded synthetic inputs shaped like the paper's workloads (arXiv 1509.05194, Sec. 5.1:
128-d SIFT descriptors, 960-d GIST descriptors).  None of those datasets is used or
reproduced; these generators only imitate shape, value range, sparsity and norm scale.

This module holds no arithmetic of the method itself.  It is the one piece shared by the
GPU path's harness and the CPU oracle's tests: both sides read the arrays produced here.

Every generator is keyed by (seed, row block) so any row range can be produced on its own
and concatenating ranges gives the same rows as one call.
"""
import numpy as np

_BLOCK = 1 << 16          # rows per independently keyed block

SEED_DATA = 150905194
SEED_INIT = 5194
SEED_HELDOUT = 5195


def _rng(seed, tag, block=0):
    # The block id goes into the third 64-bit word of Philox's 256-bit counter: the streams of two blocks start
    # 2^128 draws apart.  (In the lowest word they would start ONE counter step apart, each block's stream being
    # the previous block's shifted by four draws.)
    return np.random.Generator(np.random.Philox(key=[int(seed), int(tag)], counter=[0, 0, int(block), 0]))


def _blocks(start, count):
    """Yield (block id, first row inside the block, rows to take, output offset)."""
    out = 0
    row = start
    end = start + count
    while row < end:
        b = row // _BLOCK
        lo = row - b * _BLOCK
        take = min(_BLOCK - lo, end - row)
        yield b, lo, take, out
        out += take
        row += take


def tiny_gmm(N=10000, D=16, components=32, sigma=0.1, seed=SEED_DATA, start=0):
    """Isotropic Gaussian mixture, equal weights, means ~ U[-1,1]^D, fp32."""
    g = _rng(seed, 1)
    means = g.uniform(-1.0, 1.0, size=(components, D))
    X = np.empty((N, D), np.float32)
    for b, lo, take, out in _blocks(start, N):
        r = _rng(seed, 2, b)
        comp = r.integers(0, components, size=_BLOCK)
        z = r.standard_normal(size=(_BLOCK, D))
        blk = means[comp] + sigma * z
        X[out:out + take] = blk[lo:lo + take].astype(np.float32)
    return X


def _sift_params(D, components, seed):
    g = _rng(seed, 11)
    w = g.uniform(0.2, 1.0, size=components)
    w = w / w.sum()
    mu = 38.0 * g.exponential(1.0, size=(components, D)) - 12.7
    sig = g.uniform(6.0, 14.0, size=components)
    return w, mu, sig


def sift_like(N, D=128, components=256, seed=SEED_DATA, start=0, dtype=np.float32):
    """Integer-valued vectors in [0,255]: a Gaussian mixture whose component means follow a
    non-negative heavy-tailed (shifted exponential) profile, clipped and rounded; about 30 %
    of the entries are zero and the mean L2 norm is about 500.  dtype float32 or uint8."""
    w, mu, sig = _sift_params(D, components, seed)
    cdf = np.cumsum(w)
    cdf[-1] = 1.0
    X = np.empty((N, D), dtype)
    for b, lo, take, out in _blocks(start, N):
        r = _rng(seed, 12, b)
        comp = np.searchsorted(cdf, r.random(size=_BLOCK), side="right")
        comp = comp[lo:lo + take]
        z = r.standard_normal(size=(_BLOCK, D), dtype=np.float32)[lo:lo + take]
        blk = mu[comp].astype(np.float32) + sig[comp].astype(np.float32)[:, None] * z
        np.clip(blk, 0.0, 255.0, out=blk)
        np.rint(blk, out=blk)
        X[out:out + take] = blk.astype(dtype)
    return X


def gist_like(N, D=960, components=512, rank=64, seed=SEED_DATA, start=0):
    """fp32 vectors in [0,1] with rank-`rank` correlated structure plus noise 0.02, clipped."""
    g = _rng(seed, 21)
    B = g.standard_normal(size=(rank, D)) / np.sqrt(rank)
    A = g.standard_normal(size=(components, rank))
    B32 = B.astype(np.float32)
    X = np.empty((N, D), np.float32)
    for b, lo, take, out in _blocks(start, N):
        r = _rng(seed, 22, b)
        comp = r.integers(0, components, size=_BLOCK)[lo:lo + take]
        z = r.standard_normal(size=(_BLOCK, rank), dtype=np.float32)[lo:lo + take]
        eps = r.standard_normal(size=(_BLOCK, D), dtype=np.float32)[lo:lo + take]
        lat = A[comp].astype(np.float32) + np.float32(0.5) * z
        blk = np.float32(0.03) + np.float32(0.03) * (lat @ B32) + np.float32(0.02) * eps
        np.clip(blk, 0.0, 1.0, out=blk)
        X[out:out + take] = blk
    return X


def init_indices(N, M, K, seed=SEED_INIT):
    """int64 [M][K]: for each stage, K distinct row indices used to seed an all-zero dictionary."""
    out = np.empty((M, K), np.int64)
    for m in range(M):
        out[m] = _rng(seed, 31, m).choice(N, size=K, replace=False)
    return out


def planted_lattice(K, M, D, seed=SEED_DATA, ratio=8.0):
    """All K**M sums of M hierarchical codebooks whose scales shrink by `ratio` per stage,
    with codewords of one stage separated by more than twice the reach of all later stages.
    Returns (X fp32 [K**M][D], C float64 [M][K][D], codes uint8 [K**M][M])."""
    g = _rng(seed, 41)
    C = np.zeros((M, K, D), np.float64)
    scale = 1.0
    for m in range(M):
        # integer lattice points on a coarse grid keep every sum exactly representable
        pts = set()
        while len(pts) < K:
            pts.add(tuple(g.integers(-3, 4, size=D).tolist()))
        C[m] = np.array(sorted(pts), np.float64) * scale
        scale /= ratio
    grids = np.meshgrid(*[np.arange(K)] * M, indexing="ij")
    codes = np.stack([gr.reshape(-1) for gr in grids], axis=1).astype(np.uint8)
    X = np.zeros((codes.shape[0], D), np.float64)
    for m in range(M):
        X += C[m][codes[:, m]]
    return X.astype(np.float32), C, codes
