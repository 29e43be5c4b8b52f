"""Helpers of the GPU-vs-oracle parity tests (test infrastructure; uses the oracle)."""
import numpy as np

REL_GAP = 1e-5          # near-tie exemption: oracle top-2 gap, relative to the larger distance
TINY = 1e-300


def fresh_state(X, M, K):
    N, D = X.shape
    return (np.zeros((M, K, D), np.float64), np.zeros((N, M), np.uint8), X.astype(np.float64))


def to_dev(a, dev="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def narrow_state(C64, codes, r64, dev="cuda:0"):
    """fp32 device copies of an oracle state, and the exact widening of those copies
    (what both sides then start from)."""
    C32 = C64.astype(np.float32)
    r32 = r64.astype(np.float32)
    return (to_dev(C32, dev), to_dev(codes.copy(), dev), to_dev(r32, dev),
            C32.astype(np.float64), codes.copy(), r32.astype(np.float64))


def judge_codes(oracle, xp64, C64, m, codes_gpu_col, codes_or_col, d1, d2):
    """Compare one code column.  Returns (n_differ, n_exempt, bad_indices).
    A differing GPU code is exempt iff the oracle's own top-2 gap is below REL_GAP relative
    AND the oracle distance of the GPU's choice is itself within REL_GAP relative of the best."""
    diff = np.nonzero(codes_gpu_col != codes_or_col)[0]
    bad = []
    for n in diff:
        relgap = (d2[n] - d1[n]) / max(d2[n], TINY)
        dg = oracle.dist_to(xp64, C64, n, m, int(codes_gpu_col[n]))
        excess = (dg - d1[n]) / max(dg, TINY)
        if not (relgap < REL_GAP and excess < REL_GAP):
            bad.append(int(n))
    return len(diff), len(diff) - len(bad), bad


def rel_fro(a, b):
    return float(np.linalg.norm(np.asarray(a, np.float64) - b) / max(np.linalg.norm(b), TINY))
