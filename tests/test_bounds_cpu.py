"""The rounding allowances of the exact pruning (distance bounds of a stage, Sec. 3.1 cool-down) as arithmetic facts,
checked on the CPU in the kernel's own precision: the relative slack (D/2 + 16) 2^-23 given to the fp32 value of
||x'||^2 -- per lane a chain of D/2 fused multiply-adds, then one addition of the two half sums -- must cover its worst
rounding error at every D the library accepts, with room for the handful of fp32 operations that follow."""
import numpy as np
import pytest


def _chain_sum_sq_f32(x):
    """Sum of squares of x in fp32 the way a lane accumulates it: acc = fma(x_i, x_i, acc), one rounding per term.
    The product of two floats is exact in double; product plus accumulator is rounded to double and then to fp32,
    which can differ from the single rounding of a true fma only in rare halfway cases and then by one fp32 ulp of
    one partial sum -- nothing against a bound that is asked to hold with a factor of two to spare."""
    acc = np.float32(0.0)
    for v in x:
        acc = np.float32(np.float64(v) * np.float64(v) + np.float64(acc))
    return acc


@pytest.mark.parametrize("D", [128, 960, 4096])
def test_slack_covers_the_rounding_of_the_squared_norm(D):
    slack_rel = (((D + 63) // 64 * 64) / 2 + 16) * 2.0 ** -23
    g = np.random.default_rng(D)
    worst = 0.0
    cases = [g.uniform(0, 255, D), np.rint(g.uniform(0, 255, D)), g.standard_normal(D) * 1e-3,
             np.full(D, 1.0 + 2.0 ** -12), np.full(D, 255.0 * (1 - 2.0 ** -13)), g.uniform(0.99, 1.0, D),
             np.concatenate([[1e4], g.uniform(0, 1, D - 1)]), g.lognormal(0, 3, D)]
    for x in cases:
        x = x.astype(np.float32)
        # the two lane halves of a row take alternate groups of four coordinates
        grp = (np.arange(D) // 4) % 2
        x2 = np.float32(_chain_sum_sq_f32(x[grp == 0]) + _chain_sum_sq_f32(x[grp == 1]))
        exact = float((x.astype(np.float64) ** 2).sum())
        rel = abs(float(x2) - exact) / exact
        worst = max(worst, rel)
        assert rel <= 0.5 * slack_rel, "D=%d: error %.3g of the squared norm exceeds half the slack %.3g" % (D, rel, slack_rel)
    # the a-priori bound itself: (D/2 + 1) roundings of relative size 2^-24 on a sum of positive terms
    assert (D / 2 + 1) * 2.0 ** -24 <= 0.5 * slack_rel
    print("D=%d: worst relative error of ||x||^2 %.2e, slack %.2e" % (D, worst, slack_rel))


@pytest.mark.parametrize("D,M,K", [(128, 8, 16), (960, 4, 8), (16, 16, 4)])
def test_carried_bound_allowance_covers_the_fp32_row_passes(D, M, K):
    """Bounds carried from one sweep to the next: between two visits of stage m the fp32 x' moves by
    - sum_j d_j (d_j = c_j,new(i_new) - c_j,old(i_old) over the other stages) plus the roundings of the 2M row passes.
    The library widens the bounds by sum_j ||d_j|| (rounded up) + (8M + 16) 2^-24 sqrt(D) A, A = the largest |x'| or
    codeword coordinate seen.  Emulated here in the kernels' own precision (one fp32 rounding per heat and per new
    residue), with dictionaries and codes that change arbitrarily between the visits."""
    g = np.random.default_rng(D * 131 + M)
    N = 400
    for scale, shake in ((255.0, 0.0), (255.0, 1e-3), (1.0, 0.0), (1e-3, 5.0)):
        C = (g.standard_normal((M, K, D)) * scale * 0.3).astype(np.float32)
        codes = g.integers(0, K, size=(N, M))
        X = (g.uniform(0, scale, (N, D))).astype(np.float32)
        # a consistent fp32 state: residue = X - sum of codewords, subtracted stage by stage in fp32
        r = X.copy()
        for j in range(M):
            r = (r - C[j][codes[:, j]]).astype(np.float32)
        amax = float(np.abs(C).max())
        m = 2 % M
        # last visit of stage m: heat, (its dictionary and code stay), new residue
        xp_old = (r + C[m][codes[:, m]]).astype(np.float32)
        amax = max(amax, float(np.abs(xp_old).max()))
        r = (xp_old - C[m][codes[:, m]]).astype(np.float32)
        path = np.zeros(N)
        for step in range(1, M):
            j = (m + step) % M
            xp = (r + C[j][codes[:, j]]).astype(np.float32)
            amax = max(amax, float(np.abs(xp).max()))
            c_old, i_old = C[j].copy(), codes[:, j].copy()
            # the stage moves its dictionary a little (or not at all) and re-assigns some vectors
            C[j] = (C[j] + g.standard_normal((K, D)).astype(np.float32) * np.float32(scale * shake)).astype(np.float32)
            flip = g.random(N) < 0.1
            codes[flip, j] = g.integers(0, K, size=int(flip.sum()))
            d = C[j][codes[:, j]].astype(np.float64) - c_old[i_old].astype(np.float64)
            path += np.float32(np.sqrt((d * d).sum(1)) * 1.000001).astype(np.float64)
            r = (xp - C[j][codes[:, j]]).astype(np.float32)
        xp_new = (r + C[m][codes[:, m]]).astype(np.float32)
        amax = max(amax, float(np.abs(xp_new).max()))
        moved = np.sqrt(((xp_new.astype(np.float64) - xp_old.astype(np.float64)) ** 2).sum(1))
        allowance = (8 * M + 16) * 2.0 ** -24 * np.sqrt(D) * amax
        delta = path * (1 + 1e-9) + allowance
        assert np.all(moved <= delta), "scale %g: shift %.6g beyond the carried bound %.6g" % (
            scale, float((moved - delta).max()), float(delta.min()))
        # and the allowance is not idle: with unchanged dictionaries and codes the shift is pure rounding, within it
        if shake == 0.0:
            still = moved[path == 0.0]
            if len(still):
                assert still.max() <= allowance
                print("D=%d M=%d scale %g: rounding shift up to %.3g, allowance %.3g" % (D, M, scale, still.max(), allowance))
