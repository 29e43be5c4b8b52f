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
