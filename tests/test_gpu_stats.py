"""Dictionary re-ordering by variance (Sec. 3.3) and code statistics (Sec. 2.2) against the oracle's
plain NumPy definitions; integer results must be bit-exact."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth
from parity_util import fresh_state, to_dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_reorder_by_variance_and_stats(oracle):
    from paper_1509_05194_amd import hclae
    N, D, M, K = 30000 + 11, 32, 5, 64
    X = synth.sift_like(N, D=D)
    C, codes, r = fresh_state(X, M, K)
    oracle.sweep(C, codes, r, 2, synth.init_indices(N, M, K))
    shuffle = np.array([3, 0, 4, 2, 1])
    C32 = np.ascontiguousarray(C[shuffle].astype(np.float32))
    codes_s = np.ascontiguousarray(codes[:, shuffle])
    ctx = hclae.Context(N, D, M, K)
    Cg, codes_g = to_dev(C32), to_dev(codes_s)
    # statistics first (on the shuffled codes)
    hist, joint = ctx.code_stats(codes_g, pair=(1, 3))
    np.testing.assert_array_equal(hist, oracle.code_histogram(codes_s, K))
    np.testing.assert_array_equal(joint, oracle.joint_histogram(codes_s, 1, 3, K))
    H = [oracle.entropy_bits(h) for h in hist]
    print("H(I_m) bits:", np.round(H, 3), " I(I_1;I_3) bits: %.4f" % oracle.mutual_information_bits(joint))
    assert all(0 < h <= np.log2(K) + 1e-12 for h in H)
    # re-ordering
    var, order = ctx.reorder_by_variance(Cg, codes_g)
    v_o = oracle.dictionary_variances(C32.astype(np.float64))
    np.testing.assert_allclose(var, v_o, rtol=1e-12)
    o_o = oracle.variance_order(C32.astype(np.float64))
    np.testing.assert_array_equal(order, o_o)
    np.testing.assert_array_equal(Cg.cpu().numpy(), C32[o_o])
    np.testing.assert_array_equal(codes_g.cpu().numpy(), codes_s[:, o_o])
    # the reconstruction does not depend on the order of the dictionaries
    rec_before = oracle.reconstruct(C32.astype(np.float64), codes_s)
    rec_after = oracle.reconstruct(Cg.cpu().numpy().astype(np.float64), codes_g.cpu().numpy())
    assert np.abs(rec_before - rec_after).max() <= 1e-9 * np.abs(rec_before).max()
    hist2, none = ctx.code_stats(codes_g)
    assert none is None
    np.testing.assert_array_equal(hist2, hist[o_o])
    ctx.close()
