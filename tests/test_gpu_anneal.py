"""hclae_anneal: several sweeps in one call (Sec. 3.1, the method iterated).  The call must leave the very bits that
the same number of hclae_sweep calls leaves -- dictionaries, codes, residues and the error after every stage --
while its stages start from the distance bounds their last visit kept instead of an assignment over all vectors,
and pass into one another through the fused row pass, across sweeps too."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _fresh(ctx, X, M, K, T):
    N, D = X.shape
    C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    r = X.clone()
    ctx.sweep(C, codes, r, T, init_idx=synth.init_indices(N, M, K), want_err=False)
    return C, codes, r


def _both_ways(X, M, K, T, sweeps, contraction=0, pruning=True, n_max=None, want_err=True):
    """(state after `sweeps` hclae_sweep calls, state after one hclae_anneal call, the two work-counter triples)"""
    from paper_1509_05194_amd import hclae
    N, D = X.shape
    out = []
    for one_call in (False, True):
        ctx = hclae.Context(n_max or N, D, M, K)
        ctx.set_contraction(contraction)
        ctx.set_pruning(pruning)
        C, codes, r = _fresh(ctx, X, M, K, T)
        ctx.work_counters(reset=True)
        if one_call:
            E = ctx.anneal(C, codes, r, T, sweeps, want_err=want_err)
        else:
            E = np.stack([ctx.sweep(C, codes, r, T, want_err=True) for _ in range(sweeps)])
        torch.cuda.synchronize()
        out.append((C.clone(), codes.clone(), r.clone(), E, ctx.work_counters()))
        ctx.close()
    return out


def _assert_same(a, b, with_err=True):
    assert torch.equal(a[0], b[0]), "dictionaries differ"
    assert torch.equal(a[1], b[1]), "codes differ"
    assert torch.equal(a[2], b[2]), "residues differ"
    if with_err:
        np.testing.assert_array_equal(a[3], b[3])


SHAPES = {
    # name: (generator, N, D, M, K, T, sweeps)
    "sift_resident": ("sift", 40000 + 17, 128, 4, 256, 5, 8),
    "small_k": ("sift", 9000 + 5, 32, 3, 64, 4, 8),
    "padded_d": ("gmm", 12000 + 3, 20, 3, 50, 3, 7),
    "gist_chunked": ("gist", 6000 + 9, 960, 2, 256, 3, 6),
    "one_dictionary": ("sift", 15000 + 1, 128, 1, 256, 4, 6),
    "codes_128bit": ("sift", 30000 + 3, 128, 16, 256, 2, 5),
    "one_codeword": ("gmm", 5000 + 1, 16, 2, 1, 2, 4),
    "few_vectors": ("sift", 100, 128, 2, 64, 3, 6),
}


def _data(kind, N, D):
    if kind == "sift":
        return synth.sift_like(N, D=D)
    if kind == "gist":
        return synth.gist_like(N, D=D)
    return synth.tiny_gmm(N, D=D, components=40, sigma=0.2)


@pytest.mark.parametrize("name", list(SHAPES))
def test_anneal_equals_repeated_sweeps(name):
    kind, N, D, M, K, T, sweeps = SHAPES[name]
    X = torch.from_numpy(_data(kind, N, D)).cuda()
    a, b = _both_ways(X, M, K, T, sweeps)
    _assert_same(a, b)
    # the same number of assignments, fewer vectors recomputed: the first assignment of a stage was pruned too
    assert a[4][0] == b[4][0] == sweeps * M * (T + 1)
    print("%s: vectors recomputed %d in %d sweep calls, %d in one call" % (name, a[4][1], sweeps, b[4][1]))
    assert b[4][1] <= a[4][1] if name in ("one_codeword", "few_vectors") else b[4][1] < a[4][1]
    assert np.all(np.diff(b[3].reshape(-1)) <= 1e-7 * b[3].reshape(-1)[:-1])


def test_anneal_split_contraction_and_no_pruning():
    kind, N, D, M, K, T, sweeps = SHAPES["sift_resident"]
    X = torch.from_numpy(_data(kind, N, D)).cuda()
    ref = _both_ways(X, M, K, T, sweeps)[0]
    a, b = _both_ways(X, M, K, T, sweeps, contraction=1)
    _assert_same(a, b)
    _assert_same(ref, b)
    assert b[4][1] < a[4][1]
    a, b = _both_ways(X, M, K, T, sweeps, pruning=False)            # nothing carried: only the fused passes differ
    _assert_same(a, b)
    _assert_same(ref, b)
    assert a[4][1] == b[4][1] == sweeps * M * (T + 1) * N


def test_anneal_twice_and_with_a_larger_context():
    """A second call starts its own bookkeeping (bounds of the first call are not used), a ctx created for more
    vectors than the call brings keeps its per-stage arrays apart, and without the errors the call does not
    synchronise (the state is read after an explicit synchronisation)."""
    from paper_1509_05194_amd import hclae
    N, D, M, K, T = 20000 + 7, 128, 3, 256, 4
    X = torch.from_numpy(synth.sift_like(N, D=D)).cuda()
    ref = _both_ways(X, M, K, T, 8)[0]
    ctx = hclae.Context(3 * N, D, M, K)
    C, codes, r = _fresh(ctx, X, M, K, T)
    assert ctx.anneal(C, codes, r, T, 5, want_err=False) is None
    # something else in between on the same ctx: an encode of other data
    other = torch.from_numpy(synth.sift_like(5000, D=D, start=10 ** 6)).cuda()
    oc = torch.zeros((5000, M), dtype=torch.uint8, device="cuda:0")
    orr = torch.empty_like(other)
    ctx.encode(other, C, oc, orr)
    E = ctx.anneal(C, codes, r, T, 3)
    torch.cuda.synchronize()
    assert torch.equal(C, ref[0]) and torch.equal(codes, ref[1]) and torch.equal(r, ref[2])
    np.testing.assert_array_equal(E, ref[3][5:])
    # degenerate calls
    assert ctx.anneal(C, codes, r, T, 0).shape == (0, M)
    E1 = ctx.anneal(C, codes, r, T, 1)
    E2 = ctx.sweep(C, codes, r, T)
    assert E1.shape == (1, M) and np.all(E2 <= E1[0, -1] * (1 + 1e-7))
    ctx.close()


def test_anneal_fullsize_ten_sweeps():
    """N = 1,000,000, D = 128, M = 8, K = 256, T = 10: ten annealing sweeps in one call against ten calls."""
    N, D, M, K, T, sweeps = 1_000_000, 128, 8, 256, 10, 10
    X = torch.from_numpy(synth.sift_like(N, D=D)).cuda()
    a, b = _both_ways(X, M, K, T, sweeps)
    _assert_same(a, b)
    print("N = 1M: vectors recomputed %d in ten sweep calls, %d in one call (%.1f %%)"
          % (a[4][1], b[4][1], 100.0 * b[4][1] / a[4][1]))
    assert b[4][1] < a[4][1]


@pytest.mark.parametrize("name", ["sift_resident", "gist_chunked"])
def test_anneal_from_zero_dictionaries_in_one_call(name):
    """init_idx: the call's first sweep seeds the all-zero dictionaries (as hclae_sweep does), the others anneal and
    carry their bounds; the whole training in one call equals the sweep calls bit for bit."""
    from paper_1509_05194_amd import hclae
    kind, N, D, M, K, T, sweeps = SHAPES[name]
    X = torch.from_numpy(_data(kind, N, D)).cuda()
    idx = synth.init_indices(N, M, K)
    out = []
    for one_call in (False, True):
        ctx = hclae.Context(N, D, M, K)
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        r = X.clone()
        if one_call:
            E = ctx.anneal(C, codes, r, T, sweeps + 1, init_idx=idx)
        else:
            E = np.stack([ctx.sweep(C, codes, r, T, init_idx=idx if s == 0 else None) for s in range(sweeps + 1)])
        torch.cuda.synchronize()
        out.append((C.clone(), codes.clone(), r.clone(), E, ctx.work_counters()))
        ctx.close()
    _assert_same(out[0], out[1])
    assert out[1][4][1] < out[0][4][1]
    # without the errors the call synchronises once at the end (the seed indices are read asynchronously)
    ctx = hclae.Context(N, D, M, K)
    C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    r = X.clone()
    assert ctx.anneal(C, codes, r, T, 2, init_idx=idx, want_err=False) is None
    ctx.sweep(C, codes, r, T, want_err=False)
    ctx.close()


def test_anneal_with_the_improved_kmeans_cooldown():
    """With the cool-down of Sec. 3.2 chosen (hclae_set_cooldown) nothing is carried and no pass is fused: the call is
    the loop over the sweeps, equal to the separate calls bit for bit."""
    from paper_1509_05194_amd import hclae
    N, D, M, K, T, sweeps = 8000 + 3, 32, 3, 64, 10, 3
    X = torch.from_numpy(synth.sift_like(N, D=D)).cuda()
    idx = synth.init_indices(N, M, K)
    out = []
    for one_call in (False, True):
        ctx = hclae.Context(N, D, M, K)
        ctx.set_cooldown(True, 10)
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        r = X.clone()
        if one_call:
            E = ctx.anneal(C, codes, r, T, sweeps, init_idx=idx)
        else:
            E = np.stack([ctx.sweep(C, codes, r, T, init_idx=idx if s == 0 else None) for s in range(sweeps)])
        torch.cuda.synchronize()
        out.append((C.clone(), codes.clone(), r.clone(), E))
        ctx.close()
    _assert_same(out[0], out[1])
