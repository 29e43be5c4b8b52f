"""Pins of the CPU oracle against what the paper (arXiv 1509.05194) and the mathematics fix.
No GPU, no HIP library.  Each test states which mistake in the oracle it is there to catch."""
import os

import numpy as np
import pytest

from paper_1509_05194_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _fresh_state(X, M, K):
    """All-zero dictionaries, zero codes, residue = x (Sec. 3.1: learning from scratch)."""
    N, D = X.shape
    return (np.zeros((M, K, D), np.float64), np.zeros((N, M), np.uint8), X.astype(np.float64))


def _brute_argmin(x, c):
    d = ((x[:, None, :] - c[None, :, :]) ** 2).sum(-1)
    return d.argmin(1), d


# ---------------------------------------------------------------- golden: hand-worked example
def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = np.array([float(v) for v in vals])
    return out


def test_hand_worked_1d_stage(oracle):
    g = _read_golden("hand_1d_lloyd.txt")
    X = g["x"].astype(np.float32).reshape(-1, 1)
    C = g["c_start"].reshape(1, 2, 1).copy()
    codes = np.zeros((4, 1), np.uint8)
    r = X.astype(np.float64) - C[0][codes[:, 0]]
    E, J = oracle.anneal_stage(0, C, codes, r, int(g["T"][0]), trace=True)
    np.testing.assert_allclose(C.reshape(-1), g["c_final"], rtol=0, atol=1e-15)
    np.testing.assert_array_equal(codes[:, 0], g["codes_final"].astype(np.uint8))
    np.testing.assert_allclose(r.reshape(-1), g["residue_final"], rtol=0, atol=1e-15)
    assert E == g["E_final"][0]
    assert J[0] == g["J_entry"][0]
    assert J[1] == g["J_after_assign1"][0]
    np.testing.assert_allclose(J[2], g["J_after_update1"][0], rtol=1e-15)


# ---------------------------------------------------------------- P1 reconstruction
def test_reconstruction_after_every_step(oracle):
    """x = sum_m C_m[i_m] + r after heat/assign/update/cool (Sec. 3.1: x' is the residue with
    dictionary m dropped).  Catches a wrong sign in heat or cool, or a wrong code column."""
    X = synth.tiny_gmm(N=2000)
    M, K, T = 4, 16, 2
    C, codes, r = _fresh_state(X, M, K)
    idx = synth.init_indices(X.shape[0], M, K)
    oracle.sweep(C, codes, r, T, idx)
    X64 = X.astype(np.float64)
    tol = 1e-9 * np.abs(X64).max()
    assert np.abs(oracle.reconstruct(C, codes) + r - X64).max() <= tol
    for m in range(M):
        oracle.heat(r, codes, C, m)
        # during the stage: x = sum_{j != m} C_j[i_j] + x'
        others = oracle.reconstruct(C, codes) - C[m][codes[:, m]]
        assert np.abs(others + r - X64).max() <= tol
        oracle.assign(r, C, codes, m)
        oracle.update(r, codes, C, m)
        oracle.assign(r, C, codes, m)
        oracle.cool(r, codes, C, m)
        assert np.abs(oracle.reconstruct(C, codes) + r - X64).max() <= tol


def test_heat_then_cool_is_identity_and_uses_column_m(oracle):
    g = np.random.default_rng(7)
    N, D, M, K = 50, 3, 3, 4
    C = g.standard_normal((M, K, D))
    codes = g.integers(0, K, size=(N, M)).astype(np.uint8)
    r0 = g.standard_normal((N, D))
    for m in range(M):
        r = r0.copy()
        oracle.heat(r, codes, C, m)
        np.testing.assert_allclose(r, r0 + C[m][codes[:, m]], rtol=0, atol=0)
        oracle.cool(r, codes, C, m)
        np.testing.assert_allclose(r, r0, rtol=0, atol=1e-15)


# ---------------------------------------------------------------- P2 monotone objective
@pytest.mark.parametrize("gen", ["tiny", "sift"])
def test_objective_non_increasing(oracle, gen):
    """Sec. 3.1: a better fit of the intermediate dataset lowers the quantization error.
    Both Lloyd half-steps and the whole stage may never raise it.  Catches an update that
    is not the mean, an assign that is not the minimum, a lost empty-cluster rule."""
    if gen == "tiny":
        X, M, K, T = synth.tiny_gmm(N=3000), 4, 16, 4
    else:
        X, M, K, T = synth.sift_like(3000, D=32), 3, 64, 3   # K large vs N: empty clusters occur
    C, codes, r = _fresh_state(X, M, K)
    idx = synth.init_indices(X.shape[0], M, K)
    prev = oracle.quant_error(r)
    for s in range(3):
        for m in range(M):
            E, J = oracle.anneal_stage(m, C, codes, r, T, idx[m] if s == 0 else None, trace=True)
            if s == 0:
                # seeding replaces the zero dictionary: the entry value belongs to the old C_m
                J = J[1:]
            else:
                assert abs(J[0] - prev) <= 1e-12 * prev
            assert np.all(np.diff(J) <= 1e-12 * J[:-1]), J
            assert E <= prev * (1 + 1e-12)
            assert E == J[-1]
            prev = E


# ---------------------------------------------------------------- P3 brute force, ties
def test_assign_matches_bruteforce_and_lowest_index_ties(oracle):
    g = np.random.default_rng(3)
    for trial in range(20):
        N, D, K = 64, int(g.integers(1, 5)), int(g.integers(1, 9))
        x = g.integers(-3, 4, size=(N, D)).astype(np.float64)       # small integers: exact ties
        c = g.integers(-3, 4, size=(K, D)).astype(np.float64)
        if K > 2:
            c[K - 1] = c[0]                                          # duplicate codeword
        C = c[None].copy()
        codes = np.full((N, 1), 255, np.uint8)
        d1, d2, i2 = oracle.assign(x, C, codes, 0, top2=True)
        ref, dist = _brute_argmin(x, c)                              # numpy argmin = first minimum
        np.testing.assert_array_equal(codes[:, 0], ref)
        np.testing.assert_array_equal(d1, dist.min(1))
        if K > 1:
            srt = np.sort(dist, axis=1)
            np.testing.assert_array_equal(d2, srt[:, 1])
            assert np.all(dist[np.arange(N), i2] == d2) and np.all(i2 != codes[:, 0])
        for n in (0, N - 1):
            assert oracle.dist_to(x, C, n, 0, K - 1) == dist[n, K - 1]


def test_assign_only_touches_column_m(oracle):
    g = np.random.default_rng(4)
    N, D, M, K = 40, 3, 3, 5
    C = g.standard_normal((M, K, D))
    x = g.standard_normal((N, D))
    codes = np.full((N, M), 77, np.uint8)
    oracle.assign(x, C, codes, 1)
    assert np.all(codes[:, 0] == 77) and np.all(codes[:, 2] == 77)
    np.testing.assert_array_equal(codes[:, 1], _brute_argmin(x, C[1])[0])


# ---------------------------------------------------------------- P4 K = 1 closed form
def test_k1_closed_form(oracle):
    """K=1: the first dictionary becomes the data mean, the later ones the (zero) mean of a
    centred residue, and E is the trace of the sample covariance."""
    X = synth.tiny_gmm(N=1500)
    M = 3
    C, codes, r = _fresh_state(X, M, 1)
    idx = np.array([[5], [9], [11]], np.int64)
    err = oracle.sweep(C, codes, r, 1, idx)
    X64 = X.astype(np.float64)
    mean = X64.mean(0)
    np.testing.assert_allclose(C[0, 0], mean, rtol=0, atol=1e-14)
    np.testing.assert_allclose(C[1:], 0.0, rtol=0, atol=1e-14)
    tr = ((X64 - mean) ** 2).sum(1).mean()
    np.testing.assert_allclose(err, tr, rtol=1e-12)
    assert np.all(codes == 0)


# ---------------------------------------------------------------- P5 M = 1 is plain Lloyd
def test_m1_equals_library_lloyd(oracle):
    """M=1: x' = x exactly, so a stage with T iterations is T Lloyd iterations from the same
    start followed by a consistent labelling; checked against scikit-learn's Lloyd."""
    from sklearn.cluster import KMeans
    X = synth.tiny_gmm(N=4000)
    K, T = 16, 7
    idx = synth.init_indices(X.shape[0], 1, K)
    C, codes, r = _fresh_state(X, 1, K)
    E = oracle.anneal_stage(0, C, codes, r, T, idx[0])
    X64 = X.astype(np.float64)
    km = KMeans(n_clusters=K, init=X64[idx[0]], n_init=1, algorithm="lloyd", max_iter=T, tol=0.0).fit(X64)
    assert len(np.unique(km.labels_)) == K            # sklearn's empty-cluster rule differs; not hit here
    np.testing.assert_allclose(C[0], km.cluster_centers_, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(codes[:, 0], km.labels_)
    np.testing.assert_allclose(E * X.shape[0], km.inertia_, rtol=1e-12)
    # two sweeps of T = one run of 2T (the extra re-assign in between is idempotent)
    oracle.anneal_stage(0, C, codes, r, T, None)
    km2 = KMeans(n_clusters=K, init=X64[idx[0]], n_init=1, algorithm="lloyd", max_iter=2 * T, tol=0.0).fit(X64)
    np.testing.assert_allclose(C[0], km2.cluster_centers_, rtol=0, atol=1e-12)


def test_empty_cluster_keeps_previous_codeword(oracle):
    x = np.array([[0.0], [1.0], [2.0]])
    C = np.array([[[1.0], [100.0], [-50.0]]])
    codes = np.zeros((3, 1), np.uint8)
    oracle.assign(x, C, codes, 0)
    counts, empty = oracle.update(x, codes, C, 0)
    assert empty == 2 and counts.tolist() == [3, 0, 0]
    np.testing.assert_array_equal(C.reshape(-1), [1.0, 100.0, -50.0])


# ---------------------------------------------------------------- P6 fresh start = RVQ; Eq.3 L=1
def test_fresh_sweep_equals_stagewise_rvq(oracle):
    """Footnote of Sec. 3.1: DA on all-zero dictionaries sees the residues as its intermediate
    dataset, i.e. it is residual vector quantization: k-means on the residue, subtract, repeat."""
    from sklearn.cluster import KMeans
    X = synth.tiny_gmm(N=3000)
    M, K, T = 3, 8, 5
    idx = synth.init_indices(X.shape[0], M, K)
    C, codes, r = _fresh_state(X, M, K)
    oracle.sweep(C, codes, r, T, idx)
    res = X.astype(np.float64)
    for m in range(M):
        km = KMeans(n_clusters=K, init=res[idx[m]], n_init=1, algorithm="lloyd", max_iter=T, tol=0.0).fit(res)
        assert len(np.unique(km.labels_)) == K
        np.testing.assert_allclose(C[m], km.cluster_centers_, rtol=0, atol=1e-11)
        np.testing.assert_array_equal(codes[:, m], km.labels_)
        res = res - km.cluster_centers_[km.labels_]
    np.testing.assert_allclose(r, res, rtol=0, atol=1e-11)


def test_encode_is_eq3_with_one_path(oracle):
    """Eq. 3 with L=1: picking k by ||x-a||^2 + ||x-c_k||^2 - ||x||^2 + 2 c_k.a (a = partial
    sum so far) is the greedy residual encoder.  The objective is evaluated here in the
    paper's expanded form, not the oracle's direct form."""
    g = np.random.default_rng(11)
    N, D, M, K = 200, 6, 4, 7
    X = g.standard_normal((N, D)).astype(np.float32)
    C = g.standard_normal((M, K, D)) * (0.5 ** np.arange(M))[:, None, None]
    codes, r = oracle.encode(X, C)
    x = X.astype(np.float64)
    a = np.zeros_like(x)
    for m in range(M):
        obj = (((x - a) ** 2).sum(1)[:, None] + ((x[:, None, :] - C[m][None]) ** 2).sum(-1)
               - (x ** 2).sum(1)[:, None] + 2.0 * a @ C[m].T)
        direct = ((x - a)[:, None, :] - C[m][None]) ** 2
        np.testing.assert_allclose(obj, direct.sum(-1), rtol=1e-10, atol=1e-10)
        pick = obj.argmin(1)
        # skip rows where the expanded form's rounding could flip a near-tie
        srt = np.sort(obj, axis=1)
        safe = (srt[:, 1] - srt[:, 0]) > 1e-9
        np.testing.assert_array_equal(codes[safe, m], pick[safe])
        a = a + C[m][codes[:, m]]
    np.testing.assert_allclose(r, x - a, rtol=0, atol=1e-13)


# ---------------------------------------------------------------- P7 Eq. 1 identity
def test_eq1_expansion(oracle):
    """Eq. 1: ||x - sum c_m||^2 = sum_m ||x - c_m||^2 - (M-1)||x||^2 + sum_{a != b} c_a.c_b
    (the printed factor m-1 is read as M-1)."""
    X = synth.tiny_gmm(N=1000)
    M, K = 4, 16
    C, codes, r = _fresh_state(X, M, K)
    oracle.sweep(C, codes, r, 2, synth.init_indices(X.shape[0], M, K))
    x = X.astype(np.float64)
    sel = np.stack([C[m][codes[:, m]] for m in range(M)], 0)            # [M][N][D]
    t1 = ((x[None] - sel) ** 2).sum(-1).sum(0)
    t2 = (M - 1) * (x ** 2).sum(1)
    G = np.einsum("and,bnd->nab", sel, sel)
    t3 = G.sum((1, 2)) - np.einsum("naa->n", G)
    lhs = (r ** 2).sum(1)
    np.testing.assert_allclose(lhs, ((x - sel.sum(0)) ** 2).sum(1), rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(lhs.mean(), (t1 - t2 + t3).mean(), rtol=1e-10)
    np.testing.assert_allclose(oracle.quant_error(r), lhs.mean(), rtol=1e-13)


def test_quant_error_is_mean_not_sum(oracle):
    r = np.array([[3.0, 4.0], [0.0, 0.0], [1.0, 0.0], [0.0, 2.0]])
    assert oracle.quant_error(r) == (25.0 + 0.0 + 1.0 + 4.0) / 4.0


# ---------------------------------------------------------------- P8 planted lattice
def test_planted_lattice(oracle):
    X, C, planted = synth.planted_lattice(K=4, M=3, D=3, ratio=16.0)
    codes, r = oracle.encode(X, C)
    np.testing.assert_array_equal(codes, planted)
    assert np.abs(r).max() == 0.0
    C2 = C.copy()
    err = oracle.sweep(C2, codes, r, 2, None)
    np.testing.assert_allclose(C2, C, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(codes, planted)
    assert np.all(err <= 1e-28)


# ---------------------------------------------------------------- P10 permutation / duplication
def test_permutation_and_duplication(oracle):
    X = synth.tiny_gmm(N=1200)
    N = X.shape[0]
    M, K, T = 2, 8, 3
    idx = synth.init_indices(N, M, K)
    C, codes, r = _fresh_state(X, M, K)
    oracle.sweep(C, codes, r, T, idx)

    perm = np.random.default_rng(5).permutation(N)
    inv = np.empty(N, np.int64)
    inv[perm] = np.arange(N)
    Cp, codesp, rp = _fresh_state(X[perm], M, K)
    oracle.sweep(Cp, codesp, rp, T, inv[idx])
    np.testing.assert_allclose(Cp, C, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(codesp, codes[perm])
    np.testing.assert_allclose(rp, r[perm], rtol=0, atol=1e-12)

    Xd = np.repeat(X, 2, axis=0)
    Cd, codesd, rd = _fresh_state(Xd, M, K)
    oracle.sweep(Cd, codesd, rd, T, 2 * idx)
    np.testing.assert_allclose(Cd, C, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(codesd[::2], codes)


# ---------------------------------------------------------------- P11 idempotence
def test_t0_stage_is_idempotent(oracle):
    X = synth.tiny_gmm(N=1500)
    M, K = 3, 8
    C, codes, r = _fresh_state(X, M, K)
    oracle.sweep(C, codes, r, 2, synth.init_indices(X.shape[0], M, K))
    # perturb dictionary 1 so that some codes are stale, keeping the reconstruction invariant
    oracle.heat(r, codes, C, 1)
    C[1] += 0.05 * np.random.default_rng(2).standard_normal(C[1].shape)
    oracle.cool(r, codes, C, 1)
    C0, codes0 = C.copy(), codes.copy()
    E0 = oracle.quant_error(r)
    E1 = oracle.anneal_stage(1, C, codes, r, 0)
    np.testing.assert_array_equal(C, C0)
    assert E1 <= E0
    changed = codes[:, 1] != codes0[:, 1]
    assert changed.any() and np.all(codes[:, [0, 2]] == codes0[:, [0, 2]])
    codes1, r1 = codes.copy(), r.copy()
    E2 = oracle.anneal_stage(1, C, codes, r, 0)
    np.testing.assert_array_equal(codes, codes1)
    np.testing.assert_allclose(r, r1, rtol=0, atol=1e-15)
    np.testing.assert_allclose(E2, E1, rtol=1e-14)


def test_thread_count_does_not_change_results(oracle):
    X = synth.sift_like(2000, D=32)
    M, K, T = 2, 16, 2
    idx = synth.init_indices(X.shape[0], M, K)
    outs = []
    t0 = oracle.threads()
    for t in (1, 4):
        oracle.set_threads(t)
        C, codes, r = _fresh_state(X, M, K)
        err = oracle.sweep(C, codes, r, T, idx)
        outs.append((C, codes, r, err))
    oracle.set_threads(t0)
    for a, b in zip(outs[0], outs[1]):
        np.testing.assert_array_equal(a, b)


# ---------------------------------------------------------------- online chunks (Sec. 3.4)
def test_online_chunk_is_composition_of_pinned_steps(oracle):
    """With empty running sums an online chunk is, per dictionary, exactly the pinned steps
    assign -> update -> assign -> cool (one Lloyd iteration on the chunk's residue)."""
    X8 = synth.sift_like(1500, D=16, dtype=np.uint8)
    M, K, D = 3, 8, 16
    Cs, codes_s, r_s = _fresh_state(X8.astype(np.float32), M, K)
    oracle.sweep(Cs, codes_s, r_s, 1, synth.init_indices(1500, M, K))      # some learned dictionaries
    C = Cs.copy()
    S = np.zeros((M, K, D))
    cnt = np.zeros((M, K), np.int64)
    codes, r, E = oracle.online_chunk(X8, C, S, cnt)
    C2 = Cs.copy()
    codes2 = np.zeros((1500, M), np.uint8)
    r2 = X8.astype(np.float64)
    for m in range(M):
        oracle.assign(r2, C2, codes2, m)
        oracle.update(r2, codes2, C2, m)
        oracle.assign(r2, C2, codes2, m)
        oracle.cool(r2, codes2, C2, m)
    np.testing.assert_array_equal(codes, codes2)
    np.testing.assert_allclose(C, C2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(r, r2, rtol=0, atol=1e-12)
    assert E == oracle.quant_error(r)
    assert np.all(cnt.sum(1) == 1500)


def test_online_running_mean_closed_form(oracle):
    """M = 1, K = 2 on a line: after chunk A then chunk B the codeword is the mean of all members
    it ever received, (n_A mean_A + n_B mean_B) / (n_A + n_B); prior counts weigh the old codeword."""
    A = np.array([[0], [2], [100], [104]], np.uint8)
    B = np.array([[4], [6], [110]], np.uint8)
    C = np.array([[[1.0], [90.0]]])
    S = np.zeros((1, 2, 1))
    cnt = np.zeros((1, 2), np.int64)
    oracle.online_chunk(A, C, S, cnt)
    np.testing.assert_array_equal(C.reshape(-1), [1.0, 102.0])
    codes, r, E = oracle.online_chunk(B, C, S, cnt)
    np.testing.assert_array_equal(C.reshape(-1), [(0 + 2 + 4 + 6) / 4.0, (100 + 104 + 110) / 3.0])
    np.testing.assert_array_equal(cnt, [[4, 3]])
    np.testing.assert_array_equal(codes[:, 0], [0, 0, 1])
    np.testing.assert_allclose(r.reshape(-1), [4 - 3.0, 6 - 3.0, 110 - 314 / 3.0], rtol=0, atol=1e-13)
    # prior counts: codeword 0 carries the weight of 10 earlier vectors at 1.0
    C = np.array([[[1.0], [90.0]]])
    cnt = np.array([[10, 0]], np.int64)
    S = C * cnt[:, :, None]
    oracle.online_chunk(A, C, S, cnt)
    np.testing.assert_allclose(C.reshape(-1), [(10 * 1.0 + 0 + 2) / 12.0, 102.0], rtol=1e-15)


# ---------------------------------------------------------------- improved k-means (Sec. 3.2)
def test_dimension_schedule():
    """d_i = d^(i/I), I = 10, rounded up and deduplicated; printed values for d = 128 are not in the
    paper, so the schedule is pinned by its defining properties."""
    for D in (16, 128, 960):
        d = oracle_dims(D)
        assert d[-1] == D and np.all(np.diff(d) > 0) and d[0] == int(np.ceil(D ** 0.1 - 1e-9))
        full = [D ** (i / 10) for i in range(1, 11)]
        assert all(any(abs(x - np.ceil(f - 1e-9)) < 1e-9 for f in full) for x in d)
    assert oracle_dims(128).tolist() == [2, 3, 5, 7, 12, 19, 30, 49, 79, 128]


def oracle_dims(D):
    import oracle
    return oracle.dimension_schedule(D, 10)


def test_rotate_against_matmul(oracle):
    g = np.random.default_rng(5)
    x = g.standard_normal((37, 6))
    R = np.linalg.qr(g.standard_normal((6, 6)))[0]
    np.testing.assert_allclose(oracle.rotate(x, R), x @ R.T, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.rotate(x, R, transpose=True), x @ R, rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.rotate(oracle.rotate(x, R), R, transpose=True), x, rtol=0, atol=1e-14)
    # not symmetric: a transposed R gives something else
    assert np.abs(x @ R.T - x @ R).max() > 1e-3


def test_pca_stage_full_dimension_is_rotation_invariant(oracle):
    """With the single prefix d_1 = D the improved k-means is plain Lloyd seen through an orthogonal
    map: same codes, same dictionary, same E as the plain stage, for any orthogonal R."""
    X = synth.tiny_gmm(N=1500)
    M, K, T = 2, 8, 3
    idx = synth.init_indices(1500, M, K)
    C1, codes1, r1 = _fresh_state(X, M, K)
    C2, codes2, r2 = _fresh_state(X, M, K)
    R = np.linalg.qr(np.random.default_rng(9).standard_normal((16, 16)))[0]
    for m in range(M):
        E1 = oracle.anneal_stage(m, C1, codes1, r1, T, idx[m])
        E2 = oracle.anneal_stage_pca(m, C2, codes2, r2, R, np.array([16], np.int32), T, idx[m])
        np.testing.assert_array_equal(codes1, codes2)
        np.testing.assert_allclose(C2, C1, rtol=0, atol=1e-12)
        np.testing.assert_allclose(E2, E1, rtol=1e-12)


def test_pca_stage_prefix_clusters_on_selected_coordinates(oracle):
    """R = a coordinate permutation: the first prefix then clusters on exactly those original
    coordinates.  One phase on d_1 coordinates followed by the full-dimension phase is checked
    against scikit-learn Lloyd on the selected columns, then on all columns started from the
    full-dimension means of the first clustering."""
    from sklearn.cluster import KMeans
    X = synth.tiny_gmm(N=2000).astype(np.float64)
    K, T, d1 = 8, 4, 6                        # chosen so that no cluster empties (the empty-cluster rules differ)
    perm = np.random.default_rng(5).permutation(16)
    R = np.eye(16)[perm]                      # (R x)_i = x_perm[i]
    idx = synth.init_indices(2000, 1, K)[0]
    C, codes, r = _fresh_state(X.astype(np.float32), 1, K)
    E = oracle.anneal_stage_pca(0, C, codes, r, R, np.array([d1, 16], np.int32), T, idx)
    sel = perm[:d1]
    km1 = KMeans(n_clusters=K, init=X[idx][:, sel], n_init=1, algorithm="lloyd", max_iter=T, tol=0.0).fit(X[:, sel])
    # sklearn's final labels are re-assigned after the last update; the method's memberships are those
    # of the T-th assignment, i.e. the labels a run with T-1 updates ends with
    km1b = KMeans(n_clusters=K, init=X[idx][:, sel], n_init=1, algorithm="lloyd", max_iter=T - 1, tol=0.0).fit(X[:, sel])
    lab = km1b.labels_
    np.testing.assert_allclose(np.stack([X[lab == k][:, sel].mean(0) for k in range(K)]), km1.cluster_centers_, atol=1e-12)
    start = np.stack([X[lab == k].mean(0) for k in range(K)])            # means over ALL coordinates
    km2 = KMeans(n_clusters=K, init=start, n_init=1, algorithm="lloyd", max_iter=T, tol=0.0).fit(X)
    assert len(np.unique(km2.labels_)) == K
    np.testing.assert_allclose(C[0], km2.cluster_centers_, rtol=0, atol=1e-11)
    np.testing.assert_array_equal(codes[:, 0], km2.labels_)
    np.testing.assert_allclose(E * 2000, km2.inertia_, rtol=1e-12)


def test_pca_axes_properties(oracle):
    X = synth.sift_like(3000, D=32).astype(np.float64)
    R = oracle.pca_axes(X)
    np.testing.assert_allclose(R @ R.T, np.eye(32), atol=1e-12)
    var = oracle.rotate(X - X.mean(0), R).var(0)
    assert np.all(np.diff(var) <= 1e-9 * var[0])                          # variance descending
    np.testing.assert_allclose(var.sum(), X.var(0).sum(), rtol=1e-12)     # trace preserved


# ---------------------------------------------------------------- dictionary order, code statistics
def test_code_statistics_closed_forms(oracle):
    """Sec. 2.2: H(I_m) of a uniform code part is log2 K; a part that copies another has mutual
    information H; independent parts have (nearly) none; H(A,B) = H(A) + H(B) - I(A;B)."""
    g = np.random.default_rng(8)
    K, N = 16, 200000
    codes = np.zeros((N, 3), np.uint8)
    codes[:, 0] = np.arange(N) % K                      # exactly uniform
    codes[:, 1] = codes[:, 0]                           # a copy
    codes[:, 2] = g.integers(0, K, N)                   # independent
    hist = oracle.code_histogram(codes, K)
    assert hist.sum(1).tolist() == [N, N, N] and np.all(hist[0] == N // K)
    assert abs(oracle.entropy_bits(hist[0]) - np.log2(K)) < 1e-12
    J01 = oracle.joint_histogram(codes, 0, 1, K)
    assert abs(oracle.mutual_information_bits(J01) - np.log2(K)) < 1e-12
    J02 = oracle.joint_histogram(codes, 0, 2, K)
    mi = oracle.mutual_information_bits(J02)
    assert 0 <= mi < 3 * (K - 1) ** 2 / (2 * N * np.log(2))          # plug-in bias ~ (K-1)^2 / (2 N ln 2)
    assert abs(oracle.entropy_bits(J02) - (oracle.entropy_bits(J02.sum(1)) + oracle.entropy_bits(J02.sum(0)) - mi)) < 1e-12
    np.testing.assert_array_equal(J02.sum(1), hist[0])
    np.testing.assert_array_equal(J02.sum(0), hist[2])


def test_variance_order(oracle):
    """Sec. 3.3: a hierarchy learned from scratch has descending variance; shuffling it and
    re-ordering by variance restores the hierarchy.  Variance against NumPy's definition."""
    X, C, codes = synth.planted_lattice(K=4, M=4, D=3, ratio=4.0)
    v = oracle.dictionary_variances(C)
    np.testing.assert_allclose(v, [np.var(C[m], axis=0).sum() for m in range(4)], rtol=1e-14)
    assert np.all(np.diff(v) < 0) and oracle.variance_order(C).tolist() == [0, 1, 2, 3]
    shuffle = [2, 0, 3, 1]
    # new position j must hold the shuffled slot that contains old dictionary j: the inverse permutation
    assert oracle.variance_order(C[shuffle]).tolist() == np.argsort(shuffle).tolist() == [1, 3, 0, 2]
    Ct = C.copy()
    Ct[3] = Ct[2]                                                          # a tie keeps the lower index first
    assert oracle.variance_order(Ct).tolist() == [0, 1, 2, 3]


# ---------------------------------------------------------------- multi-path encoding (Sec. 3.3)
def test_hand_worked_1d_beam(oracle):
    g = _read_golden("hand_1d_beam.txt")
    X = g["x"].astype(np.float32).reshape(1, 1)
    C = np.stack([g["c1"], g["c2"]]).reshape(2, 2, 1)
    codes, r, err, gap = oracle.encode_beam(X, C, 1)
    np.testing.assert_array_equal(codes[0], g["greedy_codes"].astype(np.uint8))
    assert err[0] == g["greedy_err"][0] and r[0, 0] == g["greedy_residue"][0]
    A0 = np.zeros((1, 1, 1))
    par, code, e, A1, _ = oracle.beam_step(X, C[0], A0, 2)
    np.testing.assert_array_equal(code[0], g["beam2_step1_code"].astype(np.uint8))
    np.testing.assert_array_equal(e[0], g["beam2_step1_err"])
    par, code, e, A2, _ = oracle.beam_step(X, C[1], A1, 2)
    np.testing.assert_array_equal(par[0], g["beam2_step2_parent"].astype(np.uint8))
    np.testing.assert_array_equal(code[0], g["beam2_step2_code"].astype(np.uint8))
    np.testing.assert_array_equal(e[0], g["beam2_step2_err"])
    codes, r, err, gap = oracle.encode_beam(X, C, 2)
    np.testing.assert_array_equal(codes[0], g["beam2_codes"].astype(np.uint8))
    assert err[0] == g["beam2_err"][0] and r[0, 0] == g["beam2_residue"][0] and gap[0] == g["beam2_gap"][0]


def _beam_inputs(N=300, D=6, M=3, K=4, seed=3):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(N, D)).astype(np.float32)
    C = rng.normal(size=(M, K, D)) * (0.6 ** np.arange(M))[:, None, None]
    return X, C


def test_beam_single_path_is_greedy(oracle):
    """Eq. 3 with L = 1 keeps the nearest codeword of the running residue at every dictionary."""
    X, C = _beam_inputs(M=4, K=8)
    c1, r1 = oracle.encode(X, C)
    c2, r2, e2, _ = oracle.encode_beam(X, C, 1)
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_allclose(r1, r2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(e2, (r2 ** 2).sum(1), rtol=1e-13)


def test_beam_wide_enough_is_exhaustive(oracle):
    """With L >= K^(M-1) no prefix is ever dropped, so the result is the global minimiser of the
    first line of Eq. 1 over all K^M codes (brute force).  Catches a wrong sign, a wrong parent
    index and a mis-carried prefix."""
    import itertools
    X, C = _beam_inputs()
    M, K, _ = C.shape
    best = np.full(len(X), np.inf)
    bc = np.zeros((len(X), M), np.uint8)
    for combo in itertools.product(range(K), repeat=M):
        e = ((X - sum(C[m][combo[m]] for m in range(M))) ** 2).sum(1)
        u = e < best
        best[u] = e[u]
        bc[u] = combo
    for L in (K ** (M - 1), K ** M, 1000):
        codes, r, err, _ = oracle.encode_beam(X, C, L)
        np.testing.assert_array_equal(codes, bc)
        np.testing.assert_allclose(err, best, rtol=1e-13)
        np.testing.assert_allclose(r, X - oracle.reconstruct(C, codes), rtol=0, atol=1e-14)
    # a narrower beam can only be as good or worse than the exhaustive answer
    for L in (1, 2, 5):
        _, _, err, _ = oracle.encode_beam(X, C, L)
        assert (err >= best - 1e-12).all()


def test_beam_step_equals_eq3_with_lookup_tables(oracle):
    """Eq. 3 as printed: ||x - a_l||^2 + ||x - c_m(k)||^2 - ||x||^2 + 2 c_m(k)^T a_l, the last term
    from inner products of dictionary elements tabulated beforehand.  A separate NumPy beam built
    on those tables must keep the same sums as the direct-form oracle."""
    X, C = _beam_inputs(N=200, D=8, M=4, K=6, seed=11)
    M, K, D = C.shape
    L = 5
    X64 = X.astype(np.float64)
    flat = C.reshape(M * K, D)
    T = (flat @ flat.T).reshape(M, K, M, K)                  # c_a(i)^T c_b(j)
    xx = (X64 ** 2).sum(1)
    codes_o, r_o, err_o, gap = oracle.encode_beam(X, C, L)
    for n in range(len(X)):
        pre = [()]
        e_cur = np.array([xx[n]])                            # ||x - 0||^2
        for m in range(M):
            tab = ((X64[n][None, :] - C[m]) ** 2).sum(1)     # second term, one per k
            sc = np.empty((len(pre), K))
            for l, p in enumerate(pre):
                cross = sum(T[j, p[j], m, :] for j in range(m)) if m else np.zeros(K)
                sc[l] = e_cur[l] + tab - xx[n] + 2.0 * cross
            order = np.argsort(sc.reshape(-1), kind="stable")[: min(L, sc.size)]
            e_cur = sc.reshape(-1)[order]
            pre = [pre[o // K] + (o % K,) for o in order]
        if gap[n] > 1e-9:                                    # expanded and direct forms differ by rounding
            assert tuple(codes_o[n]) == pre[0]
        np.testing.assert_allclose(err_o[n], e_cur[0], rtol=1e-9, atol=1e-12)
    assert (gap > 1e-9).mean() > 0.9


def test_beam_tie_order_and_gap(oracle):
    """Equal errors are kept in (l, k) order and reported as a zero gap."""
    X = np.array([[1.0, 0.0]], np.float32)
    Cm = np.array([[1.0, 1.0], [1.0, -1.0], [0.0, 0.0], [1.0, 1.0]])   # k = 0, 1, 3 tie at e = 1
    A = np.zeros((1, 1, 2))
    par, code, err, A1, gap = oracle.beam_step(X, Cm, A, 3)
    assert code[0].tolist() == [0, 1, 2] and err[0].tolist() == [1.0, 1.0, 1.0] and gap[0] == 0.0
    # two identical beam entries: children of the lower l come first
    A = np.zeros((1, 2, 2))
    par, code, err, A2, gap = oracle.beam_step(X, Cm, A, 4)
    assert list(zip(par[0].tolist(), code[0].tolist())) == [(0, 0), (0, 1), (0, 2), (0, 3)]
    par, code, err, A2, gap = oracle.beam_step(X, np.array([[1.0, 1.0], [1.0, 0.0]]), A, 3)
    assert list(zip(par[0].tolist(), code[0].tolist())) == [(0, 1), (1, 1), (0, 0)]
