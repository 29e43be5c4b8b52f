"""GPU-vs-oracle parity of every step of the DA stage (arXiv 1509.05194, Sec. 3.1), through the
C ABI.  Step-locked: both sides start each step from the same fp32 state.  Bars: codes
bit-exact outside oracle near-ties (top-2 gap < 1e-5 relative); codebooks, residues and
quantization error within 1e-4 relative (much tighter bounds are asserted where the
arithmetic allows)."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth
from parity_util import fresh_state, judge_codes, narrow_state, rel_fro, to_dev

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


_CONTRACTION = 0


@pytest.fixture(autouse=True, params=[0, 1], ids=["f32", "splitbf16"])
def contraction(request):
    """Every test of this module runs with both matrix-core arithmetics of the distance contraction
    (hclae_set_contraction): the bar is the same, since both only pre-select candidates for the fp64
    re-check."""
    global _CONTRACTION
    _CONTRACTION = request.param
    yield request.param
    _CONTRACTION = 0


def _ctx(N, D, M, K):
    from paper_1509_05194_amd import hclae
    ctx = hclae.Context(N, D, M, K)
    ctx.set_contraction(_CONTRACTION)
    return ctx


# shapes: several tiles plus a ragged tail; padded K and D; the D-chunked path (D = 960, 132)
CASES = {
    "tiny":    dict(gen="tiny", N=10000, D=16, M=4, K=16, T=2),
    "sift":    dict(gen="sift", N=20000 + 37, D=128, M=4, K=256, T=2),
    "odd":     dict(gen="sift", N=1000 + 3, D=36, M=3, K=17, T=2),
    "k40d132": dict(gen="sift", N=3000 + 1, D=132, M=2, K=40, T=1),
    "gist":    dict(gen="gist", N=3000 + 5, D=960, M=2, K=256, T=1),
    "k256d132": dict(gen="sift", N=2000 + 9, D=132, M=2, K=256, T=1),
    # D-chunked with one, two and four 32-codeword blocks (odd and even slice counts, a ragged last slice)
    "k16d2052": dict(gen="gist", N=1500 + 3, D=2052, M=2, K=16, T=1),
    "k40d960": dict(gen="gist", N=2000 + 1, D=960, M=2, K=40, T=1),
    "k100d512": dict(gen="gist", N=2000 + 7, D=512, M=2, K=100, T=1),
    # D-chunked with more block tiles (256 vectors each) than CUs: blocks walk several tiles, and the refills
    # of the last slice of a tile already belong to the next one
    "k256d132n": dict(gen="sift", N=3 * 65536 + 300 + 11, D=132, M=1, K=256, T=1),
    # one codeword per dictionary: stage 0 takes the mean out, so the codeword of stage 1 is the mean of a
    # centred residue -- zero up to rounding
    "k1m2": dict(gen="tiny", N=761, D=144, M=2, K=1, T=1),
}


def _random_shapes(seed, count, n_max):
    """Seeded random shapes: any D that is a multiple of 4 (LDS-resident and D-chunked dictionaries, ragged
    last slices), any K (padded codeword blocks), N from a few vectors to several tiles."""
    g = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        K = int(g.choice([int(g.integers(1, 9)), int(g.integers(9, 257))]))
        D = 4 * int(g.choice([int(g.integers(1, 40)), int(g.integers(40, 560))]))
        N = int(g.integers(K + 1, n_max))
        out.append(dict(gen=str(g.choice(["sift", "gist", "tiny"])), N=N, D=D, M=int(g.integers(1, 4)), K=K,
                        T=int(g.integers(1, 4))))
    return out


for _i, _c in enumerate(_random_shapes(1509, 6, 4000)):
    CASES["rnd%d" % _i] = _c
_cache = {}


def _data(case):
    c = CASES[case]
    if c["gen"] == "tiny":
        return synth.tiny_gmm(N=c["N"], D=c["D"])
    if c["gen"] == "sift":
        return synth.sift_like(c["N"], D=c["D"])
    return synth.gist_like(c["N"], D=c["D"])


def _mid_state(case, oracle):
    """A realistic mid-sweep oracle state: one fresh sweep of T iterations."""
    if case not in _cache:
        c = CASES[case]
        X = _data(case)
        C, codes, r = fresh_state(X, c["M"], c["K"])
        idx = synth.init_indices(c["N"], c["M"], c["K"])
        oracle.sweep(C, codes, r, c["T"], idx)
        _cache[case] = (X, C, codes, r, idx)
    X, C, codes, r, idx = _cache[case]
    return X, C.copy(), codes.copy(), r.copy(), idx


@pytest.mark.parametrize("case", list(CASES))
def test_heat_and_cool_step(case, oracle):
    c = CASES[case]
    X, C, codes, r, _ = _mid_state(case, oracle)
    ctx = _ctx(c["N"], c["D"], c["M"], c["K"])
    for m in (0, c["M"] - 1):
        Cg, codes_g, rg, C64, codes64, r64 = narrow_state(C, codes, r)
        ctx.heat(m, Cg, codes_g, rg)
        oracle.heat(r64, codes64, C64, m)
        # one fp32 add per element: half an ulp of the result
        got = rg.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - r64) <= 6.0e-8 * np.abs(r64) + 1e-45)
        ctx.cool(m, Cg, codes_g, rg)
        xp64 = got.copy()
        oracle.cool(xp64, codes64, C64, m)
        got2 = rg.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got2 - xp64) <= 6.0e-8 * np.abs(xp64) + 1e-45)
    ctx.close()


@pytest.mark.parametrize("case", list(CASES))
def test_assign_step(case, oracle):
    c = CASES[case]
    X, C, codes, r, _ = _mid_state(case, oracle)
    N, M = c["N"], c["M"]
    ctx = _ctx(N, c["D"], M, c["K"])
    for m in range(M):
        Cg, codes_g, rg, C64, codes64, r64 = narrow_state(C, codes, r)
        oracle.heat(r64, codes64, C64, m)
        xg = to_dev(r64.astype(np.float32))          # x' as fp32, identical on both sides
        x64 = r64.astype(np.float32).astype(np.float64)
        codes_g.fill_(255)
        codes_g[:, m] = 0
        dmin = torch.empty(N, dtype=torch.float32, device="cuda:0")
        ctx.assign(m, xg, Cg, codes_g, dmin)
        refined = ctx.last_refined()
        d1, d2, _ = oracle.assign(x64, C64, codes64, m, top2=True)
        got = codes_g.cpu().numpy()
        others = [j for j in range(M) if j != m]
        assert np.all(got[:, others] == 255), "assign wrote outside column m"
        ndiff, nexempt, bad = judge_codes(oracle, x64, C64, m, got[:, m], codes64[:, m], d1, d2)
        print("%s m=%d: differ %d, exempt %d, refined %d of %d" % (case, m, ndiff, nexempt, refined, N))
        assert not bad, "non-exempt code mismatches at %s" % bad[:10]
        same = got[:, m] == codes64[:, m]
        dm = dmin.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(dm[same] - d1[same]) <= 2e-7 * d1[same] + 1e-30)
    ctx.close()


@pytest.mark.parametrize("case", list(CASES))
def test_update_step(case, oracle):
    c = CASES[case]
    X, C, codes, r, _ = _mid_state(case, oracle)
    N, M, K = c["N"], c["M"], c["K"]
    ctx = _ctx(N, c["D"], M, K)
    m = M - 1
    Cg, codes_g, rg, C64, codes64, r64 = narrow_state(C, codes, r)
    oracle.heat(r64, codes64, C64, m)
    x32 = r64.astype(np.float32)
    # empty two clusters on purpose: their members move to cluster 0
    if K > 3:
        col = codes64[:, m]
        col[(col == 1) | (col == K - 1)] = 0
        codes_g = to_dev(codes64)
    xg = to_dev(x32)
    C_before = Cg.cpu().numpy().copy()
    counts = torch.zeros(K, dtype=torch.int32, device="cuda:0")
    ctx.update(m, xg, Cg, codes_g, counts)
    x64 = x32.astype(np.float64)
    cnt_o, empty_o = oracle.update(x64, codes64, C64, m)
    got = Cg.cpu().numpy()
    np.testing.assert_array_equal(counts.cpu().numpy().astype(np.int64), cnt_o)
    for j in range(M):
        if j != m:
            np.testing.assert_array_equal(got[j], C_before[j])
    emp = cnt_o == 0
    np.testing.assert_array_equal(got[m][emp], C_before[m][emp])       # empty clusters keep their codeword
    scale = np.linalg.norm(C64[m]) / np.sqrt(K)
    row_abs = np.linalg.norm(got[m].astype(np.float64) - C64[m], axis=1)
    # the sums are taken on integers q = round(x' * 2^s) with max |q| in [2^29, 2^30): every element of a mean
    # is within half a step = max |x'| * 2^-30 of the exact one, whatever the codeword's own size (a codeword
    # that is a cancellation residue has no relative accuracy to speak of, in any finite arithmetic)
    floor = np.sqrt(c["D"]) * np.abs(x64).max() * 2.0 ** -30
    print("%s update: max row err %.2e (rel. to rms codeword norm %.3g), fixed-point floor %.2e, empty %d"
          % (case, row_abs.max() / scale, scale, floor, empty_o))
    assert np.all(row_abs <= 1e-5 * scale + floor)
    # run-to-run determinism: identical bits
    Cg2 = to_dev(C_before)
    ctx.update(m, xg, Cg2, codes_g, None)
    assert torch.equal(Cg, Cg2)
    ctx.close()


@pytest.mark.parametrize("case", ["tiny", "sift", "gist"])
def test_quant_error(case, oracle):
    c = CASES[case]
    X, C, codes, r, _ = _mid_state(case, oracle)
    ctx = _ctx(c["N"], c["D"], c["M"], c["K"])
    r32 = r.astype(np.float32)
    E = ctx.quant_error(to_dev(r32))
    Eo = oracle.quant_error(r32.astype(np.float64))
    assert abs(E - Eo) <= 1e-12 * Eo
    ctx.close()


@pytest.mark.parametrize("case", ["tiny", "sift", "odd", "gist", "k1m2"])
def test_encode(case, oracle):
    """Greedy encoding (Eq. 3, L=1).  A vector is followed stage by stage until its first
    differing code, which must be an exempt near-tie of that stage; later parts of such a
    vector are not compared (its residue has legitimately changed)."""
    c = CASES[case]
    X, C, _, _, _ = _mid_state(case, oracle)
    N, M, K, D = c["N"], c["M"], c["K"], c["D"]
    C32 = C.astype(np.float32)
    C64 = C32.astype(np.float64)
    ctx = _ctx(N, D, M, K)
    Xg, Cg = to_dev(X), to_dev(C32)
    codes_g = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    rg = torch.empty((N, D), dtype=torch.float32, device="cuda:0")
    ctx.encode(Xg, Cg, codes_g, rg)
    got = codes_g.cpu().numpy()
    r64 = X.astype(np.float64)
    codes_o = np.zeros((N, M), np.uint8)
    alive = np.ones(N, bool)
    n_exempt = 0
    for m in range(M):
        d1, d2, _ = oracle.assign(r64, C64, codes_o, m, top2=True)
        ndiff, nex, bad = judge_codes(oracle, r64, C64, m, np.where(alive, got[:, m], codes_o[:, m]),
                                      codes_o[:, m], d1, d2)
        assert not bad, "stage %d: non-exempt mismatches %s" % (m, bad[:10])
        n_exempt += nex
        alive &= got[:, m] == codes_o[:, m]
        oracle.cool(r64, codes_o, C64, m)
    print("%s encode: exempt %d, compared to the end %d of %d" % (case, n_exempt, alive.sum(), N))
    res = rg.cpu().numpy().astype(np.float64)
    scale = np.sqrt((r64 ** 2).sum(1).mean())
    err = np.linalg.norm(res[alive] - r64[alive], axis=1) / scale
    assert err.max() <= 1e-5
    E = ctx.quant_error(rg)
    assert abs(E - oracle.quant_error(r64)) <= 1e-4 * oracle.quant_error(r64)
    # x = sum_m C_m[i_m] + r on the GPU's own output
    recon = oracle.reconstruct(C64, got) + res
    assert np.abs(recon - X).max() <= 1e-5 * max(np.abs(X).max(), 1.0)
    ctx.close()


def _lockstep_stage(ctx, oracle, m, T, Cg, codes_g, rg, C64, codes64, r64, idx):
    """Drive one stage step by step on both sides; after each assign the oracle adopts every
    exempt GPU code so the trajectories stay locked.  Returns the number adopted."""
    adopted = 0
    ctx.heat(m, Cg, codes_g, rg)
    oracle.heat(r64, codes64, C64, m)
    if idx is not None:
        Cg[m] = rg[torch.from_numpy(idx).to(rg.device)]        # test-side seeding (buffer copy only)
        C64[m] = r64[idx]
    for t in range(T + 1):
        ctx.assign(m, rg, Cg, codes_g)
        d1, d2, _ = oracle.assign(r64, C64, codes64, m, top2=True)
        got = codes_g.cpu().numpy()[:, m]
        ndiff, nex, bad = judge_codes(oracle, r64, C64, m, got, codes64[:, m], d1, d2)
        assert not bad, "stage %d assign %d: non-exempt mismatches %s" % (m, t, bad[:10])
        adopted += nex
        codes64[:, m] = got
        if t < T:
            ctx.update(m, rg, Cg, codes_g)
            oracle.update(r64, codes64, C64, m)
            # 1e-5 relative, plus what a mean inherits from a state kept in fp32 while the other side keeps fp64:
            # half an ulp of the largest |x'| per element.  That is all there is to a codeword that cancels to
            # zero (K = 1 after the mean has been taken out).
            diff = np.linalg.norm(Cg[m].cpu().numpy().astype(np.float64) - C64[m])
            assert diff <= 1e-5 * np.linalg.norm(C64[m]) + np.sqrt(C64[m].size) * np.abs(r64).max() * 2.0 ** -24
    ctx.cool(m, Cg, codes_g, rg)
    oracle.cool(r64, codes64, C64, m)
    return adopted


@pytest.mark.parametrize("case", ["tiny", "sift", "k1m2"])
def test_lockstep_sweeps(case, oracle):
    """Fresh sweep then an annealing sweep, free-running on the GPU state, with tie adoption."""
    c = CASES[case]
    N, D, M, K, T = c["N"], c["D"], c["M"], c["K"], 3
    X = _data(case)
    idx = synth.init_indices(N, M, K)
    ctx = _ctx(N, D, M, K)
    C64, codes64, r64 = fresh_state(X, M, K)
    Cg = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes_g = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    rg = to_dev(X)
    adopted = 0
    for sweep in range(2):
        for m in range(M):
            adopted += _lockstep_stage(ctx, oracle, m, T, Cg, codes_g, rg, C64, codes64, r64,
                                       idx[m] if sweep == 0 else None)
            Eg, Eo = ctx.quant_error(rg), oracle.quant_error(r64)
            assert abs(Eg - Eo) <= 1e-4 * Eo
            assert rel_fro(rg.cpu().numpy(), r64) <= 1e-4
    print("%s lockstep: adopted %d near-ties over %d assigns" % (case, adopted, 2 * M * (T + 1)))
    assert rel_fro(Cg.cpu().numpy(), C64) <= 1e-4
    ctx.close()


def test_free_running_sweeps_tiny(oracle):
    """Three hclae_sweep calls on config-1 data (10,000 x 16, M=4, K=16) against the oracle's."""
    c = CASES["tiny"]
    N, D, M, K, T = c["N"], c["D"], c["M"], c["K"], 10
    X = _data("tiny")
    idx = synth.init_indices(N, M, K)
    ctx = _ctx(N, D, M, K)
    C64, codes64, r64 = fresh_state(X, M, K)
    Cg = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes_g = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    rg = to_dev(X)
    prev = None
    for s in range(3):
        Eo = oracle.sweep(C64, codes64, r64, T, idx if s == 0 else None)
        Eg = ctx.sweep(Cg, codes_g, rg, T, init_idx=idx if s == 0 else None)
        mism = float((codes_g.cpu().numpy() != codes64).mean())
        print("sweep %d: E gpu %s oracle %s, code mismatch %.2e, C err %.2e"
              % (s, Eg, Eo, mism, rel_fro(Cg.cpu().numpy(), C64)))
        np.testing.assert_allclose(Eg, Eo, rtol=1e-4)
        assert np.all(np.diff(Eg) <= 0) and (prev is None or Eg[0] <= prev * (1 + 1e-6))
        prev = Eg[-1]
        if mism == 0.0:
            assert rel_fro(Cg.cpu().numpy(), C64) <= 1e-4
            assert rel_fro(rg.cpu().numpy(), r64) <= 1e-4
    ctx.close()


def test_stage_stats_and_reencode_mode(oracle):
    c = CASES["tiny"]
    N, D, M, K = c["N"], c["D"], c["M"], c["K"]
    X, C, codes, r, _ = _mid_state("tiny", oracle)
    ctx = _ctx(N, D, M, K)
    Cg, codes_g, rg, C64, codes64, r64 = narrow_state(C, codes, r)
    before = codes_g.clone()
    E0 = oracle.quant_error(r64)
    st = ctx.anneal_stage(1, Cg, codes_g, rg, 2)
    E1 = oracle.anneal_stage(1, C64, codes64, r64, 2)
    assert abs(st["err_before"] - E0) <= 1e-6 * E0 and abs(st["err_after"] - E1) <= 1e-4 * E1
    assert st["iters_run"] == 2 and st["empty_clusters"] == 0
    assert st["codes_changed"] == int((codes_g[:, 1] != before[:, 1]).sum())
    assert st["err_after"] <= st["err_before"]
    # reencode_mode 1: state after the sweep is the greedy encoding of X under the final C
    Xg = to_dev(X)
    ctx.sweep(Cg, codes_g, rg, 1, X=Xg, reencode_mode=1)
    codes2 = torch.zeros_like(codes_g)
    r2 = torch.empty_like(rg)
    ctx.encode(Xg, Cg, codes2, r2)
    assert torch.equal(codes2, codes_g) and torch.equal(r2, rg)
    ctx.close()


def test_exact_integer_regime(oracle):
    """Integer-valued data in [0,255] with codewords that are data rows: every product and
    partial sum of the first assignment is an integer below 2^24, so fp32 is exact and the
    codes must equal the oracle's with no exemption, exact ties included."""
    N, D, K = 50000 + 11, 128, 256
    X = synth.sift_like(N, D=D)
    X[1000:1200] = X[:200]                    # exact duplicates of other rows
    idx = synth.init_indices(N, 1, K)[0]
    idx[5] = 1003                             # two seeds that are duplicates of each other: an exact tie
    idx[200] = 3
    ctx = _ctx(N, D, 1, K)
    C32 = X[idx][None].copy()
    Cg, xg = to_dev(C32), to_dev(X)
    codes_g = torch.zeros((N, 1), dtype=torch.uint8, device="cuda:0")
    ctx.assign(0, xg, Cg, codes_g)
    codes_o = np.zeros((N, 1), np.uint8)
    oracle.assign(X.astype(np.float64), C32.astype(np.float64), codes_o, 0)
    np.testing.assert_array_equal(codes_g.cpu().numpy(), codes_o)
    assert codes_o[1003, 0] == 5 and codes_o[3, 0] == 5      # the tie went to the lower index
    ctx.close()


def test_degenerate_shapes(oracle):
    """K = 1, M = 1, N below one tile, N = 0, all-zero dictionaries (every score ties)."""
    from paper_1509_05194_amd import hclae
    # K = 1
    X = synth.tiny_gmm(N=500, D=16)
    ctx = _ctx(500, 16, 2, 1)
    Cg = torch.zeros((2, 1, 16), dtype=torch.float32, device="cuda:0")
    codes_g = torch.zeros((500, 2), dtype=torch.uint8, device="cuda:0")
    rg = to_dev(X)
    E = ctx.sweep(Cg, codes_g, rg, 1, init_idx=np.array([[3], [4]], np.int64))
    mean = X.astype(np.float64).mean(0)
    assert np.abs(Cg[0, 0].cpu().numpy() - mean).max() <= 1e-6
    assert abs(E[0] - ((X - mean) ** 2).sum(1).mean()) <= 1e-5 * E[0]
    assert int(codes_g.max()) == 0
    # N = 0 is a no-op
    empty_r = torch.empty((0, 16), dtype=torch.float32, device="cuda:0")
    assert ctx.quant_error(empty_r) == 0.0
    ctx.heat(0, Cg, torch.empty((0, 2), dtype=torch.uint8, device="cuda:0"), empty_r)
    ctx.close()
    # tiny N, all-zero dictionaries: every codeword ties, lowest index wins
    for N in (1, 31, 33):
        X = synth.sift_like(N, D=128)
        ctx = _ctx(N, 128, 3, 256)
        Cg = torch.zeros((3, 256, 128), dtype=torch.float32, device="cuda:0")
        codes_g = torch.full((N, 3), 9, dtype=torch.uint8, device="cuda:0")
        rg = torch.empty((N, 128), dtype=torch.float32, device="cuda:0")
        ctx.encode(to_dev(X), Cg, codes_g, rg)
        assert int(codes_g.max()) == 0 and torch.equal(rg.cpu(), torch.from_numpy(X))
        ctx.close()
    # shape mismatch against the ctx, and N beyond N_max
    ctx = _ctx(100, 16, 2, 4)
    L = hclae.lib()
    assert L.hclae_heat(ctx._h, 0, 10, 32, None, 2, 4, None, None) == hclae.ESTATE
    assert L.hclae_heat(ctx._h, 0, 101, 16, None, 2, 4, None, None) == hclae.ESTATE
    assert L.hclae_heat(ctx._h, 2, 10, 16, None, 2, 4, None, None) == hclae.EINVAL
    # a float array whose base is not 16-byte aligned is refused before anything is launched
    flat = torch.zeros(10 * 16 + 4, dtype=torch.float32, device="cuda:0")
    good, off = flat[:160].view(10, 16), flat[1:161].view(10, 16)
    Cs = torch.zeros((2, 4, 16), dtype=torch.float32, device="cuda:0")
    cs = torch.zeros((10, 2), dtype=torch.uint8, device="cuda:0")
    assert off.data_ptr() % 16 == 4
    with pytest.raises(hclae.HclaeError) as e:
        ctx.heat(0, Cs, cs, off)
    assert e.value.code == hclae.EINVAL and b"aligned" in L.hclae_last_error(ctx._h)
    with pytest.raises(hclae.HclaeError):
        ctx.sweep(Cs, cs, off, 1)
    with pytest.raises(hclae.HclaeError):
        ctx.encode(off, Cs, cs, good)
    ctx.heat(0, Cs, cs, good)
    ctx.close()


@pytest.mark.parametrize("case", ["tiny", "sift", "gist"])
def test_sweep_equals_stage_by_stage(case, oracle):
    """hclae_sweep fuses the end of stage m with the heat of stage m+1 into one pass; the result must
    equal calling hclae_anneal_stage for m = 0..M-1 bit for bit, stats included."""
    c = CASES[case]
    N, D, M, K = c["N"], c["D"], c["M"], c["K"]
    X = _data(case)
    idx = synth.init_indices(N, M, K)
    ctx = _ctx(N, D, M, K)
    outs = []
    for fused in (True, False):
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        r = to_dev(X)
        errs = []
        for s in range(2):
            ii = idx if s == 0 else None
            if fused:
                errs.append(ctx.sweep(C, codes, r, 2, init_idx=ii))
            else:
                errs.append(np.array([ctx.anneal_stage(m, C, codes, r, 2, ii[m] if ii is not None else None)["err_after"]
                                      for m in range(M)]))
        outs.append((C, codes, r, np.concatenate(errs)))
    assert torch.equal(outs[0][0], outs[1][0])
    assert torch.equal(outs[0][1], outs[1][1])
    assert torch.equal(outs[0][2], outs[1][2])
    np.testing.assert_array_equal(outs[0][3], outs[1][3])
    ctx.close()


@pytest.mark.parametrize("shape", [dict(N=300 + 7, D=4096, M=1, K=256), dict(N=400 + 1, D=4, M=256, K=3),
                                   dict(N=257, D=64, M=2, K=256)])
def test_limits_of_the_shape_check(shape, oracle):
    """Largest D and M the ABI accepts, the smallest D, K = 256 with D = 64 (one register chunk)."""
    N, D, M, K = shape["N"], shape["D"], shape["M"], shape["K"]
    g = np.random.default_rng(N)
    X = g.standard_normal((N, D)).astype(np.float32)
    idx = np.stack([g.choice(N, K, replace=False) for _ in range(M)]).astype(np.int64)
    T = 1
    stages = min(M, 3)
    C64, codes64, r64 = fresh_state(X, M, K)
    ctx = _ctx(N, D, M, K)
    Cg = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes_g = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    rg = to_dev(X)
    adopted = 0
    for m in list(range(stages - 1)) + [M - 1]:
        adopted += _lockstep_stage(ctx, oracle, m, T, Cg, codes_g, rg, C64, codes64, r64, idx[m])
    assert rel_fro(Cg.cpu().numpy(), C64) <= 1e-5
    # with N close to K most vectors are their own codeword and the residue is (nearly) zero:
    # measure its error against the scale of the data
    assert np.linalg.norm(rg.cpu().numpy().astype(np.float64) - r64) <= 1e-6 * np.linalg.norm(X)
    Eo = oracle.quant_error(r64)
    assert abs(ctx.quant_error(rg) - Eo) <= 1e-5 * Eo + 1e-10 * float((X.astype(np.float64) ** 2).sum(1).mean())
    ctx.close()


@pytest.mark.parametrize("gen,N,D,M,K,T", [("sift", 40000 + 9, 128, 3, 256, 6), ("gist", 6000 + 5, 960, 2, 256, 5),
                                           ("tiny", 10000 + 3, 16, 4, 16, 6), ("sift", 8000 + 1, 132, 2, 40, 4),
                                           ("gist", 5000 + 3, 512, 2, 100, 4), ("gist", 3000 + 7, 1412, 2, 20, 4),
                                           ("sift", 2 * 65536 + 5000 + 5, 132, 1, 256, 4)]
                         + [(c["gen"], c["N"], c["D"], c["M"], c["K"], c["T"] + 2) for c in _random_shapes(5194, 10, 9000)])
def test_stage_equals_its_single_steps_bitwise(gen, N, D, M, K, T):
    """hclae_anneal_stage prunes its Lloyd iterations (distance bounds; centroid sums advanced by the moved
    vectors, exact integer totals); the single-step calls run every assignment and every sum over all
    vectors.  Both must give the same bits: dictionaries, codes, residues.  Shapes: LDS-resident and
    D-chunked dictionaries, padded K and D."""
    X = {"sift": lambda: synth.sift_like(N, D=D), "gist": lambda: synth.gist_like(N, D=D),
         "tiny": lambda: synth.tiny_gmm(N=N, D=D)}[gen]()
    idx = synth.init_indices(N, M, K)
    out = []
    for one_call in (True, False):
        ctx = _ctx(N, D, M, K)
        Xg = to_dev(X)
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        r = Xg.clone()
        for sweep in range(2):
            for m in range(M):
                if one_call:
                    ctx.anneal_stage(m, C, codes, r, T, init_idx=idx[m] if sweep == 0 else None, want_stats=False)
                else:
                    ctx.heat(m, C, codes, r)
                    if sweep == 0:
                        C[m] = r[torch.from_numpy(idx[m]).cuda()]
                    for _ in range(T):
                        ctx.assign(m, r, C, codes)
                        ctx.update(m, r, C, codes)
                    ctx.assign(m, r, C, codes)
                    ctx.cool(m, C, codes, r)
        torch.cuda.synchronize()
        out.append((C.clone(), codes.clone(), r.clone()))
        ctx.close()
    assert torch.equal(out[0][0], out[1][0]), "dictionaries differ"
    assert torch.equal(out[0][1], out[1][1]), "codes differ"
    assert torch.equal(out[0][2], out[1][2]), "residues differ"
