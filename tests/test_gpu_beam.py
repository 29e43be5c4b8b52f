"""Multi-path encoding (Sec. 3.3, Eq. 3 of arXiv 1509.05194) on the GPU against the oracle: one
dictionary at a time from the oracle's own beam (step-locked), the whole encoder, and the sweep
that re-encodes with it."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth
from parity_util import REL_GAP, fresh_state, to_dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

SHAPES = {
    "tiny": dict(gen="tiny", N=3000 + 3, D=16, M=3, K=16),
    "sift": dict(gen="sift", N=3000 + 5, D=128, M=4, K=256),
    "k100": dict(gen="sift", N=1500 + 1, D=20, M=3, K=100),
    "gist": dict(gen="gist", N=600 + 7, D=960, M=2, K=256),
    # D-chunked scoring with more block tiles than CUs (24 vectors per block tile at L = 10)
    "d132n": dict(gen="sift", N=7000 + 3, D=132, M=2, K=256),
}


def _data(c):
    if c["gen"] == "tiny":
        return synth.tiny_gmm(N=c["N"], D=c["D"])
    if c["gen"] == "sift":
        return synth.sift_like(c["N"], D=c["D"])
    return synth.gist_like(c["N"], D=c["D"])


def _dictionaries(oracle, X, M, K, T=2):
    """DA dictionaries learned from scratch by the oracle, narrowed to fp32 (both sides then use the
    exact widening of those)."""
    C, codes, r = fresh_state(X, M, K)
    oracle.sweep(C, codes, r, T, synth.init_indices(X.shape[0], M, K))
    C32 = C.astype(np.float32)
    return C32, C32.astype(np.float64)


_CONTRACTION = 0


@pytest.fixture(autouse=True, params=[0, 1], ids=["f32", "splitbf16"])
def contraction(request):
    """Both matrix-core arithmetics of the scoring contraction (hclae_set_contraction); same bar."""
    global _CONTRACTION
    _CONTRACTION = request.param
    yield request.param
    _CONTRACTION = 0


def _ctx(c):
    from paper_1509_05194_amd import hclae
    ctx = hclae.Context(c["N"], c["D"], c["M"], c["K"])
    ctx.set_contraction(_CONTRACTION)
    return ctx


def _cand_err(X64, A, Cm, par, code):
    """fp64 direct-form error of the candidates (par, code) chosen per vector."""
    n = np.arange(X64.shape[0])[:, None]
    t = X64[:, None, :] - A[n, par] - Cm[code]
    return (t * t).sum(-1)


@pytest.mark.parametrize("case,L", [("tiny", 1), ("tiny", 3), ("tiny", 10), ("tiny", 32), ("sift", 2), ("sift", 10),
                                    ("sift", 16), ("sift", 32), ("k100", 10), ("k100", 7), ("gist", 10), ("gist", 4),
                                    ("d132n", 10)])
def test_beam_step_locked(case, L, oracle):
    """Every dictionary: the GPU starts from the oracle's beam (residuals narrowed to fp32) and must
    keep the same sums in the same order wherever the oracle's neighbouring errors differ by more than
    1e-5 relative; elsewhere its choice must be as good within that tolerance."""
    c = SHAPES[case]
    X = _data(c)
    N, D, M, K = c["N"], c["D"], c["M"], c["K"]
    C32, C64 = _dictionaries(oracle, X, M, K)
    X64 = X.astype(np.float64)
    ctx = _ctx(c)
    A = np.zeros((N, 1, D))
    err_c = (X64 ** 2).sum(1)[:, None]
    scale = np.abs(X64).max()
    exempt_total = 0
    for m in range(M):
        Lc = A.shape[1]
        par, code, err, A_next, gap = oracle.beam_step(X, C64[m], A, L)
        Ln = par.shape[1]
        rows = to_dev((X64[:, None, :] - A).astype(np.float32))
        rows_n = torch.full((N, Ln, D), float("nan"), dtype=torch.float32, device="cuda:0")
        err_n = torch.full((N, Ln), float("nan"), dtype=torch.float64, device="cuda:0")
        par_g = torch.full((N, Ln), 255, dtype=torch.uint8, device="cuda:0")
        code_g = torch.full((N, Ln), 255, dtype=torch.uint8, device="cuda:0")
        ctx.beam_step(rows, to_dev(err_c) if m else None, to_dev(C32[m]), L, rows_n, err_n, par_g, code_g)
        torch.cuda.synchronize()
        par_g, code_g = par_g.cpu().numpy(), code_g.cpu().numpy()
        err_g, rows_g = err_n.cpu().numpy(), rows_n.cpu().numpy().astype(np.float64)
        assert par_g.max() < Lc and code_g.max() < K
        same = (par_g == par).all(1) & (code_g == code).all(1)
        differ = np.nonzero(~same)[0]
        bad = [int(n) for n in differ if not gap[n] < REL_GAP]
        assert not bad, "stage %d: %d vectors differ outside near-ties, first %s" % (m, len(bad), bad[:5])
        if len(differ):
            e_sel = _cand_err(X64[differ], A[differ], C64[m], par_g[differ].astype(int), code_g[differ].astype(int))
            ref = err[differ]
            assert (np.abs(e_sel - ref) <= REL_GAP * np.maximum(ref, 1e-300) + 1e-12).all()
            # no candidate kept twice
            ids = par_g[differ].astype(int) * K + code_g[differ]
            assert all(len(set(row)) == Ln for row in ids)
        exempt_total += len(differ)
        ok = np.nonzero(same)[0]
        np.testing.assert_allclose(err_g[ok], err[ok], rtol=2e-6, atol=1e-6 * scale * scale)
        want_rows = (X64[:, None, :] - A_next)
        assert np.abs(rows_g[ok] - want_rows[ok]).max() <= 2e-7 * scale * max(m + 1, 1) + 1e-30
        A, err_c = A_next, err
    print("%s L=%d: %d near-tie rows differ over %d stages" % (case, L, exempt_total, M))
    assert exempt_total <= max(3, N * M // 2000)
    ctx.close()


@pytest.mark.parametrize("case,L", [("tiny", 1), ("tiny", 5), ("sift", 1), ("sift", 10), ("k100", 32), ("gist", 10),
                                    ("d132n", 10)])
def test_encode_beam_against_oracle(case, L, oracle):
    c = SHAPES[case]
    X = _data(c)
    N, D, M, K = c["N"], c["D"], c["M"], c["K"]
    C32, C64 = _dictionaries(oracle, X, M, K)
    codes_o, r_o, err_o, gap = oracle.encode_beam(X, C64, L)
    ctx = _ctx(c)
    Xg, Cg = to_dev(X), to_dev(C32)
    codes = torch.full((N, M), 255, dtype=torch.uint8, device="cuda:0")
    res = torch.full((N, D), float("nan"), dtype=torch.float32, device="cuda:0")
    err = torch.full((N,), float("nan"), dtype=torch.float64, device="cuda:0")
    ctx.encode_beam(Xg, Cg, L, codes, res, err)
    torch.cuda.synchronize()
    codes_g, res_g, err_g = codes.cpu().numpy(), res.cpu().numpy().astype(np.float64), err.cpu().numpy()
    differ = np.nonzero((codes_g != codes_o).any(1))[0]
    bad = [int(n) for n in differ if not gap[n] < REL_GAP]
    assert not bad, "%d vectors differ outside near-ties, first %s" % (len(bad), bad[:5])
    print("%s L=%d: %d of %d vectors differ (near-ties)" % (case, L, len(differ), N))
    assert len(differ) <= max(3, N // 500)
    ok = np.ones(N, bool)
    ok[differ] = False
    scale = np.abs(X).max()
    assert np.abs(res_g[ok] - r_o[ok]).max() <= 1e-6 * scale * M
    np.testing.assert_allclose(err_g[ok], err_o[ok], rtol=5e-6, atol=1e-6 * scale * scale)
    # whatever the codes, the residue is x minus their codewords and err its squared norm
    recon = oracle.reconstruct(C64, codes_g)
    assert np.abs(X.astype(np.float64) - recon - res_g).max() <= 1e-6 * scale * M
    np.testing.assert_allclose(err_g, (res_g ** 2).sum(1), rtol=5e-6, atol=1e-6 * scale * scale)
    if L == 1:
        codes1 = torch.empty_like(codes)
        res1 = torch.empty_like(res)
        ctx.encode(Xg, Cg, codes1, res1)
        torch.cuda.synchronize()
        assert torch.equal(codes1, codes) and torch.equal(res1, res)
    ctx.close()


def test_encode_beam_batches_and_degenerate_shapes():
    """More vectors than one batch of the internal buffers holds: equal to the slices encoded alone.
    Also N = 0, N = 1, K = 1 and a beam wider than K."""
    from paper_1509_05194_amd import hclae
    D, M, K, L = 960, 2, 256, 32
    N = 150000 + 3                                   # 2^31 / (32 * 960) = 69905 vectors per batch
    g = torch.Generator(device="cuda:0").manual_seed(5194)
    X = torch.rand((N, D), generator=g, device="cuda:0")
    C = torch.rand((M, K, D), generator=g, device="cuda:0") * torch.tensor([1.0, 0.3], device="cuda:0")[:, None, None]
    ctx = hclae.Context(N, D, M, K)
    codes = torch.empty((N, M), dtype=torch.uint8, device="cuda:0")
    res = torch.empty((N, D), dtype=torch.float32, device="cuda:0")
    ctx.encode_beam(X, C, L, codes, res)
    for lo, hi in ((0, 9000), (69905 - 5, 69905 + 5000), (2 * 69905 - 1, N)):
        n = hi - lo
        c2 = torch.empty((n, M), dtype=torch.uint8, device="cuda:0")
        r2 = torch.empty((n, D), dtype=torch.float32, device="cuda:0")
        ctx.encode_beam(X[lo:hi].contiguous(), C, L, c2, r2)
        torch.cuda.synchronize()
        assert torch.equal(c2, codes[lo:hi]) and torch.equal(r2, res[lo:hi])
    ctx.encode_beam(X[:0].contiguous(), C, L, codes[:0].contiguous(), res[:0].contiguous())
    ctx.close()

    ctx = hclae.Context(16, 8, 3, 1)                  # K = 1: one candidate per path
    X = torch.rand((5, 8), generator=g, device="cuda:0")
    C = torch.rand((3, 1, 8), generator=g, device="cuda:0")
    codes = torch.full((5, 3), 9, dtype=torch.uint8, device="cuda:0")
    res = torch.empty((5, 8), dtype=torch.float32, device="cuda:0")
    ctx.encode_beam(X, C, 4, codes, res)
    torch.cuda.synchronize()
    assert int(codes.max()) == 0
    want = ((X - C[0, 0]) - C[1, 0]) - C[2, 0]
    assert torch.equal(res, want)
    with pytest.raises(hclae.HclaeError):
        ctx.encode_beam(X, C, 33, codes, res)
    with pytest.raises(hclae.HclaeError):
        ctx.encode_beam(X, C, 0, codes, res)
    ctx.close()


def test_sweep_with_multipath_reencode_is_the_composition(oracle):
    """reencode_mode 2 = after every stage, hclae_encode_beam of X under the current dictionaries."""
    from paper_1509_05194_amd import hclae
    c = SHAPES["tiny"]
    X = _data(c)
    N, D, M, K = c["N"], c["D"], c["M"], c["K"]
    C32, _ = _dictionaries(oracle, X, M, K)
    Xg = to_dev(X)
    out = []
    for fused in (True, False):
        ctx = hclae.Context(N, D, M, K)
        ctx.set_beam_width(4)
        C = to_dev(C32)
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        res = torch.empty((N, D), dtype=torch.float32, device="cuda:0")
        ctx.encode(Xg, C, codes, res)
        if fused:
            errs = ctx.sweep(C, codes, res, 2, X=Xg, reencode_mode=2)
        else:
            errs = []
            for m in range(M):
                ctx.anneal_stage(m, C, codes, res, 2, want_stats=False)
                ctx.encode_beam(Xg, C, 4, codes, res)
                errs.append(ctx.quant_error(res))
        torch.cuda.synchronize()
        out.append((C.clone(), codes.clone(), res.clone(), np.asarray(errs)))
        ctx.close()
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1]) and torch.equal(out[0][2], out[1][2])
    np.testing.assert_allclose(out[0][3], out[1][3], rtol=1e-12)


def test_beam_all_candidates_tie(oracle):
    """Every codeword of a dictionary equal: all K * Lc candidates tie exactly, more than the exact
    evaluation lists at once.  Equal errors keep (l, k) order, so the result is fully determined."""
    from paper_1509_05194_amd import hclae
    N, D, K, L = 150, 16, 256, 10
    X = synth.tiny_gmm(N=N, D=D)
    rng = np.random.default_rng(7)
    C32 = np.repeat(rng.normal(size=(2, 1, D)).astype(np.float32) * 0.3, K, axis=1)
    C64 = C32.astype(np.float64)
    X64 = X.astype(np.float64)
    ctx = hclae.Context(N, D, 2, K)
    ctx.set_contraction(_CONTRACTION)
    A = np.zeros((N, 1, D))
    err_c = None
    for m in range(2):
        par, code, err, A_next, gap = oracle.beam_step(X, C64[m], A, L)
        assert (gap == 0).all()
        Ln = par.shape[1]
        rows = to_dev((X64[:, None, :] - A).astype(np.float32))
        rows_n = torch.empty((N, Ln, D), dtype=torch.float32, device="cuda:0")
        par_g = torch.full((N, Ln), 255, dtype=torch.uint8, device="cuda:0")
        code_g = torch.full((N, Ln), 255, dtype=torch.uint8, device="cuda:0")
        ctx.beam_step(rows, to_dev(err_c) if err_c is not None else None, to_dev(C32[m]), L, rows_n, None, par_g, code_g)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(par_g.cpu().numpy(), par)
        np.testing.assert_array_equal(code_g.cpu().numpy(), code)
        assert code[0].tolist() == list(range(L)) and par[0].tolist() == [0] * L
        A, err_c = A_next, err
    ctx.close()
