"""Parity at the full size of the GIST-shaped configuration (N = 1,000,000, D = 960, K = 256), where the
dictionary does not fit LDS and the D-chunked kernels run, every block walking about fifteen 256-vector
tiles: sampled outputs against the oracle one by one, the rest through properties that hold at any size."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth
from parity_util import judge_codes, to_dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

N, D, K = 1_000_000, 960, 256


@pytest.fixture(scope="module")
def data():
    X = synth.gist_like(N, D=D)
    return X, to_dev(X)


@pytest.mark.parametrize("contraction", [0, 1], ids=["f32", "splitbf16"])
def test_gist_fullsize_assign_sampled(data, oracle, contraction):
    from paper_1509_05194_amd import hclae
    X, Xg = data
    M = 2
    idx = synth.init_indices(N, M, K)
    ctx = hclae.Context(N, D, M, K)
    ctx.set_contraction(contraction)
    C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    C[0] = Xg[torch.from_numpy(idx[0]).cuda()]
    codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    rng = np.random.default_rng(3)
    sample = np.sort(rng.choice(N, 2048, replace=False))
    sample[-1] = N - 1                                     # the ragged tail tile
    sample[0] = 0
    xs64 = X[sample].astype(np.float64)
    dmin = torch.empty(N, dtype=torch.float32, device="cuda:0")
    ctx.assign(0, Xg, C, codes, dmin)
    C64 = C.cpu().numpy().astype(np.float64)
    codes_s = np.zeros((len(sample), M), np.uint8)
    d1, d2, _ = oracle.assign(xs64, C64, codes_s, 0, top2=True)
    got = codes.cpu().numpy()
    ndiff, nex, bad = judge_codes(oracle, xs64, C64, 0, got[sample, 0], codes_s[:, 0], d1, d2)
    print("GIST-shaped full-size assign: %d of %d sampled codes differ (%d exempt), refined %d"
          % (ndiff, len(sample), nex, ctx.last_refined()))
    assert not bad
    same = got[sample, 0] == codes_s[:, 0]
    dm = dmin.cpu().numpy()[sample].astype(np.float64)
    assert np.all(np.abs(dm[same] - d1[same]) <= 2e-7 * d1[same])
    assert np.all(got[:, 1] == 0)
    ctx.close()


def test_gist_fullsize_sweep_properties(data, oracle):
    """Fresh sweep + annealing sweep (M = 8, T = 2, exact shortcuts on): E never rises, x = sum_m C_m[i_m] + r,
    E equals its plain definition, sampled final codes of one more stage are the oracle's nearest codewords
    of the GPU's own x'."""
    from paper_1509_05194_amd import hclae
    X, Xg = data
    M, T = 8, 2
    idx = synth.init_indices(N, M, K)
    ctx = hclae.Context(N, D, M, K)
    C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    r = Xg.clone()
    E1 = ctx.sweep(C, codes, r, T, init_idx=idx)
    E2 = ctx.sweep(C, codes, r, T)
    allE = np.concatenate([E1, E2])
    print("GIST-shaped full-size E per stage:", allE)
    assert np.all(np.diff(allE) <= 1e-7 * allE[:-1])
    recon = r.clone()
    for m in range(M):
        recon += C[m][codes[:, m].long()]
    assert (recon - Xg).abs().max().item() <= 1e-5
    del recon
    E_ref = (r.double() ** 2).sum().item() / N
    assert abs(allE[-1] - E_ref) <= 1e-10 * E_ref

    st = ctx.anneal_stage(3, C, codes, r, T)
    assert st["err_before"] == pytest.approx(E_ref, rel=1e-10) and st["err_after"] <= st["err_before"]
    rng = np.random.default_rng(4)
    sample = np.sort(rng.choice(N, 1024, replace=False))
    sg = torch.from_numpy(sample).cuda()
    xp = (r[sg] + C[3][codes[sg, 3].long()]).cpu().numpy().astype(np.float64)
    C64 = C.cpu().numpy().astype(np.float64)
    codes_s = np.zeros((len(sample), M), np.uint8)
    d1, d2, _ = oracle.assign(xp, C64, codes_s, 3, top2=True)
    got = codes[sg, 3].cpu().numpy()
    ndiff, nex, bad = judge_codes(oracle, xp, C64, 3, got, codes_s[:, 3], d1, d2)
    print("GIST-shaped full-size stage: %d of %d sampled codes differ (%d exempt); stats %s" % (ndiff, len(sample), nex, st))
    assert not bad
    ctx.close()


def test_more_than_2_to_31_elements(data, oracle):
    """N * D = 2.2e9 floats in one array (N = 2,300,003, D = 960): row offsets no longer fit 32 bits.  The
    sweep with the exact shortcuts must equal the single steps bit for bit, and an assignment sampled at the
    head, the middle and the tail of the array must be the oracle's."""
    from paper_1509_05194_amd import hclae
    _, Xg = data
    Xbig = torch.cat([Xg, Xg * 0.97 + 0.001, Xg[:300_003] * 1.04])
    Nb, M, T = Xbig.shape[0], 2, 2
    assert Nb * D > 2 ** 31
    idx = synth.init_indices(Nb, M, K)
    outs = []
    for one_call in (True, False):
        ctx = hclae.Context(Nb, D, M, K)
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((Nb, M), dtype=torch.uint8, device="cuda:0")
        r = Xbig.clone()
        for sweep in range(2):
            if one_call:
                ctx.sweep(C, codes, r, T, init_idx=idx if sweep == 0 else None, want_err=False)
            else:
                for m in range(M):
                    ctx.heat(m, C, codes, r)
                    if sweep == 0:
                        C[m] = r[torch.from_numpy(idx[m]).cuda()]
                    for _ in range(T):
                        ctx.assign(m, r, C, codes)
                        ctx.update(m, r, C, codes)
                    ctx.assign(m, r, C, codes)
                    ctx.cool(m, C, codes, r)
        torch.cuda.synchronize()
        outs.append((C.clone(), codes.clone(), r.clone()))
        if one_call:
            ctx.heat(M - 1, C, codes, r)
            cg = codes.clone()
            ctx.assign(M - 1, r, C, cg)
            sel = np.concatenate([np.arange(0, 1000), np.arange(Nb // 2, Nb // 2 + 1000), np.arange(Nb - 1000, Nb)])
            sel_g = torch.from_numpy(sel).cuda()
            xs64 = r[sel_g].cpu().numpy().astype(np.float64)
            C64 = C.cpu().numpy().astype(np.float64)
            codes_s = np.zeros((len(sel), M), np.uint8)
            d1, d2, _ = oracle.assign(xs64, C64, codes_s, M - 1, top2=True)
            got = cg[sel_g, M - 1].cpu().numpy()
            ndiff, nex, bad = judge_codes(oracle, xs64, C64, M - 1, got, codes_s[:, M - 1], d1, d2)
            assert not bad
        ctx.close()
        del C, codes, r
    assert torch.equal(outs[0][0], outs[1][0]), "dictionaries differ"
    assert torch.equal(outs[0][1], outs[1][1]), "codes differ"
    assert torch.equal(outs[0][2], outs[1][2]), "residues differ"
