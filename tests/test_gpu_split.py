"""The split-bf16 distance contraction (hclae_set_contraction 1) against the fp32 one: since both only
pre-select candidates for the fp64 direct-form re-check, every output must be bit-identical; only the
number of vectors that take the re-check may differ."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth
from parity_util import judge_codes, to_dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _run_sweeps(X, M, K, T, mode, sweeps=2):
    from paper_1509_05194_amd import hclae
    N, D = X.shape
    Xg = to_dev(X)
    ctx = hclae.Context(N, D, M, K)
    ctx.set_contraction(mode)
    C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
    r = Xg.clone()
    errs = []
    refined = 0
    for s in range(sweeps):
        for m in range(M):
            st = ctx.anneal_stage(m, C, codes, r, T, init_idx=synth.init_indices(N, M, K)[m] if s == 0 else None)
            errs.append(st["err_after"])
            refined += st["refined"]
    q = torch.empty((N, M), dtype=torch.uint8, device="cuda:0")
    qr = torch.empty_like(Xg)
    ctx.encode(Xg, C, q, qr)
    torch.cuda.synchronize()
    out = (C.clone(), codes.clone(), r.clone(), q.clone(), qr.clone(), np.asarray(errs), refined)
    ctx.close()
    return out


@pytest.mark.parametrize("gen,N,D,M,K", [("tiny", 10000 + 3, 16, 4, 16), ("sift", 30000 + 7, 128, 3, 256),
                                         ("sift", 5000 + 1, 20, 2, 100), ("gist", 3000 + 5, 64, 2, 256),
                                         # D-chunked shapes: 8, 4, 2 and 1 codeword blocks, a ragged last slice
                                         ("gist", 6000 + 5, 960, 2, 256), ("gist", 3000 + 1, 516, 2, 100),
                                         ("gist", 2000 + 3, 1412, 2, 40), ("gist", 1500 + 7, 2052, 2, 16)])
def test_split_contraction_gives_identical_results(gen, N, D, M, K):
    X = {"tiny": lambda: synth.tiny_gmm(N=N, D=D), "sift": lambda: synth.sift_like(N, D=D),
         "gist": lambda: synth.gist_like(N, D=D)}[gen]()
    a = _run_sweeps(X, M, K, 3, 0)
    b = _run_sweeps(X, M, K, 3, 1)
    for i, name in enumerate(["C", "codes", "residue", "encode codes", "encode residue"]):
        assert torch.equal(a[i], b[i]), name
    np.testing.assert_array_equal(a[5], b[5])
    print("%s N=%d D=%d K=%d: final-assign re-checks fp32 %d, split-bf16 %d" % (gen, N, D, K, a[6], b[6]))


def test_split_contraction_fullsize_sampled(oracle):
    """N = 1,000,000 in the launch configuration of `bench.py --contraction split`: sampled codes against
    the oracle one by one, all codes against the fp32 kernel."""
    from paper_1509_05194_amd import hclae
    N, D, K, M = 1_000_000, 128, 256, 2
    X = synth.sift_like(N, D=D)
    Xg = to_dev(X)
    idx = synth.init_indices(N, M, K)
    C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
    C[0] = Xg[torch.from_numpy(idx[0]).cuda()]
    codes = {}
    refined = {}
    for mode in (0, 1):
        ctx = hclae.Context(N, D, M, K)
        ctx.set_contraction(mode)
        c = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        ctx.assign(0, Xg, C, c)
        # a non-integer x' (residue-like): one centroid update, then the residue of stage 0 against codeword means
        codes[mode] = c
        refined[mode] = ctx.last_refined()
        ctx.close()
    assert torch.equal(codes[0], codes[1])
    print("full-size assign: re-checks fp32 %d, split-bf16 %d of %d" % (refined[0], refined[1], N))
    rng = np.random.default_rng(2)
    sample = np.sort(rng.choice(N, 4096, replace=False))
    sample[-1] = N - 1
    xs64 = X[sample].astype(np.float64)
    C64 = C.cpu().numpy().astype(np.float64)
    codes_s = np.zeros((len(sample), M), np.uint8)
    d1, d2, _ = oracle.assign(xs64, C64, codes_s, 0, top2=True)
    got = codes[1].cpu().numpy()
    ndiff, nex, bad = judge_codes(oracle, xs64, C64, 0, got[sample, 0], codes_s[:, 0], d1, d2)
    assert not bad

    # second case: real-valued residues (x minus its codeword) against a dictionary of real-valued means
    ctx = hclae.Context(N, D, M, K)
    ctx.update(0, Xg, C, codes[0])
    r = Xg.clone()
    ctx.cool(0, C, codes[0], r)
    C[1] = r[torch.from_numpy(idx[1]).cuda()]
    ctx.close()
    out = {}
    for mode in (0, 1):
        ctx = hclae.Context(N, D, M, K)
        ctx.set_contraction(mode)
        c = codes[0].clone()
        ctx.assign(1, r, C, c)
        out[mode] = (c, ctx.last_refined())
        ctx.close()
    assert torch.equal(out[0][0], out[1][0])
    print("full-size assign on residues: re-checks fp32 %d, split-bf16 %d of %d" % (out[0][1], out[1][1], N))
    rs64 = r.cpu().numpy()[sample].astype(np.float64)
    C64 = C.cpu().numpy().astype(np.float64)
    d1, d2, _ = oracle.assign(rs64, C64, codes_s, 1, top2=True)
    got = out[1][0].cpu().numpy()
    ndiff, nex, bad = judge_codes(oracle, rs64, C64, 1, got[sample, 1], codes_s[:, 1], d1, d2)
    assert not bad
