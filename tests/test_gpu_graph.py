"""hclae_sweep without host-side outputs (no init_idx, no err_per_stage) is kernel launches only: no
allocation, no memset, no host synchronisation.  It can therefore be captured in a HIP graph on the
context's stream and replayed; every replay must give the bits of the eager call."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


@pytest.mark.parametrize("contraction", [0, 1], ids=["f32", "splitbf16"])
def test_captured_sweep_replays_like_the_eager_call(contraction):
    from paper_1509_05194_amd import hclae
    N, D, M, K, T = 30000 + 7, 128, 3, 256, 4
    X = synth.sift_like(N, D=D)
    idx = synth.init_indices(N, M, K)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        Xg = torch.from_numpy(X).cuda()
        ctx = hclae.Context(N, D, M, K)                   # takes the current stream: s
        ctx.set_contraction(contraction)
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        r = Xg.clone()
        ctx.sweep(C, codes, r, T, init_idx=idx, want_err=False)   # fresh sweep, eager (it copies init_idx)
        torch.cuda.synchronize()
        state = [(C.clone(), codes.clone(), r.clone())]
        for _ in range(3):                                # the next three sweeps, eager
            ctx.sweep(C, codes, r, T, want_err=False)
            torch.cuda.synchronize()
            state.append((C.clone(), codes.clone(), r.clone()))
        C.copy_(state[0][0]); codes.copy_(state[0][1]); r.copy_(state[0][2])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            ctx.sweep(C, codes, r, T, want_err=False)     # captured, not run
        torch.cuda.synchronize()
        assert torch.equal(C, state[0][0]) and torch.equal(r, state[0][2])
        for i in range(1, 4):
            g.replay()
            torch.cuda.synchronize()
            for got, want, name in zip((C, codes, r), state[i], ("C", "codes", "residue")):
                assert torch.equal(got, want), "replay %d: %s" % (i, name)
            # eager work of the program between replays: a reduction and an encode on the same stream
            E = ctx.quant_error(r)
            assert np.isfinite(E)
        ctx.close()


def test_captured_anneal_call_replays_like_the_eager_call():
    """hclae_anneal without the errors: once the carried-bounds arrays exist (first call), a call is kernel launches
    only; a captured call of six sweeps, replayed from restored states, gives the bits of the eager one."""
    from paper_1509_05194_amd import hclae
    N, D, M, K, T, sweeps = 30000 + 7, 128, 3, 256, 4, 6
    X = synth.sift_like(N, D=D)
    idx = synth.init_indices(N, M, K)
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        Xg = torch.from_numpy(X).cuda()
        ctx = hclae.Context(N, D, M, K)
        C = torch.zeros((M, K, D), dtype=torch.float32, device="cuda:0")
        codes = torch.zeros((N, M), dtype=torch.uint8, device="cuda:0")
        r = Xg.clone()
        ctx.sweep(C, codes, r, T, init_idx=idx, want_err=False)
        torch.cuda.synchronize()
        start = (C.clone(), codes.clone(), r.clone())
        ctx.anneal(C, codes, r, T, sweeps, want_err=False)        # eager; allocates the carried-bounds arrays
        torch.cuda.synchronize()
        want = (C.clone(), codes.clone(), r.clone())
        C.copy_(start[0]); codes.copy_(start[1]); r.copy_(start[2])
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            ctx.anneal(C, codes, r, T, sweeps, want_err=False)
        torch.cuda.synchronize()
        assert torch.equal(C, start[0]) and torch.equal(r, start[2])
        for i in range(3):
            g.replay()
            torch.cuda.synchronize()
            for got, w, name in zip((C, codes, r), want, ("C", "codes", "residue")):
                assert torch.equal(got, w), "replay %d: %s" % (i, name)
            assert np.isfinite(ctx.quant_error(r))
            C.copy_(start[0]); codes.copy_(start[1]); r.copy_(start[2])
            torch.cuda.synchronize()
        ctx.close()
