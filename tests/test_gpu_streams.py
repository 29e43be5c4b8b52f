"""Two contexts on two HIP streams, their stages enqueued alternately with no synchronisation in between:
each must give the bits of the same work done alone.  Everything a context enqueues goes to its own stream
and its scratch is its own, so neither ordering nor memory is shared."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

JOBS = [dict(gen="sift", N=60000 + 11, D=128, M=3, K=256, T=3),
        dict(gen="gist", N=9000 + 5, D=260, M=3, K=100, T=3)]


def _state(job):
    X = synth.sift_like(job["N"], D=job["D"]) if job["gen"] == "sift" else synth.gist_like(job["N"], D=job["D"])
    Xg = torch.from_numpy(X).cuda()
    C = torch.zeros((job["M"], job["K"], job["D"]), dtype=torch.float32, device="cuda:0")
    codes = torch.zeros((job["N"], job["M"]), dtype=torch.uint8, device="cuda:0")
    return Xg, C, codes, Xg.clone(), synth.init_indices(job["N"], job["M"], job["K"])


def test_two_contexts_on_two_streams_do_not_disturb_each_other():
    from paper_1509_05194_amd import hclae
    alone = []
    for job in JOBS:                                       # each job alone, on the default stream
        Xg, C, codes, r, idx = _state(job)
        ctx = hclae.Context(job["N"], job["D"], job["M"], job["K"])
        for sweep in range(2):
            for m in range(job["M"]):
                ctx.anneal_stage(m, C, codes, r, job["T"], init_idx=idx[m] if sweep == 0 else None, want_stats=False)
        ctx.encode(Xg, C, codes, r)
        torch.cuda.synchronize()
        alone.append((C.clone(), codes.clone(), r.clone()))
        ctx.close()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs, states = [], []
    for job, s in zip(JOBS, streams):
        with torch.cuda.stream(s):
            states.append(_state(job))
            ctxs.append(hclae.Context(job["N"], job["D"], job["M"], job["K"]))   # bound to s
    torch.cuda.synchronize()
    for sweep in range(2):
        for m in range(3):
            for job, s, ctx, (Xg, C, codes, r, idx) in zip(JOBS, streams, ctxs, states):
                with torch.cuda.stream(s):
                    ctx.anneal_stage(m, C, codes, r, job["T"], init_idx=idx[m] if sweep == 0 else None,
                                     want_stats=False)
    for s, ctx, (Xg, C, codes, r, idx) in zip(streams, ctxs, states):
        with torch.cuda.stream(s):
            ctx.encode(Xg, C, codes, r)
    torch.cuda.synchronize()
    for i, ((Xg, C, codes, r, idx), want) in enumerate(zip(states, alone)):
        for got, ref, name in zip((C, codes, r), want, ("C", "codes", "residue")):
            assert torch.equal(got, ref), "job %d: %s" % (i, name)
    for ctx in ctxs:
        ctx.close()
