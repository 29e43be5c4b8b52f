"""Online chunked learning (Sec. 3.4 of arXiv 1509.05194, read as running per-codeword sums and
counts) against the oracle at reduced scale, and the double-buffered host-to-device pipeline."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth
from parity_util import fresh_state, rel_fro, to_dev

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

D, M, K = 128, 4, 256
CH, NCH = 20000 + 13, 4


def _chunks():
    return [synth.sift_like(CH, D=D, start=i * CH, dtype=np.uint8) for i in range(NCH)]


def _start_dictionaries(oracle, chunk0):
    C, codes, r = fresh_state(chunk0.astype(np.float32), M, K)
    oracle.sweep(C, codes, r, 1, synth.init_indices(CH, M, K))
    return C.astype(np.float32)


@pytest.mark.parametrize("weighted", [False, True])
def test_online_chunks_match_oracle(oracle, weighted):
    """Step-locked per chunk: the oracle starts every chunk from the GPU's exported state
    (dictionaries, running sums, counts) and replays the chunk stage by stage with the pinned
    primitives, judging the GPU's first-assignment and final codes under the near-tie rule and
    adopting exempt ones, so that one legitimate near-tie cannot snowball."""
    from paper_1509_05194_amd import hclae
    from parity_util import judge_codes
    chunks = _chunks()
    C0 = _start_dictionaries(oracle, chunks[0])
    n0 = np.random.default_rng(3).integers(0, 5000, size=(M, K)).astype(np.int64) if weighted else None
    ctx = hclae.Context(CH, D, M, K)
    Cg = to_dev(C0)
    ctx.online_begin(Cg, n0)
    S0, cnt0 = ctx.online_export()
    np.testing.assert_array_equal(cnt0, n0 if weighted else np.zeros((M, K), np.int64))
    np.testing.assert_allclose(S0, C0.astype(np.float64) * cnt0[:, :, None], rtol=1e-15)
    codes_g = torch.zeros((CH, M), dtype=torch.uint8, device="cuda:0")
    first_g = torch.zeros((CH, M), dtype=torch.uint8, device="cuda:0")
    rg = torch.empty((CH, D), dtype=torch.float32, device="cuda:0")
    adopted = 0
    # the chunk's sums are taken on integers q = round(x' * 2^s), max |q| in [2^29, 2^30): each vector adds at
    # most half a step = max |x'| * 2^-30 of error to an element of its cluster's running sum
    tol = np.zeros((M, K, 1))
    for i, ch in enumerate(chunks):
        Co = Cg.cpu().numpy().astype(np.float64)
        S, cnt = ctx.online_export()
        E_g = ctx.online_chunk(to_dev(ch), Cg, codes_g, rg, want_err=True, codes_first=first_g)
        got, first = codes_g.cpu().numpy(), first_g.cpu().numpy()
        Cgpu = Cg.cpu().numpy()
        r = ch.astype(np.float64)
        codes_o = np.zeros((CH, M), np.uint8)
        for m in range(M):
            d1, d2, _ = oracle.assign(r, Co, codes_o, m, top2=True)
            nd, nex, bad = judge_codes(oracle, r, Co, m, first[:, m], codes_o[:, m], d1, d2)
            assert not bad, "chunk %d stage %d first assign: %s" % (i, m, bad[:5])
            adopted += nex
            codes_o[:, m] = first[:, m]
            tol[m, :, 0] += np.bincount(codes_o[:, m], minlength=K) * np.abs(r).max() * 2.0 ** -30
            np.add.at(S[m], codes_o[:, m], r)
            cnt[m] += np.bincount(codes_o[:, m], minlength=K)
            has = cnt[m] > 0
            Co[m][has] = S[m][has] / cnt[m][has][:, None]
            assert rel_fro(Cgpu[m], Co[m]) <= 1e-6
            Co[m] = Cgpu[m].astype(np.float64)                     # both sides re-assign against the fp32 dictionary
            d1, d2, _ = oracle.assign(r, Co, codes_o, m, top2=True)
            nd, nex, bad = judge_codes(oracle, r, Co, m, got[:, m], codes_o[:, m], d1, d2)
            assert not bad, "chunk %d stage %d re-assign: %s" % (i, m, bad[:5])
            adopted += nex
            codes_o[:, m] = got[:, m]
            oracle.cool(r, codes_o, Co, m)
            r = r.astype(np.float32).astype(np.float64)            # the GPU residue is stored in fp32 between stages
        res = rg.cpu().numpy().astype(np.float64)
        assert rel_fro(res, r) <= 1e-6
        assert abs(E_g - oracle.quant_error(res)) <= 1e-12 * E_g
        S_g, cnt_g = ctx.online_export()
        np.testing.assert_array_equal(cnt_g, cnt)
        assert np.all(np.abs(S_g - S) <= tol + 1e-13 * np.abs(S)) and rel_fro(S_g, S) <= 1e-8
    print("online (weighted=%s): adopted %d near-ties over %d assigns of %d vectors" % (weighted, adopted, 2 * M * NCH, CH))
    # resume: a second context fed the exported state continues identically
    S_g, cnt_g = ctx.online_export()
    ctx2 = hclae.Context(CH, D, M, K)
    C2 = Cg.clone()
    ctx2.online_begin(C2, None)
    ctx2.online_import(S_g, cnt_g)
    nxt = to_dev(synth.sift_like(CH, D=D, start=NCH * CH, dtype=np.uint8))
    ctx.online_chunk(nxt, Cg, codes_g, rg)
    codes2, r2 = torch.zeros_like(codes_g), torch.empty_like(rg)
    ctx2.online_chunk(nxt, C2, codes2, r2)
    assert torch.equal(C2, Cg) and torch.equal(codes2, codes_g) and torch.equal(r2, rg)
    ctx.close()
    ctx2.close()


def test_online_chunks_any_row_length(oracle, monkeypatch):
    """The same step-locked comparison on a shape whose rows are no multiple of 16 bytes (D = 36), with a
    padded codeword block (K = 17) and a chunk byte count that leaves a tail of 12 bytes."""
    import sys
    mod = sys.modules[__name__]
    for name, value in dict(D=36, M=3, K=17, CH=3000 + 7, NCH=3).items():
        monkeypatch.setattr(mod, name, value)
    assert (CH * D) % 16 == 12
    test_online_chunks_match_oracle(oracle, True)


def test_pipelined_host_chunks_give_identical_results():
    """uint8 chunks in pinned host memory, copied by hipMemcpyAsync on a side stream into two
    device staging buffers while the previous chunk is processed; same bits as the serial run."""
    from paper_1509_05194_amd import hclae
    chunks = _chunks()
    C0 = synth.sift_like(M * K, D=D, seed=77).reshape(M, K, D) * (0.5 ** np.arange(M))[:, None, None].astype(np.float32)
    C0 = np.ascontiguousarray(C0, np.float32)

    def run(pipelined):
        ctx = hclae.Context(CH, D, M, K)
        Cg = to_dev(C0)
        ctx.online_begin(Cg, None)
        codes = [torch.zeros((CH, M), dtype=torch.uint8, device="cuda:0") for _ in chunks]
        rg = torch.empty((CH, D), dtype=torch.float32, device="cuda:0")
        if not pipelined:
            for ch, cd in zip(chunks, codes):
                ctx.online_chunk(to_dev(ch), Cg, cd, rg)
        else:
            host = [torch.from_numpy(ch).pin_memory() for ch in chunks]
            stage = [torch.empty((CH, D), dtype=torch.uint8, device="cuda:0") for _ in range(2)]
            side = torch.cuda.Stream()                     # default priority
            main = torch.cuda.current_stream()
            copied = [torch.cuda.Event() for _ in chunks]
            freed = [torch.cuda.Event() for _ in chunks]
            for i in range(len(chunks)):
                with torch.cuda.stream(side):
                    if i >= 2:
                        side.wait_event(freed[i - 2])      # staging buffer no longer read
                    stage[i % 2].copy_(host[i], non_blocking=True)
                    copied[i].record(side)
                main.wait_event(copied[i])
                ctx.online_chunk(stage[i % 2], Cg, codes[i], rg)
                freed[i].record(main)
        torch.cuda.synchronize()
        out = (Cg.clone(), [c.clone() for c in codes])
        ctx.close()
        return out

    Ca, codes_a = run(False)
    Cb, codes_b = run(True)
    assert torch.equal(Ca, Cb)
    for a, b in zip(codes_a, codes_b):
        assert torch.equal(a, b)


def test_online_chunks_free_running_against_oracle_online_chunk(oracle):
    """Free-running: hclae_online_chunk and the oracle's own online_chunk each process the same chunks from the
    same start, nothing exchanged in between.  The case has no near-tie that the two sides decide differently
    (the codes must be EQUAL), so dictionaries, running sums, residues and E must agree to the fp32 bars."""
    from paper_1509_05194_amd import hclae
    n, nch = 6000 + 5, 3
    chunks = [synth.sift_like(n, D=D, start=7_000_000 + i * n, dtype=np.uint8) for i in range(nch)]
    C0 = _start_dictionaries(oracle, np.ascontiguousarray(synth.sift_like(CH, D=D, dtype=np.uint8)))
    n0 = np.full((M, K), 40, np.int64)
    ctx = hclae.Context(n, D, M, K)
    Cg = to_dev(C0)
    ctx.online_begin(Cg, n0)
    Co = C0.astype(np.float64)
    S = Co * n0[:, :, None]
    cnt = n0.copy()
    codes_g = torch.zeros((n, M), dtype=torch.uint8, device="cuda:0")
    rg = torch.empty((n, D), dtype=torch.float32, device="cuda:0")
    for i, ch in enumerate(chunks):
        E_g = ctx.online_chunk(to_dev(ch), Cg, codes_g, rg, want_err=True)
        codes_o, r_o, E_o = oracle.online_chunk(ch, Co, S, cnt)
        ndiff = int((codes_g.cpu().numpy() != codes_o).sum())
        print("free-running online chunk %d: %d codes differ, E gpu %.6f oracle %.6f, C err %.2e"
              % (i, ndiff, E_g, E_o, rel_fro(Cg.cpu().numpy(), Co)))
        assert ndiff == 0
        assert abs(E_g - E_o) <= 1e-4 * E_o
        assert rel_fro(rg.cpu().numpy(), r_o) <= 1e-4
        for m in range(M):
            assert rel_fro(Cg[m].cpu().numpy(), Co[m]) <= 1e-4
    S_g, cnt_g = ctx.online_export()
    np.testing.assert_array_equal(cnt_g, cnt)
    assert rel_fro(S_g, S) <= 1e-6
    ctx.close()
