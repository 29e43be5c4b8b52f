"""hclae_quant_error_noalloc (the entry point for callers that cannot allocate: static device scratch, no ctx)
against hclae_quant_error, through the C ABI, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

from paper_1509_05194_amd import synth

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def test_no_alloc_quant_error_matches_the_ctx_entry_point():
    from paper_1509_05194_amd import hclae
    out = torch.full((1,), -1.0, dtype=torch.float64, device="cuda:0")
    # second call smaller than the first (fewer blocks: stale partials of the first call lie beyond its range),
    # then one smaller than a single block, then an empty one
    for N, D in ((300_000 + 3, 128), (1000 + 1, 128), (7, 16), (0, 128)):
        X = synth.sift_like(max(N, 1), D=D)[:N]
        r = torch.from_numpy(np.ascontiguousarray(X)).to("cuda:0") - 100.0
        before = torch.cuda.memory_allocated()
        hclae.quant_error_noalloc(r, out)
        assert torch.cuda.memory_allocated() == before
        got = float(out.cpu()[0])
        ctx = hclae.Context(max(N, 1), D, 1, 1)
        want = ctx.quant_error(r)
        ctx.close()
        ref = float((r.double() ** 2).sum().item() / N) if N else 0.0
        print("N=%d D=%d: no-alloc %.17g, ctx %.17g, plain definition %.17g" % (N, D, got, want, ref))
        assert got == want                                  # same grid, same order of additions: the same bits
        assert abs(got - ref) <= 1e-12 * max(ref, 1e-300)
    # arguments beyond the limits are refused before anything is launched
    L = hclae.lib()
    r = torch.zeros((4, 8), dtype=torch.float32, device="cuda:0")
    assert L.hclae_quant_error_noalloc(r.data_ptr(), 2 ** 31, 8, out.data_ptr(), None) == hclae.EINVAL
    assert b"limits" in L.hclae_last_error(None)
    assert L.hclae_quant_error_noalloc(r.data_ptr(), 4, 6, out.data_ptr(), None) == hclae.EINVAL
    assert L.hclae_quant_error_noalloc(r.data_ptr(), 4, 8192, out.data_ptr(), None) == hclae.EINVAL
    assert L.hclae_quant_error_noalloc(None, 4, 8, out.data_ptr(), None) == hclae.EINVAL
    assert L.hclae_quant_error_noalloc(r.data_ptr(), 4, 8, None, None) == hclae.EINVAL
    assert L.hclae_quant_error_noalloc(r.data_ptr() + 4, 1, 8, out.data_ptr(), None) == hclae.EINVAL
