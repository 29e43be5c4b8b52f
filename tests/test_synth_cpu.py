"""The seeded synthetic inputs: the acceptance statistics stated for the stand-ins of the paper's datasets (Sec. 5.1),
the property that any row range can be generated alone, and the independence of the row blocks' random streams."""
import numpy as np

from paper_1509_05194_amd import synth


def test_sift_like_statistics_and_ranges():
    X = synth.sift_like(150_000)
    assert X.dtype == np.float32 and X.min() >= 0 and X.max() <= 255 and np.array_equal(X, np.rint(X))
    assert 0.25 <= float((X == 0).mean()) <= 0.35
    assert 450.0 <= float(np.linalg.norm(X, axis=1).mean()) <= 600.0
    a = synth.sift_like(3000, start=65536 - 1000)
    b = np.concatenate([synth.sift_like(1000, start=65536 - 1000), synth.sift_like(2000, start=65536)])
    assert np.array_equal(a, b)
    assert np.array_equal(synth.sift_like(500, dtype=np.uint8).astype(np.float32), X[:500])


def test_gist_like_statistics_and_ranges():
    X = synth.gist_like(70_000, D=960)
    assert X.min() >= 0 and X.max() <= 1
    assert 1.0 <= float((X.astype(np.float64) ** 2).sum(1).mean()) <= 3.0
    assert float(((X == 0) | (X == 1)).mean()) < 0.4
    assert np.array_equal(synth.gist_like(100, D=960, start=65500)[36:], X[65536:65600])


def test_row_blocks_draw_from_streams_that_do_not_overlap():
    """Two blocks must not be shifted copies of one stream: no run of 16 consecutive noise values of block 0 may
    reappear anywhere in block 1 (with overlapping counters every run did, a few positions further on)."""
    r0, r1 = synth._rng(synth.SEED_DATA, 12, 0), synth._rng(synth.SEED_DATA, 12, 1)
    a, b = r0.random(size=4096), r1.random(size=4096)
    pos = {v: i for i, v in enumerate(b)}
    hits = [i for i, v in enumerate(a) if v in pos]
    assert not hits
    X = synth.sift_like(2 * 65536)
    assert len(np.unique(X[:, :16], axis=0)) > 2 * 65536 * 0.99


def test_init_indices_are_distinct_rows():
    idx = synth.init_indices(100_000, 8, 256)
    assert idx.shape == (8, 256) and idx.min() >= 0 and idx.max() < 100_000
    for m in range(8):
        assert len(set(idx[m].tolist())) == 256
    assert not np.array_equal(idx[0], idx[1])
