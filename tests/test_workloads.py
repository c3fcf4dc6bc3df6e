"""The seeded input generators: shapes, ranges, reproducibility and the skew they are meant
to have (Section 2.3 of the paper: a small popular fraction of the embeddings takes most of
the updates)."""
import numpy as np

from paper_2112_07221_amd import workloads as wl


def test_shapes_ranges_and_reproducibility():
    w = wl.WORKLOADS[1]
    a = wl.IdStream(w).batches(5)
    b = wl.IdStream(w).batches(5)
    assert a.shape == (5, 128 * 26) and a.dtype == np.int64 and np.array_equal(a, b)
    per_field = a.reshape(5, 128, 26)
    for f in range(26):
        lo, hi = (f * w.vocab) // 26, ((f + 1) * w.vocab) // 26
        assert per_field[:, :, f].min() >= lo and per_field[:, :, f].max() < hi
    g = wl.grad_pool(w)
    assert g.shape == (8, w.n, 16) and g.dtype == np.float32
    assert abs(float(g.std()) - 1.0) < 0.01
    t = wl.table_init(w)
    assert t.shape == (10_000, 16) and abs(float(t.std()) - 0.01) < 2e-4


def test_flat_and_bag_layouts():
    w4 = wl.WORKLOADS[4].scaled(vocab=4000, batch=64, capacity=400)
    ids = wl.IdStream(w4).batches(3)
    assert ids.shape == (3, 64 * 7) and ids.min() >= 0 and ids.max() < 4000
    w5 = wl.WORKLOADS[5].scaled(vocab=1000, batch=16, capacity=50)
    assert w5.pooled and w5.n_grad_rows == 16
    assert wl.bag_offsets(w5).tolist() == [200 * b for b in range(17)]
    assert wl.grad_pool(w5).shape == (8, 16, 256)


def test_popular_tenth_takes_most_of_the_accesses():
    w = wl.WORKLOADS[2].scaled(vocab=100_000, batch=1024)
    ids = wl.IdStream(w).batches(20).ravel()
    counts = np.sort(np.bincount(ids, minlength=w.vocab))[::-1]
    top = counts[: w.vocab // 10].sum() / counts.sum()
    assert top > 0.75


def test_big_table_init_repeats_a_seeded_block():
    w = wl.WORKLOADS[1].scaled(vocab=2500)
    t = wl.table_init(w, tile_rows=1000)
    assert t.shape == (2500, 16)
    assert np.array_equal(t[:1000], t[1000:2000]) and np.array_equal(t[:500], t[2000:])
