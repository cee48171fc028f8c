"""Sanity checks of the synthetic workload generators (inputs only)."""
import numpy as np

from paper_2003_03477_amd import synth


def test_batches_are_seeded_and_shaped():
    wl = synth.tiny()
    g = synth.BatchGenerator(wl)
    a, b = g.batch(3), synth.BatchGenerator(wl).batch(3)
    for u, v in zip(a.as_tuple(), b.as_tuple()):
        assert np.array_equal(u, v)
    B, T = wl.batch, wl.num_tables
    assert a.dense.shape == (B, 13) and a.labels.shape == (B,)
    assert a.offsets.shape == (T * B + 1,) and a.offsets[0] == 0
    assert a.offsets[-1] == len(a.indices)
    assert np.all(np.diff(a.offsets) >= 1)
    assert a.indices.min() >= 0 and a.indices.max() < 1000
    assert not np.array_equal(a.indices[:50], g.batch(4).indices[:50])


def test_bag_length_and_zipf_slope():
    wl = synth.mid().scaled(batch=512, rows=(100_000,) * 2)
    g = synth.BatchGenerator(wl)
    b = g.batch(0)
    lens = np.diff(b.offsets)
    assert abs(lens.mean() - 21.0) < 0.5
    # rank-frequency slope of the sampler itself
    rng = np.random.default_rng(0)
    ranks = g.zipf[0].ranks(rng.random(400_000))
    counts = np.bincount(ranks, minlength=64)[:64].astype(float)
    k = np.arange(1, 65)
    slope = np.polyfit(np.log(k), np.log(counts), 1)[0]
    assert abs(slope + 1.05) < 0.08
    # the rank -> row map is a bijection
    z = g.zipf[0]
    assert len(np.unique(z.rows_of_ranks(np.arange(z.n)))) == z.n


def test_label_rate_and_h0_hash():
    wl = synth.mid().scaled(batch=4096, rows=(10_000,) * 8)
    y = synth.BatchGenerator(wl).batch(0).labels
    assert 0.1 < y.mean() < 0.4
    h = synth.table_rows_h0(7, 2, np.arange(5000), 16)
    assert h.dtype == np.float32 and np.all(np.abs(h) <= 0.05)
    assert abs(h.mean()) < 1e-3 and abs(h.std() - 0.05 / np.sqrt(3)) < 1e-3
    # rows are addressable independently
    assert np.array_equal(synth.table_rows_h0(7, 2, np.array([4321]), 16)[0], h[4321])
    assert not np.array_equal(synth.table_rows_h0(7, 3, np.array([4321]), 16)[0], h[4321])


def test_compaction_preserves_sort_order_and_values():
    wl = synth.tiny()
    g = synth.BatchGenerator(wl)
    batches = [g.batch(s) for s in range(3)]
    cp = synth.compact_problem(wl, batches)
    full = synth.full_tables_h0(wl)
    B = wl.batch
    base_c = np.concatenate(([0], np.cumsum(cp.rows)))
    for ob, cb in zip(batches, cp.batches):
        for t in range(wl.num_tables):
            lo, hi = ob.offsets[t * B], ob.offsets[(t + 1) * B]
            assert np.array_equal(cp.touched[t][cb.indices[lo:hi]], ob.indices[lo:hi])
            assert np.array_equal(np.argsort(ob.indices[lo:hi], kind="stable"),
                                  np.argsort(cb.indices[lo:hi], kind="stable"))
            assert np.array_equal(cp.h0[base_c[t] + cb.indices[lo:hi]],
                                  full[wl.row_base[t] + ob.indices[lo:hi]])


def test_large_row_counts():
    rows = synth.large().rows
    assert len(rows) == 26 and min(rows) >= 1000 and max(rows) <= 40_000_000
    assert 1.5e8 < sum(rows) < 2.5e8
