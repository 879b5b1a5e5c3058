"""Shape checks of the seeded input generators (no GCN arithmetic involved)."""
import numpy as np

from synth import graphs, rng, workloads


def _is_symmetric(n, rowptr, col):
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rowptr))
    a = set(zip(rows.tolist(), col.tolist()))
    return all((j, i) in a for (i, j) in a)


def test_rng_is_reproducible_and_counter_based():
    a = rng.bits(3, 5, 1000)
    b = rng.bits(3, 5, 400, offset=600)
    np.testing.assert_array_equal(a[600:], b)
    assert np.any(a != rng.bits(4, 5, 1000)) and np.any(a != rng.bits(3, 6, 1000))
    z = rng.normal_f32(1, 1, 200001)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    assert sorted(rng.permutation(2, 2, 100).tolist()) == list(range(100))


def test_tiny_workload_shape():
    w = workloads.tiny()
    assert w.n == 2048 and w.nnz == 2 * 4096 and w.x.shape == (2048, 256) and w.dims == [256, 16, 7]
    assert _is_symmetric(w.n, w.rowptr, w.col)
    w2 = workloads.tiny()
    np.testing.assert_array_equal(w.col, w2.col)
    np.testing.assert_array_equal(w.x, w2.x)
    a = np.sqrt(6.0 / (256 + 16))
    assert np.abs(w.weights[0]).max() <= a and w.weights[0].shape == (256, 16)


def test_messy_copy_keeps_the_adjacency():
    w = workloads.tiny(n=300)
    rp, cl = graphs.messy_copy(w.n, w.rowptr, w.col, 5)
    assert rp[-1] > w.rowptr[-1]
    for i in range(w.n):
        a = set(w.col[w.rowptr[i]:w.rowptr[i + 1]].tolist())
        b = set(cl[rp[i]:rp[i + 1]].tolist()) - {i}
        assert a == b


def test_partition_workload_structure():
    w = workloads.reddit_partition(scale=0.05)
    n_extra = w.extra["n_extra"]
    assert w.n == w.n_local + n_extra and n_extra == round(0.02 * w.n_local)
    assert _is_symmetric(w.n, w.rowptr, w.col)
    deg = np.diff(w.rowptr)
    # extra vertices: only local neighbours, outside the train mask, smoother features
    for i in range(w.n_local, w.n):
        assert np.all(w.col[w.rowptr[i]:w.rowptr[i + 1]] < w.n_local)
    assert w.mask[w.n_local:].sum() == 0 and 0.6 < w.mask[:w.n_local].mean() < 0.72
    assert w.x[w.n_local:].std() < 0.5 < w.x[:w.n_local].std()
    assert deg[w.n_local:].mean() > deg[:w.n_local].mean()
    assert w.labels.max() < 41 and w.labels.min() >= 0


def test_chung_lu_has_heavy_tail_and_communities():
    w = workloads.chung_lu_mid(scale=0.05)
    deg = np.diff(w.rowptr)
    assert 18 < deg.mean() <= 20.2 and deg.max() > 5 * deg.mean()
    rows = np.repeat(np.arange(w.n), deg)
    block = -(-w.n // 20)
    assert np.mean(rows // block == w.col // block) > 0.75


def test_rmat_shape():
    w = workloads.rmat_large(scale=0.002)
    deg = np.diff(w.rowptr)
    assert w.nnz == 50 * w.n and deg.max() > 10 * deg.mean()
    assert _is_symmetric(w.n, w.rowptr, w.col)
