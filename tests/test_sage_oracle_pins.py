"""Pins of the GraphSAGE-mean oracle (oracle/sage_oracle.py) to facts outside itself: the published first outputs
of SplitMix64, set membership and uniformity of the neighbour samples, a dense-matrix statement of the same
two layers, closed forms, the large-sample limit of the mean aggregator, and finite differences."""
import numpy as np
import pytest

from oracle import sage_oracle as S
from synth import graphs, rng


def _graph(n=60, m=240, seed=3):
    """Random graph + self loops, rows sorted; vertex n-1 is isolated, vertex n-2 has exactly one neighbour."""
    rowptr, col = graphs.erdos_renyi_gnm(n - 2, m, seed)
    rows = [set(col[rowptr[i]:rowptr[i + 1]].tolist()) | {i} for i in range(n - 2)]
    rows.append({n - 2, 5})
    rows[5].add(n - 2)
    rows.append({n - 1})
    rp = np.zeros(n + 1, dtype=np.int64)
    cl = []
    for i, r in enumerate(rows):
        cl += sorted(r)
        rp[i + 1] = len(cl)
    return n, rp, np.array(cl, dtype=np.int32)


def _problem(seed=1, n=60, f=7, hidden=5, classes=4, B=9, S1=6, S2=3):
    n, rp, cl = _graph(n)
    X = rng.normal_f32(seed, 1, n * f).reshape(n, f).astype(np.float64)
    W1 = rng.normal_f32(seed, 2, 2 * f * hidden).reshape(2 * f, hidden).astype(np.float64) * 0.4
    W2 = rng.normal_f32(seed, 3, 2 * hidden * classes).reshape(2 * hidden, classes).astype(np.float64) * 0.4
    labels_all = rng.integers(seed, 4, n, classes).astype(np.int64)
    batch = np.array([0, 7, n - 1, 3, n - 2, 7, 12, 30, 41][:B], dtype=np.int64)      # an isolated one, a repeated one
    return dict(n=n, rp=rp, cl=cl, X=X, W1=W1, W2=W2, labels=labels_all[batch], batch=batch, S1=S1, S2=S2)


def test_generator_matches_the_published_splitmix64_stream():
    # SplitMix64 seeded with 0: the first three outputs, as printed with the reference implementation
    assert S.mix(0) == 0xE220A8397B1DCDAF
    assert S.mix(0x9E3779B97F4A7C15) == 0x6E789E6AA1B965F4
    assert S.mix((2 * 0x9E3779B97F4A7C15) & (2 ** 64 - 1)) == 0x06C45D188009454F
    z = np.array([0, 0x9E3779B97F4A7C15], dtype=np.uint64)
    assert [int(v) for v in S._mix_np(z)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4]


def test_samples_are_neighbours_never_the_vertex_itself():
    n, rp, cl = _graph()
    nodes = np.array(list(range(n)) + [-1, 3, 3], dtype=np.int64)
    out = S.sample_neighbours(rp, cl, nodes, 11, S.level_key(5, 2, 1))
    assert out.shape == (len(nodes), 11) and out.dtype == np.int32
    for m, v in enumerate(nodes):
        if v < 0 or v == n - 1:
            assert (out[m] == -1).all()                       # no vertex / no neighbour
            continue
        nb = set(cl[rp[v]:rp[v + 1]].tolist()) - {int(v)}
        assert set(out[m].tolist()) <= nb
    assert (out[n - 2] == 5).all()                            # a single neighbour is drawn every time
    assert not np.array_equal(out[-1], out[-2])               # the same vertex twice: independent draws
    # a draw depends on (key, instance number, vertex) only
    nodes2 = nodes.copy()
    nodes2[:10] = nodes[10:20]
    out2 = S.sample_neighbours(rp, cl, nodes2, 11, S.level_key(5, 2, 1))
    np.testing.assert_array_equal(out2[20:], out[20:])
    assert not np.array_equal(S.sample_neighbours(rp, cl, nodes, 11, S.level_key(5, 3, 1)), out)   # another step
    assert not np.array_equal(S.sample_neighbours(rp, cl, nodes, 11, S.level_key(5, 2, 2)), out)   # another level


def test_draws_are_uniform_over_the_neighbours():
    d = 7
    rp = np.array([0, d + 1] + [d + 1 + 2 * (i + 1) for i in range(d)], dtype=np.int64)     # a star, centre 0
    cl = np.array(list(range(d + 1)) + sum(([0, i + 1] for i in range(d)), []), dtype=np.int32)
    draws = 70000
    out = S.sample_neighbours(rp, cl, np.array([0]), draws, S.level_key(1, 0, 1))[0]
    counts = np.bincount(out, minlength=d + 1)
    assert counts[0] == 0
    sigma = np.sqrt(draws * (1 / d) * (1 - 1 / d))
    assert np.abs(counts[1:] - draws / d).max() < 4.5 * sigma


def test_two_layers_equal_their_dense_matrix_statement():
    p = _problem()
    t = S.forward(p["rp"], p["cl"], p["X"], p["W1"], p["W2"], p["batch"], p["S1"], p["S2"], seed=9, step=4)
    n, B, S1, S2 = p["n"], len(p["batch"]), p["S1"], p["S2"]
    n1 = B * (1 + S2)
    assert t.nodes1.shape == (n1,) and t.outer.shape == (n1, S1) and t.inner.shape == (B, S2)
    np.testing.assert_array_equal(t.nodes1.reshape(B, 1 + S2)[:, 0], p["batch"])
    sel1 = np.zeros((n1, n))
    cnt1 = np.zeros((n1, n))
    for m in range(n1):
        if t.nodes1[m] >= 0:
            sel1[m, t.nodes1[m]] = 1.0
        for j in range(S1):
            if t.outer[m, j] >= 0:
                cnt1[m, t.outer[m, j]] += 1.0 / S1
    H1 = np.maximum(np.hstack([sel1 @ p["X"], cnt1 @ p["X"]]) @ p["W1"], 0.0)
    self2 = np.kron(np.eye(B), np.eye(1, 1 + S2, 0))                                   # picks instance 0 of each target
    mean2 = np.kron(np.eye(B), np.hstack([[0.0], np.full(S2, 1.0 / S2)])[None, :])      # averages instances 1..S2
    logits = np.hstack([self2 @ H1, mean2 @ H1]) @ p["W2"]
    np.testing.assert_allclose(t.H1, H1, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(t.logits, logits, rtol=1e-12, atol=1e-14)
    # the isolated target: its own features only, its sampled part is zero
    iso = list(p["batch"]).index(n - 1)
    assert (t.inner[iso] == -1).all() and (t.C1[iso * (1 + S2), p["X"].shape[1]:] == 0).all()
    assert (t.H1[iso * (1 + S2) + 1: (iso + 1) * (1 + S2)] == 0).all()


def test_constant_features_give_the_closed_form():
    p = _problem()
    keep = p["batch"] != p["n"] - 1                     # every remaining vertex has a neighbour
    batch = p["batch"][keep]
    c = np.array([0.5, -1.0, 2.0, 0.25, -0.75, 1.5, 3.0])
    X = np.tile(c, (p["n"], 1))
    X[p["n"] - 1] = 0.0                                  # never reached: nobody is its neighbour
    t = S.forward(p["rp"], p["cl"], X, p["W1"], p["W2"], batch, p["S1"], p["S2"], seed=2, step=0)
    h = np.maximum(np.concatenate([c, c]) @ p["W1"], 0.0)
    z = np.concatenate([h, h]) @ p["W2"]
    np.testing.assert_allclose(t.H1, np.tile(h, (len(batch) * (1 + p["S2"]), 1)), rtol=1e-13)
    np.testing.assert_allclose(t.logits, np.tile(z, (len(batch), 1)), rtol=1e-13)


def test_many_samples_approach_the_neighbourhood_mean():
    p = _problem(B=4)
    S1 = 40000
    t = S.forward(p["rp"], p["cl"], p["X"], p["W1"], p["W2"], p["batch"][:2], S1, 1, seed=3, step=1)
    f = p["X"].shape[1]
    for m, v in enumerate(t.nodes1):
        nb = [u for u in p["cl"][p["rp"][v]:p["rp"][v + 1]] if u != v]
        want = p["X"][nb].mean(axis=0)
        spread = p["X"][nb].std(axis=0).max() + 1e-12
        assert np.abs(t.C1[m, f:] - want).max() < 5 * spread / np.sqrt(S1)


def test_loss_and_its_gradient():
    loss, correct, d = S.loss_acc(np.zeros((6, 5)), np.array([0, 1, 2, 3, 4, 0]))
    assert abs(loss - np.log(5.0)) < 1e-15 and correct == 2           # ties go to class 0
    np.testing.assert_allclose(d.sum(axis=1), 0.0, atol=1e-16)
    np.testing.assert_allclose(d[0], (np.full(5, 0.2) - np.eye(5)[0]) / 6, rtol=1e-15)
    big = np.array([[1000.0, 0.0, -1000.0]])
    loss, correct, d = S.loss_acc(big, np.array([1]))
    assert abs(loss - 1000.0) < 1e-9 and correct == 0 and np.isfinite(d).all()


def test_gradients_against_finite_differences():
    p = _problem()
    args = (p["rp"], p["cl"], p["X"])
    kw = dict(S1=p["S1"], S2=p["S2"], seed=11, step=6)

    def loss_of(W1, W2):
        t = S.forward(*args, W1, W2, p["batch"], **kw)
        return S.loss_acc(t.logits, p["labels"])[0]

    t = S.forward(*args, p["W1"], p["W2"], p["batch"], **kw)
    dW1, dW2 = S.backward(t, p["W2"], p["labels"], p["S2"])
    # the gradient through the mean: what reaches the S2 samples adds up to what reached their mean
    hidden = p["W1"].shape[1]
    dC2 = t.dlogits @ p["W2"].T
    pre = t.dZ1.copy()
    assert pre.shape == t.Z1.shape
    eps = 1e-6
    for W, dW, which in ((p["W1"], dW1, 0), (p["W2"], dW2, 1)):
        for idx in [(0, 0), (3, 2), (W.shape[0] - 1, W.shape[1] - 1), (W.shape[0] // 2 + 1, 1)]:
            Wp, Wm = W.copy(), W.copy()
            Wp[idx] += eps
            Wm[idx] -= eps
            num = (loss_of(Wp, p["W2"]) - loss_of(Wm, p["W2"])) if which == 0 else \
                  (loss_of(p["W1"], Wp) - loss_of(p["W1"], Wm))
            num /= 2 * eps
            assert abs(num - dW[idx]) < 1e-7 * max(1.0, abs(num)), (which, idx, num, dW[idx])
    # with every unit switched on (all pre-activations positive) the pieces of dH are exactly the split of dC2
    t.Z1 = np.abs(t.Z1) + 1.0
    S.backward(t, p["W2"], p["labels"], p["S2"])
    B, S2 = len(p["batch"]), p["S2"]
    dH = t.dZ1.reshape(B, 1 + S2, hidden)
    np.testing.assert_allclose(dH[:, 0], dC2[:, :hidden], rtol=1e-13)
    np.testing.assert_allclose(dH[:, 1:].sum(axis=1), dC2[:, hidden:], rtol=1e-12)
