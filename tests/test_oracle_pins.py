"""Pins for the CPU oracle: each part is checked against something that is not the oracle —
hand-worked values, closed forms, invariants of the normalised adjacency, a dense-matrix
evaluation with numpy, brute force on tiny graphs and finite differences.  CPU only."""
import os

import numpy as np
import pytest

from synth import graphs, rng, workloads

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _load(name):
    return np.loadtxt(os.path.join(GOLD, name), comments="#")


def _csr_from_dense(a):
    n = a.shape[0]
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols = []
    for i in range(n):
        js = np.nonzero(a[i])[0]
        cols.extend(js.tolist())
        rowptr[i + 1] = len(cols)
    return rowptr, np.array(cols, dtype=np.int32)


def _dense_ahat(a):
    """D^-1/2 (A + I) D^-1/2 written with dense numpy, independent of the oracle's loops."""
    n = a.shape[0]
    b = ((a + a.T) > 0).astype(np.float64)
    np.fill_diagonal(b, 1.0)
    d = b.sum(1)
    return b / np.sqrt(np.outer(d, d)), b, d


def _random_sym(n, p, seed):
    u = rng.uniform(seed, 1, n * n).reshape(n, n)
    a = np.triu(u < p, 1)
    return (a | a.T).astype(np.float64)


def _oracle_dense_ahat(oracle, g):
    n = g.n
    return oracle.aggregate(g, np.eye(n))


# ------------------------------------------------------------------ canonical pattern, degrees
@pytest.mark.parametrize("n,p,seed", [(5, 0.5, 1), (17, 0.3, 2), (64, 0.1, 3), (40, 0.9, 4)])
def test_canonical_pattern_matches_dense_brute_force(oracle, n, p, seed):
    a = _random_sym(n, p, seed)
    rowptr, col = _csr_from_dense(a)
    rp, cl = graphs.messy_copy(n, rowptr, col, seed)       # duplicates, loops, scrambled order
    g = oracle.canonicalise(n, rp, cl)
    _, b, d = _dense_ahat(a)
    for i in range(n):
        row = g.col[g.rowptr[i]:g.rowptr[i + 1]]
        assert row.tolist() == np.nonzero(b[i])[0].tolist()
    assert g.deg.tolist() == d.astype(int).tolist()
    assert int(g.rowptr[-1]) == int(b.sum())
    assert np.all(g.deg == 1 + a.sum(1).astype(int))


def test_self_loop_counts_once_and_isolated_vertex(oracle):
    # vertex 0: loop stored three times and neighbour 1 twice; vertex 2 isolated
    rowptr = np.array([0, 5, 6, 6], dtype=np.int64)
    col = np.array([0, 1, 0, 1, 0, 0], dtype=np.int32)
    g = oracle.canonicalise(3, rowptr, col)
    assert g.col.tolist() == [0, 1, 0, 1, 2]
    assert g.deg.tolist() == [2, 2, 1]
    ah = _oracle_dense_ahat(oracle, g)
    assert ah[2, 2] == 1.0 and abs(ah[0, 0] - 0.5) < 1e-15


def test_rejects_bad_input(oracle):
    with pytest.raises(oracle.OracleError):
        oracle.canonicalise(2, np.array([0, 1, 2]), np.array([1, 5], dtype=np.int32))      # column out of range
    with pytest.raises(oracle.OracleError):
        oracle.canonicalise(2, np.array([0, 2, 1]), np.array([1, 0], dtype=np.int32))      # rowptr not monotone
    with pytest.raises(oracle.OracleError):
        oracle.canonicalise(3, np.array([0, 1, 1, 1]), np.array([1], dtype=np.int32))      # (0,1) without (1,0)


# ------------------------------------------------------------------ A_hat
def test_path3_hand_worked(oracle):
    want = _load("path3_ahat.txt")
    g = oracle.canonicalise(3, np.array([0, 1, 3, 4]), np.array([1, 0, 2, 1], dtype=np.int32))
    np.testing.assert_allclose(_oracle_dense_ahat(oracle, g), want, rtol=0, atol=1e-14)


def test_star4_hand_worked(oracle):
    want = _load("star4_forward.txt")
    g = oracle.canonicalise(4, np.array([0, 3, 4, 5, 6]), np.array([1, 2, 3, 0, 0, 0], dtype=np.int32))
    got = oracle.aggregate(g, np.array([[8.0], [2.0], [4.0], [6.0]]))[:, 0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("n,p,seed", [(24, 0.2, 5), (64, 0.08, 6)])
def test_ahat_invariants(oracle, n, p, seed):
    a = _random_sym(n, p, seed)
    g = oracle.canonicalise(n, *_csr_from_dense(a))
    ah = _oracle_dense_ahat(oracle, g)
    want, _, d = _dense_ahat(a)
    np.testing.assert_allclose(ah, want, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(ah, ah.T)                                  # symmetric
    np.testing.assert_allclose(np.diag(ah), 1.0 / d, rtol=1e-15)             # A_hat_ii = 1/d_i
    np.testing.assert_allclose(ah @ np.sqrt(d), np.sqrt(d), rtol=1e-12)      # sqrt(d) is a fixed vector
    ev = np.linalg.eigvalsh(ah)
    assert ev.max() <= 1.0 + 1e-12 and ev.min() > -1.0                       # spectrum in (-1, 1]


def test_regular_graph_rows_sum_to_one(oracle):
    n, k = 30, 4                          # circulant: i ~ i+-1, i+-2
    a = np.zeros((n, n))
    for i in range(n):
        for s in (1, 2):
            a[i, (i + s) % n] = a[i, (i - s) % n] = 1
    g = oracle.canonicalise(n, *_csr_from_dense(a))
    assert np.all(g.deg == k + 1)
    np.testing.assert_allclose(oracle.aggregate(g, np.ones((n, 3))), 1.0, rtol=1e-14)


def test_complete_graph_gives_column_mean(oracle):
    n = 12
    a = np.ones((n, n)) - np.eye(n)
    g = oracle.canonicalise(n, *_csr_from_dense(a))
    x = rng.normal_f32(7, 1, n * 5).reshape(n, 5).astype(np.float64)
    z = oracle.aggregate(g, x)
    np.testing.assert_allclose(z, np.tile(x.mean(0), (n, 1)), rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ dense products
def test_matmuls_match_numpy(oracle):
    a = rng.normal_f32(1, 1, 37 * 19).reshape(37, 19).astype(np.float64)
    b = rng.normal_f32(1, 2, 19 * 11).reshape(19, 11).astype(np.float64)
    c = rng.normal_f32(1, 3, 37 * 11).reshape(37, 11).astype(np.float64)
    np.testing.assert_allclose(oracle.matmul_nn(a, b), a @ b, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.matmul_tn(a, c), a.T @ c, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(oracle.matmul_nt(c, b), c @ b.T, rtol=1e-13, atol=1e-13)


# ------------------------------------------------------------------ forward
def _tiny_problem(n=32, dims=(8, 5, 3), p=0.15, seed=11, mask_p=0.6):
    a = _random_sym(n, p, seed)
    rowptr, col = _csr_from_dense(a)
    x = rng.normal_f32(seed, 10, n * dims[0]).reshape(n, dims[0]).astype(np.float64)
    ws = [w.astype(np.float64) for w in workloads.glorot_weights(list(dims), seed)]
    labels = rng.integers(seed, 11, n, dims[-1]).astype(np.int32)
    mask = (rng.uniform(seed, 12, n) < mask_p).astype(np.uint8)
    mask[0] = 1
    return a, rowptr, col, x, ws, labels, mask


def _dense_forward(a, x, ws):
    ah, _, _ = _dense_ahat(a)
    h = x
    zs = []
    for l, w in enumerate(ws):
        z = ah @ (h @ w)
        zs.append(z)
        h = np.maximum(z, 0.0) if l < len(ws) - 1 else z
    return zs


@pytest.mark.parametrize("dims", [(8, 5, 3), (6, 7, 4, 3)])
def test_forward_equals_dense_matrix_gcn(oracle, dims):
    a, rowptr, col, x, ws, labels, mask = _tiny_problem(dims=dims)
    g = oracle.canonicalise(a.shape[0], rowptr, col)
    tr = oracle.forward(g, x, ws)
    for z, want in zip(tr.Z, _dense_forward(a, x, ws)):
        np.testing.assert_allclose(z, want, rtol=1e-12, atol=1e-13)
    assert np.all(tr.H[1] >= 0)


def test_empty_graph_is_an_mlp(oracle):
    n, dims = 20, (6, 4, 3)
    _, _, _, x, ws, labels, mask = _tiny_problem(n=n, dims=dims)
    g = oracle.canonicalise(n, np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32))
    tr = oracle.forward(g, x, ws)
    np.testing.assert_allclose(tr.Z[-1], np.maximum(x @ ws[0], 0) @ ws[1], rtol=1e-13, atol=1e-14)


def test_permutation_equivariance(oracle):
    a, rowptr, col, x, ws, labels, mask = _tiny_problem(n=40)
    n = a.shape[0]
    g = oracle.canonicalise(n, rowptr, col)
    tr = oracle.backward(g, oracle.forward(g, x, ws), ws, labels, mask)
    perm = rng.permutation(3, 1, n)                     # vertex i becomes perm[i]
    rp2, col2 = graphs.relabel(n, rowptr, col, perm)
    inv = np.empty(n, dtype=np.int64)
    inv[perm] = np.arange(n)
    g2 = oracle.canonicalise(n, rp2, col2)
    tr2 = oracle.backward(g2, oracle.forward(g2, x[inv], ws), ws, labels[inv], mask[inv])
    np.testing.assert_allclose(tr2.Z[-1][perm], tr.Z[-1], rtol=1e-12, atol=1e-13)
    assert abs(tr2.loss - tr.loss) < 1e-13 and tr2.correct == tr.correct
    for d1, d2 in zip(tr.dW, tr2.dW):
        np.testing.assert_allclose(d2, d1, rtol=1e-11, atol=1e-14)


# ------------------------------------------------------------------ loss, accuracy
def test_zero_last_layer_gives_log_c(oracle):
    table = _load("log_classes.txt")
    for c, want in table:
        c = int(c)
        n = 50
        labels = rng.integers(c, 1, n, c).astype(np.int32)
        mask = (rng.uniform(c, 2, n) < 0.5).astype(np.uint8)
        mask[3] = 1
        loss, correct, nt, dz = oracle.loss_acc(np.zeros((n, c)), labels, mask)
        assert abs(loss - want) < 1e-14
        assert nt == int(mask.sum())
        assert correct == int(np.sum((labels == 0) & (mask == 1)))        # ties go to class 0
        onehot = np.eye(c)[labels]
        np.testing.assert_allclose(dz, mask[:, None] * (1.0 / c - onehot) / nt, rtol=1e-13, atol=1e-16)


def test_loss_properties(oracle):
    n, c = 64, 9
    z = rng.normal_f32(5, 1, n * c).reshape(n, c).astype(np.float64) * 3
    labels = rng.integers(5, 2, n, c).astype(np.int32)
    mask = (rng.uniform(5, 3, n) < 0.7).astype(np.uint8)
    loss, correct, nt, dz = oracle.loss_acc(z, labels, mask)
    # textbook softmax cross-entropy with numpy
    zs = z - z.max(1, keepdims=True)
    logp = zs - np.log(np.exp(zs).sum(1, keepdims=True))
    m = mask.astype(bool)
    assert abs(loss - (-logp[m, labels[m]].mean())) < 1e-13
    assert correct == int(np.sum(z.argmax(1)[m] == labels[m]))
    np.testing.assert_allclose(dz.sum(1), 0.0, atol=1e-16)                 # every row of dZ_L sums to zero
    assert np.all(dz[~m] == 0.0)                                           # rows outside the mask are zero
    shift = rng.normal_f32(5, 4, n).astype(np.float64)[:, None] * 10
    loss2, correct2, _, dz2 = oracle.loss_acc(z + shift, labels, mask)
    assert abs(loss2 - loss) < 1e-12 and correct2 == correct              # constant per row changes nothing
    np.testing.assert_allclose(dz2, dz, rtol=1e-10, atol=1e-15)
    with pytest.raises(oracle.OracleError):
        oracle.loss_acc(z, labels, np.zeros(n, dtype=np.uint8))            # empty train mask
    bad = labels.copy()
    bad[0] = c
    with pytest.raises(oracle.OracleError):
        oracle.loss_acc(z, bad, mask)


# ------------------------------------------------------------------ backward
@pytest.mark.parametrize("dims", [(8, 5, 3), (5, 6, 4, 3)])
def test_gradients_by_central_differences(oracle, dims):
    a, rowptr, col, x, ws, labels, mask = _tiny_problem(dims=dims)
    g = oracle.canonicalise(a.shape[0], rowptr, col)
    tr = oracle.backward(g, oracle.forward(g, x, ws), ws, labels, mask)

    def loss_of(wlist):
        return oracle.loss_acc(oracle.forward(g, x, wlist).Z[-1], labels, mask, want_grad=False)[0]

    eps = 1e-5
    for l in range(len(ws)):
        num = np.zeros_like(ws[l])
        for idx in np.ndindex(*ws[l].shape):
            wp = [w.copy() for w in ws]
            wm = [w.copy() for w in ws]
            wp[l][idx] += eps
            wm[l][idx] -= eps
            num[idx] = (loss_of(wp) - loss_of(wm)) / (2 * eps)
        err = np.abs(num - tr.dW[l]).max() / max(np.abs(num).max(), 1e-12)
        assert err < 1e-6, (l, err)


def test_gradients_equal_hand_derived_mlp_when_graph_is_empty(oracle):
    n, dims = 25, (6, 4, 3)
    _, _, _, x, ws, labels, mask = _tiny_problem(n=n, dims=dims)
    g = oracle.canonicalise(n, np.zeros(n + 1, dtype=np.int64), np.zeros(0, dtype=np.int32))
    tr = oracle.backward(g, oracle.forward(g, x, ws), ws, labels, mask)
    z1 = x @ ws[0]
    h1 = np.maximum(z1, 0)
    z2 = h1 @ ws[1]
    e = np.exp(z2 - z2.max(1, keepdims=True))
    sm = e / e.sum(1, keepdims=True)
    nt = mask.sum()
    dz2 = mask[:, None] * (sm - np.eye(dims[-1])[labels]) / nt
    np.testing.assert_allclose(tr.dW[1], h1.T @ dz2, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(tr.dW[0], x.T @ ((dz2 @ ws[1].T) * (z1 > 0)), rtol=1e-12, atol=1e-15)


def test_backward_equals_dense_chain_rule(oracle):
    a, rowptr, col, x, ws, labels, mask = _tiny_problem(n=48, dims=(7, 6, 4))
    g = oracle.canonicalise(a.shape[0], rowptr, col)
    tr = oracle.backward(g, oracle.forward(g, x, ws), ws, labels, mask)
    ah, _, _ = _dense_ahat(a)
    z1 = ah @ (x @ ws[0])
    h1 = np.maximum(z1, 0)
    z2 = ah @ (h1 @ ws[1])
    e = np.exp(z2 - z2.max(1, keepdims=True))
    dz2 = mask[:, None] * (e / e.sum(1, keepdims=True) - np.eye(4)[labels]) / mask.sum()
    g2 = ah.T @ dz2
    np.testing.assert_allclose(tr.G[1], g2, rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(tr.dW[1], h1.T @ g2, rtol=1e-12, atol=1e-16)
    dz1 = (g2 @ ws[1].T) * (z1 > 0)
    np.testing.assert_allclose(tr.dZ[0], dz1, rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(tr.dW[0], x.T @ (ah.T @ dz1), rtol=1e-12, atol=1e-16)


# ------------------------------------------------------------------ update, dropout
def test_sgd_closed_form_and_descent(oracle):
    wl = workloads.tiny(seed=0, n=256)
    g = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
    ws = [w.astype(np.float64) for w in wl.weights]
    new, tr = oracle.train_epoch(g, wl.x, ws, wl.labels, wl.mask, lr=0.02)
    for w, d, w2 in zip(ws, tr.dW, new):
        np.testing.assert_array_equal(w2, w - 0.02 * d)
    loss_after = oracle.loss_acc(oracle.forward(g, wl.x, new).Z[-1], wl.labels, wl.mask, want_grad=False)[0]
    assert loss_after < tr.loss


def test_dropout_mask(oracle):
    rows, width, p = 400, 64, 0.3
    keep = oracle.dropout_keep(9, 2, 1, rows, width, p)
    frac = keep.mean()
    sigma = np.sqrt(p * (1 - p) / keep.size)
    assert abs(frac - (1 - p)) < 5 * sigma
    np.testing.assert_array_equal(keep, oracle.dropout_keep(9, 2, 1, rows, width, p))
    assert np.any(keep != oracle.dropout_keep(9, 3, 1, rows, width, p))      # another epoch, another mask
    assert np.any(keep != oracle.dropout_keep(9, 2, 2, rows, width, p))
    assert oracle.dropout_keep(9, 2, 1, 10, 10, 0.0).all()
    # the mask is the stated integer function: recompute three entries by hand in Python integers
    M = (1 << 64) - 1

    def sm(z):
        z = (z + 0x9E3779B97F4A7C15) & M
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
        return z ^ (z >> 31)

    key = sm(sm(9) ^ ((2 * 0xD1B54A32D192ED03) & M) ^ ((1 * 0x8CB92BA72F3D8DD7) & M))
    thr = int(np.floor(p * 2 ** 32))
    for e in (0, 77, rows * width - 1):
        want = (sm((key + e * 0x9E3779B97F4A7C15) & M) >> 32) >= thr
        assert bool(keep.reshape(-1)[e]) == want
    # forward with dropout: H = relu(Z) * keep / (1 - p), and the backward uses the same mask
    a, rowptr, col, x, ws, labels, mask = _tiny_problem(n=40, dims=(8, 16, 3))
    g = oracle.canonicalise(40, rowptr, col)
    tr = oracle.forward(g, x, ws, p=0.5, training=True, seed=4, epoch=1)
    k = oracle.dropout_keep(4, 1, 1, 40, 16, 0.5)
    np.testing.assert_allclose(tr.H[1], np.maximum(tr.Z[0], 0) * k / 0.5, rtol=1e-15)
    oracle.backward(g, tr, ws, labels, mask, p=0.5)
    assert np.all(tr.dZ[0][k == 0] == 0)
    tr_eval = oracle.forward(g, x, ws, p=0.5, training=False)
    np.testing.assert_allclose(tr_eval.H[1], np.maximum(tr_eval.Z[0], 0), rtol=0)


@pytest.mark.parametrize("dims,p", [((8, 16, 3), 0.5), ((6, 7, 5, 3), 0.25)])
def test_gradients_with_dropout_by_central_differences(oracle, dims, p):
    """With the keep mask held fixed (same seed and epoch) the loss is a smooth function of the weights, and its
    central differences must equal the backward pass: a missing or misplaced 1 / (1 - p) in the backward pass
    (or a mask applied on one side only) changes dW of every layer below the last by that factor."""
    a, rowptr, col, x, ws, labels, mask = _tiny_problem(n=40, dims=dims)
    g = oracle.canonicalise(40, rowptr, col)
    kw = dict(p=p, training=True, seed=11, epoch=3)
    tr = oracle.backward(g, oracle.forward(g, x, ws, **kw), ws, labels, mask, p=p)
    assert any((k == 0).any() for k in tr.keep) and any((k != 0).any() for k in tr.keep)

    def loss_of(wlist):
        return oracle.loss_acc(oracle.forward(g, x, wlist, **kw).Z[-1], labels, mask, want_grad=False)[0]

    eps = 1e-5
    for l in range(len(ws)):
        num = np.zeros_like(ws[l])
        for idx in np.ndindex(*ws[l].shape):
            wp = [w.copy() for w in ws]
            wm = [w.copy() for w in ws]
            wp[l][idx] += eps
            wm[l][idx] -= eps
            num[idx] = (loss_of(wp) - loss_of(wm)) / (2 * eps)
        err = np.abs(num - tr.dW[l]).max() / max(np.abs(num).max(), 1e-12)
        assert err < 1e-6, (l, err)
    # and the closed form of the step itself: dZ = dH * [Z > 0] * keep / (1 - p)
    nl = len(ws)
    for l in range(nl - 1, 0, -1):
        dH = tr.G[l] @ ws[l].T
        np.testing.assert_allclose(tr.dZ[l - 1], dH * (tr.Z[l - 1] > 0) * tr.keep[l - 1] / (1.0 - p), rtol=1e-13, atol=0)


# ------------------------------------------------------------------ Adam (the paper's optimiser, Section 4.1)
def test_adam_closed_forms(oracle):
    g = rng.normal_f32(3, 1, 60).reshape(12, 5).astype(np.float64)
    w0 = rng.normal_f32(3, 2, 60).reshape(12, 5).astype(np.float64)
    lr, eps = 0.02, 1e-8
    # first step: bias correction makes m_hat = g and v_hat = g^2, so the move is lr * g / (|g| + eps)
    st = {}
    w1 = oracle.adam([w0], [g], st, lr)[0]
    np.testing.assert_allclose(w0 - w1, lr * g / (np.abs(g) + eps), rtol=1e-12)
    # a constant gradient keeps m_hat = g and v_hat = g^2 at every step: same move each time
    w = w1
    for _ in range(5):
        w_next = oracle.adam([w], [g], st, lr)[0]
        np.testing.assert_allclose(w - w_next, lr * g / (np.abs(g) + eps), rtol=1e-10)
        w = w_next
    assert st["t"] == 6
    # zero gradient from the start: nothing moves (0 / (0 + eps))
    st0 = {}
    np.testing.assert_array_equal(oracle.adam([w0], [np.zeros_like(g)], st0, lr)[0], w0)
    # textbook recurrences with numpy over a varying gradient sequence
    st2, w, m, v = {}, w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    b1, b2 = 0.9, 0.999
    for t in range(1, 8):
        gt = rng.normal_f32(9, t, 60).reshape(12, 5).astype(np.float64) * (0.1 * t)
        m = b1 * m + (1 - b1) * gt
        v = b2 * v + (1 - b2) * gt * gt
        w = w - lr * (m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps)
        got = oracle.adam([w0 if t == 1 else got], [gt], st2, lr)[0]
        np.testing.assert_allclose(got, w, rtol=1e-12, atol=1e-15)
