"""GraphSAGE-mean batch step on the GPU against its CPU oracle (run with -m gpu): the neighbour samples are integer
work and must be bit-exact; features, logits, loss and gradients within 1e-4 in float32."""
import numpy as np
import pytest
import torch

from oracle import sage_oracle as SO
from synth import graphs, rng, workloads
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2012_04930_amd import binding
    binding.lib()
    return binding


def _weights(f, hidden, classes, seed):
    a1 = np.sqrt(6.0 / (2 * f + hidden))
    a2 = np.sqrt(6.0 / (2 * hidden + classes))
    w1 = ((rng.uniform(seed, 1, 2 * f * hidden) * 2 - 1) * a1).astype(np.float32).reshape(2 * f, hidden)
    w2 = ((rng.uniform(seed, 2, 2 * hidden * classes) * 2 - 1) * a2).astype(np.float32).reshape(2 * hidden, classes)
    return w1, w2


def _batch(wl, seed, size):
    train = np.nonzero(wl.mask)[0]
    return train[rng.permutation(seed, 77, len(train))[:size]].astype(np.int32)


class Case:
    def __init__(self, B, oracle, wl, hidden=128, s1=25, s2=10, max_batch=256, seed=3):
        self.B, self.wl, self.hidden, self.s1, self.s2, self.seed = B, wl, hidden, s1, s2, seed
        self.g = H.gpu_graph(B, wl)
        self.og = oracle.canonicalise(wl.n, wl.rowptr, wl.col)
        self.model = B.gcn_sage_create(self.g, hidden, s1, s2, max_batch, seed=seed)
        self.w1, self.w2 = _weights(wl.x.shape[1], hidden, wl.dims[-1], seed)
        B.gcn_sage_set_weights(self.model, self.w1, self.w2)

    def gpu_forward(self, batch, step):
        B, m = self.B, self.model
        B.gcn_sage_forward(m, torch.from_numpy(batch).cuda(), step)
        get = lambda which: B.gcn_sage_get_tensor(m, which).cpu().numpy()
        return dict(inner=get(B.GCN_SAGE_INNER), outer=get(B.GCN_SAGE_OUTER), mean=get(B.GCN_SAGE_C1_MEAN),
                    H1=get(B.GCN_SAGE_H1), logits=get(B.GCN_SAGE_LOGITS))

    def oracle_forward(self, batch, step, w1=None, w2=None):
        return SO.forward(self.og.rowptr, self.og.col, self.wl.x, self.w1 if w1 is None else w1,
                          self.w2 if w2 is None else w2, batch, self.s1, self.s2, self.seed, step)


def _oracle_backward(t, h1_gpu, w2, labels, s2):
    """The oracle's backward pass on its own trace.  The ReLU decision is a yes/no taken by floating point: where the
    GPU's activation disagrees with the oracle's pre-activation, that pre-activation must be ~0 (|Z1| < 1e-5) and
    such entries must be rare; the test then turns the sign of exactly those entries in a copy of the oracle's own
    Z1 (a change below the tolerance) and runs the unchanged oracle on it."""
    flips = (np.asarray(h1_gpu) > 0) != (t.Z1 > 0)
    n_flips = int(flips.sum())
    print("ReLU decisions that differ: %d of %d" % (n_flips, flips.size))
    assert np.abs(t.Z1[flips]).max(initial=0.0) < 1e-5
    assert n_flips <= max(1, int(np.ceil(1e-5 * flips.size)))
    if n_flips:
        z = t.Z1.copy()
        z[flips] = np.where(z[flips] > 0, -1.0, 1.0) * np.maximum(np.abs(z[flips]), np.finfo(np.float64).tiny)
        t.Z1 = z
    return SO.backward(t, w2, labels, s2)


def _compare_forward(case, batch, step):
    got = case.gpu_forward(batch, step)
    t = case.oracle_forward(batch, step)
    np.testing.assert_array_equal(got["inner"], t.inner)
    np.testing.assert_array_equal(got["outer"], t.outer)
    f = case.wl.x.shape[1]
    H.assert_close(got["mean"], t.C1[:, f:], what="mean of the sampled feature rows")
    H.assert_close(got["H1"], t.H1, what="layer 1")
    H.assert_close(got["logits"], t.logits, what="logits")
    return got, t


def test_samples_are_bit_exact_and_both_layers_match(B, oracle):
    wl = workloads.reddit_partition(scale=0.05)               # 2,377 vertices, 602 features, 41 classes
    case = Case(B, oracle, wl)
    batch = _batch(wl, 1, 256)
    got, t = _compare_forward(case, batch, step=0)
    assert got["inner"].min() >= 0                             # every vertex of this graph has neighbours
    loss, acc, correct = B.gcn_sage_loss_acc(case.model)
    ref_loss, ref_correct, _ = SO.loss_acc(t.logits, wl.labels[batch])
    assert abs(loss - ref_loss) <= 1e-4 * abs(ref_loss)
    assert correct == ref_correct and abs(acc - ref_correct / len(batch)) < 1e-6
    # another step draws other samples, the same step the same ones
    again = case.gpu_forward(batch, 0)
    other = case.gpu_forward(batch, 1)
    np.testing.assert_array_equal(again["outer"], got["outer"])
    np.testing.assert_array_equal(again["logits"], got["logits"])
    assert not np.array_equal(other["outer"], got["outer"])


def test_gradients_and_adam_steps_follow_the_oracle(B, oracle):
    wl = workloads.reddit_partition(scale=0.05)
    case = Case(B, oracle, wl)
    lr, b1, b2, eps = (float(np.float32(x)) for x in (1e-4, 0.9, 0.999, 1e-8))     # the ABI carries float32
    ws = [case.w1.astype(np.float64), case.w2.astype(np.float64)]
    state = {}
    gpu_loss, ref_loss = [], []
    for step in range(4):
        batch = _batch(wl, 10 + step, 256 if step < 3 else 100)                    # the last batch is a short one
        got = case.gpu_forward(batch, step)
        gpu_loss.append(B.gcn_sage_loss_acc(case.model)[0])
        B.gcn_sage_backward(case.model)
        dw1 = B.gcn_sage_get_tensor(case.model, B.GCN_SAGE_DW1).cpu().numpy()
        dw2 = B.gcn_sage_get_tensor(case.model, B.GCN_SAGE_DW2).cpu().numpy()
        t = case.oracle_forward(batch, step, ws[0], ws[1])
        ref_dw1, ref_dw2 = _oracle_backward(t, got["H1"], ws[1], wl.labels[batch], case.s2)
        ref_loss.append(t.loss)
        if step == 0:                                                               # same weights on both sides
            H.assert_close(dw1, ref_dw1, what="dW1")
            H.assert_close(dw2, ref_dw2, what="dW2")
        B.gcn_sage_adam_step(case.model, 1e-4)
        ws = oracle.adam(ws, [ref_dw1, ref_dw2], state, lr, b1, b2, eps)
    np.testing.assert_allclose(gpu_loss, ref_loss, rtol=2e-4)
    for which, ref in ((B.GCN_SAGE_W1, ws[0]), (B.GCN_SAGE_W2, ws[1])):
        got_w = B.gcn_sage_get_tensor(case.model, which).cpu().numpy().astype(np.float64)
        rel = np.linalg.norm(got_w - ref) / np.linalg.norm(ref)
        assert rel < 1e-4, (which, rel)


def _odd_graph():
    """200 vertices: a random part, vertex 198 with one neighbour, vertex 199 alone; 13 features, 5 classes."""
    n = 200
    rowptr, col = graphs.erdos_renyi_gnm(198, 900, 5)
    u = np.repeat(np.arange(198), np.diff(rowptr))
    u = np.concatenate([u, [198, 17]])
    v = np.concatenate([col, [17, 198]])
    rp, cl = graphs.pairs_to_csr(n, u[u < v], v[u < v])
    wl = workloads.tiny(n=n)
    wl.rowptr, wl.col = rp, cl
    wl.x = rng.normal_f32(4, 1, n * 13).reshape(n, 13)
    wl.labels = rng.integers(4, 2, n, 5).astype(np.int32)
    wl.mask = np.ones(n, dtype=np.uint8)
    wl.dims = [13, 9, 5]
    return wl


@pytest.mark.parametrize("hidden,s1,s2,bsz", [(9, 3, 2, 7), (100, 1, 1, 1), (16, 25, 10, 64), (33, 7, 30, 20)])
def test_odd_shapes_and_degenerate_vertices(B, oracle, hidden, s1, s2, bsz):
    wl = _odd_graph()
    case = Case(B, oracle, wl, hidden=hidden, s1=s1, s2=s2, max_batch=64, seed=8)
    base = np.array([199, 198, 17, 17, 0, 199, 5] + list(range(20, 20 + 64)), dtype=np.int32)   # alone, one neighbour, repeats
    batch = base[:bsz]
    got, t = _compare_forward(case, batch, step=2)
    iso = np.nonzero(batch == 199)[0]
    assert (got["inner"][iso] == -1).all()
    one = np.nonzero(batch == 198)[0]
    assert (got["inner"][one] == 17).all()
    B.gcn_sage_loss_acc(case.model, sync=False)
    B.gcn_sage_backward(case.model)
    ref_dw1, ref_dw2 = _oracle_backward(t, got["H1"], case.w2.astype(np.float64), wl.labels[batch], s2)
    H.assert_close(B.gcn_sage_get_tensor(case.model, B.GCN_SAGE_DW1).cpu().numpy(), ref_dw1, what="dW1")
    H.assert_close(B.gcn_sage_get_tensor(case.model, B.GCN_SAGE_DW2).cpu().numpy(), ref_dw2, what="dW2")


def test_errors(B, oracle):
    wl = _odd_graph()
    case = Case(B, oracle, wl, hidden=8, s1=2, s2=2, max_batch=4)
    with pytest.raises(B.GcnError):
        B.gcn_sage_backward(case.model)                                                         # nothing to differentiate
    B.gcn_sage_forward(case.model, torch.tensor([0, 200, -3], dtype=torch.int32).cuda(), 0)    # vertices out of range:
    assert (B.gcn_sage_get_tensor(case.model, B.GCN_SAGE_INNER).cpu().numpy()[1:] == -1).all()  # computed as empty ones
    with pytest.raises(B.GcnError) as e:
        B.gcn_sage_loss_acc(case.model)                                                         # ... and reported here
    assert e.value.code == -1
    B.gcn_sage_forward(case.model, torch.tensor([0, 1], dtype=torch.int32).cuda(), 0)
    B.gcn_sage_loss_acc(case.model)                                                             # the flag was cleared
    with pytest.raises(B.GcnError):
        B.gcn_sage_forward(case.model, torch.zeros(5, dtype=torch.int32).cuda(), 0)            # larger than max_batch
    with pytest.raises(B.GcnError):
        B.gcn_sage_create(case.g, 300, 2, 2, 4)                                                 # too many hidden units
    g16 = H.gpu_graph(B, wl, dtype=B.GCN_BF16)
    with pytest.raises(B.GcnError):
        B.gcn_sage_create(g16, 8, 2, 2, 4)                                                      # needs float32 features
    torch.cuda.synchronize()
