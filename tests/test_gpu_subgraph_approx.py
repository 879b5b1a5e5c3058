"""GPU subgraph approximation (Algorithm 1 + edge dropping) vs its CPU oracle: bit-exact (run with -m gpu)."""
import time

import numpy as np
import pytest
import torch

from oracle import subgraph_approx as SA
from synth import graphs, rng, workloads
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2012_04930_amd import binding
    binding.lib()
    return binding


def _gpu_augment(B, rowptr, col, part, n_parts, p, overlap, seed):
    v, n_local, rp, cl = B.gcn_augment_partition(torch.from_numpy(np.ascontiguousarray(rowptr, dtype=np.int64)).cuda(),
                                                 torch.from_numpy(np.ascontiguousarray(col, dtype=np.int32)).cuda(),
                                                 torch.from_numpy(np.ascontiguousarray(part, dtype=np.int32)).cuda(),
                                                 n_parts, p, overlap, seed)
    return v.cpu().numpy(), n_local, rp.cpu().numpy(), cl.cpu().numpy()


def _check_against_oracle(B, n, rowptr, col, part, n_parts, p, overlap, seed):
    want_v, want_nl, levels = SA.augmented_partition(n, rowptr, col, part, n_parts, p, overlap, seed)
    want_rp, want_cl = SA.induced_subgraph(n, rowptr, col, want_v)
    v, nl, rp, cl = _gpu_augment(B, rowptr, col, part, n_parts, p, overlap, seed)
    assert nl == want_nl
    np.testing.assert_array_equal(v, want_v)
    np.testing.assert_array_equal(rp, want_rp)
    np.testing.assert_array_equal(cl, want_cl)
    return levels


@pytest.mark.parametrize("n,n_parts,overlap,seed", [(200, 3, 0.3, 1), (500, 5, 0.1, 2), (300, 2, 0.9, 3),
                                                    (400, 4, 2.5, 4), (64, 1, 0.5, 5), (300, 6, 0.0, 6)])
def test_small_random_graphs_every_partition(B, n, n_parts, overlap, seed):
    m = 3 * n
    rowptr, col = graphs.erdos_renyi_gnm(n, m, seed)
    part = rng.integers(seed, 50, n, n_parts).astype(np.int32)
    for p in range(n_parts):
        _check_against_oracle(B, n, rowptr, col, part, n_parts, p, overlap, seed)


def test_sparse_graph_needs_several_levels(B):
    # a long cycle cut into 4 arcs: each level adds two vertices per neighbouring arc, so nts = 10 needs 5+ levels
    n = 400
    rowptr, col = graphs.pairs_to_csr(n, np.arange(n), (np.arange(n) + 1) % n)
    part = (np.arange(n) // 100).astype(np.int32)
    levels = _check_against_oracle(B, n, rowptr, col, part, 4, 1, 0.3, seed=9)
    assert len(levels[0]) >= 5 and len(levels[2]) >= 5 and levels[3] == []      # arc 3 does not touch arc 1


def test_community_graph_with_partitions_of_communities(B):
    wl = workloads.chung_lu_mid(scale=0.06)                  # 6,000 vertices, 20 communities of consecutive ids
    part = (np.arange(wl.n) // (wl.n // 5)).clip(max=4).astype(np.int32)
    for overlap in (0.1, 0.5):
        for p in (0, 3):
            _check_against_oracle(B, wl.n, wl.rowptr, wl.col, part, 5, p, overlap, seed=11)


def test_full_size_graph_five_partitions(B, capsys):
    """The Reddit-shaped graph (46,600 vertices, 23.6 M stored entries) cut into 5 partitions of 10 communities;
    partition 2 extended with the paper's 10 % overlap (2 % overhead).  Bit-exact against the array oracle."""
    wl = workloads.reddit_partition(extra_frac=0.0)
    n_parts, p, overlap, seed = 5, 2, 0.10, 1
    part = (np.arange(wl.n) // (wl.n // n_parts)).clip(max=n_parts - 1).astype(np.int32)
    d = H.to_dev(wl)
    part_dev = torch.from_numpy(part).cuda()
    B.gcn_augment_partition(d["rowptr"], d["col"], part_dev, n_parts, p, overlap, seed)      # warm-up
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    v, n_local, rp, cl = B.gcn_augment_partition(d["rowptr"], d["col"], part_dev, n_parts, p, overlap, seed)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    want_v, want_nl = SA.augmented_partition_np(wl.n, wl.rowptr, wl.col, part, n_parts, p, overlap, seed)
    want_rp, want_cl = SA.induced_subgraph_np(wl.n, wl.rowptr, wl.col, want_v)
    assert n_local == want_nl == 9320 and len(want_v) - want_nl == 4 * 233          # nts = floor(0.1 * 9320 / 4)
    np.testing.assert_array_equal(v.cpu().numpy(), want_v)
    np.testing.assert_array_equal(rp.cpu().numpy(), want_rp)
    np.testing.assert_array_equal(cl.cpu().numpy(), want_cl)
    with capsys.disabled():
        print("\n    gcn_augment_partition: %d vertices / %d entries -> %d + %d vertices, %d entries in %.1f ms"
              % (wl.n, wl.nnz, n_local, len(want_v) - n_local, len(want_cl), dt * 1e3), end="", flush=True)


def test_bad_arguments(B):
    n = 100
    rowptr, col = graphs.erdos_renyi_gnm(n, 200, 1)
    part = np.zeros(n, dtype=np.int32)
    part[7] = 3
    with pytest.raises(B.GcnError) as e:
        _gpu_augment(B, rowptr, col, part, 3, 0, 0.1, 0)         # partition id 3 with n_parts = 3
    assert e.value.code == -1
    bad = col.copy()
    bad[0] = n
    with pytest.raises(B.GcnError) as e:
        _gpu_augment(B, rowptr, bad, np.zeros(n, dtype=np.int32), 1, 0, 0.1, 0)
    assert e.value.code == -2
    torch.cuda.synchronize()


def test_pipeline_augment_then_train(B, oracle):
    """Whole method on one worker: partition a community graph, extend partition 2 by Algorithm 1 with a 10 %
    overlap, drop the other cut edges, then one training epoch on the result; the oracle does the same on the
    CPU, from the same full graph."""
    wl = workloads.chung_lu_mid(scale=0.06)
    n_parts, p, overlap, seed = 5, 2, 0.10, 3
    part = (np.arange(wl.n) // (wl.n // n_parts)).clip(max=n_parts - 1).astype(np.int32)
    d = H.to_dev(wl)
    v, n_local, rp, cl = B.gcn_augment_partition(d["rowptr"], d["col"], torch.from_numpy(part).cuda(), n_parts, p,
                                                 overlap, seed)
    x = B.gcn_gather_rows(d["x"], v)
    labels = B.gcn_gather_rows(d["labels"], v)
    mask = torch.zeros(v.numel(), dtype=torch.uint8, device="cuda")
    mask[:n_local] = torch.from_numpy(wl.mask[part == p]).cuda()         # sampled vertices stay outside the loss
    g = B.gcn_graph_create(rp, cl, x, labels, mask, wl.dims[-1])
    # the oracle's version of the same worker input
    ov, onl, _ = SA.augmented_partition(wl.n, wl.rowptr, wl.col, part, n_parts, p, overlap, seed)
    orp, ocl = SA.induced_subgraph(wl.n, wl.rowptr, wl.col, ov)
    assert onl == n_local and len(ov) == v.numel() and len(ov) - onl == 4 * int(np.floor(overlap * onl / 4))
    sub = workloads.Workload("partition %d with overlap" % p, len(ov), onl, orp, ocl, wl.x[ov], wl.labels[ov],
                             np.concatenate([wl.mask[part == p], np.zeros(len(ov) - onl, dtype=np.uint8)]), wl.dims,
                             wl.weights)
    np.testing.assert_array_equal(x.cpu().numpy(), sub.x)
    np.testing.assert_array_equal(labels.cpu().numpy(), sub.labels)
    _, gpu = H.gpu_epoch(B, g, sub)
    _, tr, new = H.oracle_epoch(oracle, sub, gpu=gpu)
    H.compare_epoch(oracle, sub, gpu, tr, new)


def test_workers_train_then_average_parameters(B, oracle):
    """Section 3.2 on one GPU: three workers, each with its own augmented partition and its own copy of the
    network, train one epoch from the same weights; the parameter server step replaces every copy by the mean."""
    wl = workloads.chung_lu_mid(scale=0.045)
    n_parts, overlap, seed = 3, 0.2, 5
    part = (np.arange(wl.n) // (wl.n // n_parts)).clip(max=n_parts - 1).astype(np.int32)
    d = H.to_dev(wl)
    part_dev = torch.from_numpy(part).cuda()
    models, graphs_, ref_new = [], [], []
    for p in range(n_parts):
        v, n_local, rp, cl = B.gcn_augment_partition(d["rowptr"], d["col"], part_dev, n_parts, p, overlap, seed)
        mask = torch.zeros(v.numel(), dtype=torch.uint8, device="cuda")
        mask[:n_local] = torch.from_numpy(wl.mask[part == p]).cuda()
        g = B.gcn_graph_create(rp, cl, B.gcn_gather_rows(d["x"], v), B.gcn_gather_rows(d["labels"], v), mask,
                               wl.dims[-1])
        m = B.gcn_model_create(g, wl.dims)
        B.gcn_set_weights(m, wl.weights)
        B.gcn_forward(m, True)
        B.gcn_loss_acc(m, sync=False)
        B.gcn_backward(m)
        B.gcn_sgd_step(m, wl.lr)
        models.append(m)
        graphs_.append(g)
        ov, onl, _ = SA.augmented_partition(wl.n, wl.rowptr, wl.col, part, n_parts, p, overlap, seed)
        orp, ocl = SA.induced_subgraph(wl.n, wl.rowptr, wl.col, ov)
        og = oracle.canonicalise(len(ov), orp, ocl)
        omask = np.concatenate([wl.mask[part == p], np.zeros(len(ov) - onl, dtype=np.uint8)])
        new, _ = oracle.train_epoch(og, wl.x[ov], [w.astype(np.float64) for w in wl.weights], wl.labels[ov], omask,
                                    wl.lr)
        ref_new.append(new)
    B.gcn_average_weights(models)
    for l in (1, 2):
        want = np.mean([rn[l - 1] for rn in ref_new], axis=0)
        got = [B.gcn_get_tensor(m, B.GCN_T_W, l).cpu().numpy() for m in models]
        for gw in got:
            H.assert_close(gw, want, what="averaged W%d" % l)
            np.testing.assert_array_equal(gw, got[0])            # every worker holds the same bits afterwards
    # training continues from the aggregate
    B.gcn_forward(models[0], True)
    assert np.isfinite(B.gcn_loss_acc(models[0])[0])


def test_training_scheme_on_streams_follows_the_oracle_for_several_epochs(B, oracle):
    """Section 3.2 as a whole: three workers on three streams, every epoch one full-batch step each on its own
    extended partition (Algorithm 1, overlap 20 %), then the parameter average.  The oracle runs the same scheme on
    the CPU; the averaged weights are compared after every epoch, and so are the workers' losses."""
    from paper_2012_04930_amd import partition_training as PT
    wl = workloads.planted_classes(n=1800, n_comm=6, avg_degree=12.0, f=24, hidden=16)
    n_parts, overlap, seed, epochs = 3, 0.2, 7, 4
    part = (np.arange(wl.n) // (wl.n // n_parts)).clip(max=n_parts - 1).astype(np.int32)
    d = H.to_dev(wl)
    workers = PT.Workers(d["rowptr"], d["col"], d["x"], d["labels"], d["mask"], torch.from_numpy(part).cuda(), n_parts,
                         overlap, wl.dims, wl.weights, seed=seed, sampled_vertices_train=True)
    # the oracle's workers
    subs = []
    for p in range(n_parts):
        ov, onl, _ = SA.augmented_partition(wl.n, wl.rowptr, wl.col, part, n_parts, p, overlap, seed)
        orp, ocl = SA.induced_subgraph(wl.n, wl.rowptr, wl.col, ov)
        subs.append((oracle.canonicalise(len(ov), orp, ocl), wl.x[ov], wl.labels[ov], wl.mask[ov]))
        assert workers.sizes[p][0] == len(ov) and workers.sizes[p][1] == onl
    ws = [w.astype(np.float64) for w in wl.weights]
    lr = 0.5
    for e in range(epochs):
        stats = workers.epoch(lr, "sgd")
        new, ref_loss = [], []
        for og, x, y, msk in subs:
            w_p, tr = oracle.train_epoch(og, x, ws, y, msk, lr)
            new.append(w_p)
            ref_loss.append(tr.loss)
        ws = [np.mean([w_p[l] for w_p in new], axis=0) for l in range(len(ws))]
        np.testing.assert_allclose([s[0] for s in stats], ref_loss, rtol=2e-4)
        for l, got in enumerate(workers.weights()):
            H.assert_close(got.cpu().numpy(), ws[l], rtol=2e-4, what="averaged W%d after epoch %d" % (l + 1, e + 1))
    # it learns: the averaged model classifies the held-out vertices of the whole graph far better than chance (1/6)
    ev = PT.Evaluator(d["rowptr"], d["col"], d["x"], d["labels"],
                      torch.from_numpy(wl.extra["heldout"]).cuda(), wl.dims)
    for _ in range(40):
        workers.epoch(lr, "sgd", read_back=False)
    assert ev(workers.weights())[1] > 0.5
