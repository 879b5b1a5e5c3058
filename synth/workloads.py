"""The five benchmark workloads as seeded synthetic inputs.

Each function returns a Workload: a raw symmetric CSR adjacency, the feature matrix,
labels, the train mask, the layer widths and host-generated initial weights.  The
same arrays go to the CPU oracle and to the GPU library.  Sizes can be scaled down
(`scale` < 1) for quick tests; scale = 1 gives the stated shape.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import graphs, rng


@dataclass
class Workload:
    name: str
    n: int                      # vertices, local + extra
    n_local: int
    rowptr: np.ndarray          # int64 [n+1]  raw A
    col: np.ndarray             # int32 [nnz]
    x: np.ndarray               # float32 [n, f]
    labels: np.ndarray          # int32 [n]
    mask: np.ndarray            # uint8 [n]
    dims: list                  # [f, hidden..., classes]
    weights: list               # float32 [d_in, d_out] per layer
    lr: float = 0.02            # the learning rate the paper states for KW-GCN (Section 4.1)
    epochs: int = 1
    dtype: str = "f32"
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def glorot_weights(dims, seed: int):
    """U(-a, a), a = sqrt(6 / (d_in + d_out)), per layer, float32."""
    out = []
    for l in range(len(dims) - 1):
        d_in, d_out = dims[l], dims[l + 1]
        a = np.sqrt(6.0 / (d_in + d_out))
        u = rng.uniform(seed, 9000 + l, d_in * d_out)
        out.append(((2.0 * u - 1.0) * a).astype(np.float32).reshape(d_in, d_out))
    return out


def _features(seed: int, n: int, f: int) -> np.ndarray:
    return rng.normal_f32(seed, 7000, n * f).reshape(n, f)


def _bernoulli_mask(seed: int, n: int, p: float) -> np.ndarray:
    return (rng.uniform(seed, 7100, n) < p).astype(np.uint8)


def tiny(seed: int = 0, n: int = 2048, messy: bool = False, classes: int = 7) -> Workload:
    """Config 1: Erdos-Renyi, average degree 4, 256 -> 16 -> 7 (or another number of classes)."""
    m = 2 * n
    rowptr, col = graphs.erdos_renyi_gnm(n, m, seed)
    if messy:
        rowptr, col = graphs.messy_copy(n, rowptr, col, seed)
    dims = [256, 16, classes]
    x = _features(seed, n, dims[0])
    labels = rng.integers(seed, 7200, n, dims[-1]).astype(np.int32)
    mask = _bernoulli_mask(seed, n, 0.5)
    return Workload("c1_tiny_er", n, n, rowptr, col, x, labels, mask, dims, glorot_weights(dims, seed), epochs=1)


def chung_lu_mid(seed: int = 0, scale: float = 1.0) -> Workload:
    """Config 2: power-law (exponent 2.5) graph, average degree 20, 20 communities with
    80 % of edges inside; 128 -> 128 -> 40; label = 2 * community + (id mod 2)."""
    n = max(400, int(round(100_000 * scale)))
    rowptr, col, comm = graphs.community_power_law(n, 20, 20.0, 2.5, seed, p_intra=0.8)
    dims = [128, 128, 40]
    x = _features(seed, n, dims[0])
    labels = (2 * comm + (np.arange(n) % 2)).astype(np.int32)
    mask = _bernoulli_mask(seed, n, 0.6)
    return Workload("c2_chung_lu_100k", n, n, rowptr, col, x, labels, mask, dims, glorot_weights(dims, seed),
                    epochs=20)


def reddit_partition(seed: int = 0, scale: float = 1.0, avg_degree: float = 490.0, extra_frac: float = 0.02,
                     shuffle_ids: bool = False, p_intra: float = 0.8, p_cut: float = 0.05) -> Workload:
    """Config 3: one partition of a Reddit-shaped graph plus boundary-approximation vertices.

    n_local vertices in 50 communities; 5 % of edge draws are cut edges whose far end is
    one of extra_frac * n_local extra vertices (Section 3.1: the approximate view of the
    other partitions); 80 % of the remaining draws stay inside the community.  Extra
    vertices carry the mean of 8 independent N(0,1) feature rows, are outside the train
    mask and have no edges among themselves.  602 -> 128 -> 41.
    """
    n_local = max(500, int(round(46_600 * scale)))
    n_extra = int(round(extra_frac * n_local))
    deg = avg_degree * min(1.0, max(scale, 0.05) ** 0.5) if scale < 1.0 else avg_degree
    rowptr, col, comm = graphs.community_power_law(n_local, 50, deg, 2.5, seed, p_intra=p_intra,
                                                   n_extra=n_extra, p_cut=p_cut)
    n = n_local + n_extra
    dims = [602, 128, 41]
    x = np.empty((n, dims[0]), dtype=np.float32)
    x[:n_local] = _features(seed, n_local, dims[0])
    if n_extra:
        acc = np.zeros((n_extra, dims[0]), dtype=np.float64)
        for k in range(8):
            acc += rng.normal_f32(seed, 7010 + k, n_extra * dims[0]).reshape(n_extra, dims[0])
        x[n_local:] = (acc / 8.0).astype(np.float32)
    labels = np.zeros(n, dtype=np.int32)
    labels[:n_local] = comm % dims[-1]
    mask = np.zeros(n, dtype=np.uint8)
    mask[:n_local] = _bernoulli_mask(seed, n_local, 0.66)
    if shuffle_ids:
        new_id = rng.permutation(seed, 7300, n)
        rowptr, col = graphs.relabel(n, rowptr, col, new_id)
        inv = np.empty(n, dtype=np.int64)
        inv[new_id] = np.arange(n)
        x, labels, mask = x[inv], labels[inv], mask[inv]
    return Workload("c3_reddit_partition", n, n_local, rowptr, col, x, labels, mask, dims,
                    glorot_weights(dims, seed), epochs=200,
                    extra={"n_extra": n_extra, "shuffled": shuffle_ids})


def reddit_full(seed: int = 0, scale: float = 1.0, avg_degree: float = 490.0) -> Workload:
    """Config 4: the whole Reddit-shaped graph, 232,965 vertices, no extra vertices."""
    n = max(500, int(round(232_965 * scale)))
    deg = avg_degree * min(1.0, max(scale, 0.05) ** 0.5) if scale < 1.0 else avg_degree
    rowptr, col, comm = graphs.community_power_law(n, 50, deg, 2.5, seed, p_intra=0.8)
    dims = [602, 128, 41]
    x = _features(seed, n, dims[0])
    labels = (comm % dims[-1]).astype(np.int32)
    mask = _bernoulli_mask(seed, n, 0.66)
    return Workload("c4_reddit_full", n, n, rowptr, col, x, labels, mask, dims, glorot_weights(dims, seed),
                    epochs=20)


def rmat_large(seed: int = 0, scale: float = 1.0) -> Workload:
    """Config 5: R-MAT (0.57, 0.19, 0.19, 0.05), average degree 50, 100 -> 256 -> 256 -> 47,
    features and activations stored in bf16."""
    n = max(1000, int(round(2_400_000 * scale)))
    bits = max(10, int(np.ceil(np.log2(n))))
    rowptr, col = graphs.rmat(bits, n, 25 * n, 0.57, 0.19, 0.19, seed)
    dims = [100, 256, 256, 47]
    x = _features(seed, n, dims[0])
    labels = rng.integers(seed, 7200, n, dims[-1]).astype(np.int32)
    mask = _bernoulli_mask(seed, n, 0.10)
    return Workload("c5_rmat_2p4m_bf16", n, n, rowptr, col, x, labels, mask, dims, glorot_weights(dims, seed),
                    epochs=5, dtype="bf16")


def planted_classes(seed: int = 0, n: int = 20_000, n_comm: int = 40, avg_degree: float = 30.0, p_intra: float = 0.7,
                    f: int = 64, hidden: int = 32, signal: float = 0.35, train_frac: float = 0.7) -> Workload:
    """A community graph whose labels can be learnt, for the training scheme of Section 3.2 (partitions, one model
    copy per worker, parameter averaging): n vertices in n_comm equal communities (blocks of consecutive ids),
    power-law degrees, a share p_intra of the edges inside the communities; label = community; features = signal
    times a seeded unit-variance centroid of the class plus N(0, 1) noise, so one vertex alone says little and the
    neighbourhood mean says a lot.  mask: train_frac of the vertices; extra["heldout"]: all the others."""
    rowptr, col, comm = graphs.community_power_law(n, n_comm, avg_degree, 2.5, seed, p_intra=p_intra)
    dims = [f, hidden, n_comm]
    centroids = rng.normal_f32(seed, 7400, n_comm * f).reshape(n_comm, f)
    x = (signal * centroids[comm] + _features(seed, n, f)).astype(np.float32)
    mask = _bernoulli_mask(seed, n, train_frac)
    return Workload("planted_%d_classes" % n_comm, n, n, rowptr, col, x, comm.astype(np.int32), mask, dims,
                    glorot_weights(dims, seed), epochs=30, extra={"heldout": (1 - mask).astype(np.uint8)})


BY_NAME = {
    "c1": tiny,
    "c2": chung_lu_mid,
    "c3": reddit_partition,
    "c4": reddit_full,
    "c5": rmat_large,
}
