"""CPU oracle of the GraphSAGE-mean training step (TEST INFRASTRUCTURE ONLY).

Only the tests and the benchmark's CPU-baseline leg may import this module; it shares no code with the GPU
package.  Plain numpy in fp64, written from the method's statement (Section 4.1: sample a fixed number of
neighbours, aggregate their features with the element-wise mean, two layers, batches of 256 vertices, Adam),
one batch at a time:

    sample    for every target v of the batch: S2 neighbours;  for every level-1 vertex u (the targets and
              their samples): S1 neighbours
    layer 1   h_u = relu(W1^T [x_u | mean of the S1 sampled x])            for every level-1 vertex
    layer 2   z_v = W2^T [h_v | mean of the S2 sampled h]                  for every target
    loss      softmax cross-entropy averaged over the batch, accuracy (Section 2.2)
    backward  dW2, then through the mean and the ReLU, dW1 (the features are constants)
    update    Adam

Readings where the paper is silent (all listed in the design notes):
  * a vertex's own row and the mean of its sampled neighbours are concatenated (Hamilton et al.'s Algorithm 1
    with the mean aggregator); no normalisation of the embeddings; the last layer has no activation;
  * sample sizes are parameters; S1 belongs to layer 1 (the outer hop), S2 to layer 2 (the targets' hop);
  * neighbours are drawn uniformly WITH replacement, always exactly S draws, from N(v) = the row of v without
    v itself; a vertex without neighbours contributes a zero mean; level-1 vertices are not deduplicated (a vertex
    sampled twice is computed twice, with independent outer samples);
  * draw j of instance m at a level uses the counter-based generator below with counter m * S + j, so a sample
    depends only on (seed, step, level, m, j) and the vertex's row.
"""
from __future__ import annotations

import numpy as np

_M = (1 << 64) - 1
_GOLD = 0x9E3779B97F4A7C15


def mix(z: int) -> int:
    """SplitMix64 output function applied to z + the golden-ratio increment."""
    z = (z + _GOLD) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def _mix_np(z):
    with np.errstate(over="ignore"):
        z = z + np.uint64(_GOLD)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def level_key(seed: int, step: int, level: int) -> int:
    return mix(mix(seed & _M) ^ ((step * 0xD1B54A32D192ED03) & _M) ^ ((level * 0x8CB92BA72F3D8DD7) & _M))


def sample_neighbours(rowptr, col, nodes, S: int, key: int) -> np.ndarray:
    """-> [len(nodes), S] int32.  Entry (m, j): the floor(u * d)-th member, in ascending order, of N(nodes[m]),
    where d = |N| and u in [0, 1) is the top 32 bits of mix(key + (m S + j) * golden) over 2^32; -1 when the
    vertex is -1 or has no neighbour."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col)
    nodes = np.asarray(nodes, dtype=np.int64)
    out = np.full((len(nodes), S), -1, dtype=np.int32)
    for m, v in enumerate(nodes):
        if v < 0:
            continue
        row = col[rowptr[v]:rowptr[v + 1]]
        nb = row[row != v]                       # ascending, as the rows are
        d = len(nb)
        if d == 0:
            continue
        counters = np.arange(m * S, (m + 1) * S, dtype=np.uint64)
        with np.errstate(over="ignore"):
            r = _mix_np(np.uint64(key) + counters * np.uint64(_GOLD))
        u = ((r >> np.uint64(32)) * np.uint64(d)) >> np.uint64(32)
        out[m] = nb[u.astype(np.int64)]
    return out


def _rows_or_zero(mat, idx):
    """mat[idx] with an all-zero row wherever idx is -1."""
    out = mat[np.maximum(idx, 0)].astype(np.float64)
    out[idx < 0] = 0.0
    return out


class Trace:
    """Everything one batch computes (fp64)."""


def forward(rowptr, col, X, W1, W2, batch, S1: int, S2: int, seed: int, step: int) -> Trace:
    t = Trace()
    X = np.asarray(X)
    W1 = np.asarray(W1, dtype=np.float64)
    W2 = np.asarray(W2, dtype=np.float64)
    batch = np.asarray(batch, dtype=np.int64)
    B = len(batch)
    f = X.shape[1]
    assert W1.shape[0] == 2 * f and W2.shape[0] == 2 * W1.shape[1]
    t.inner = sample_neighbours(rowptr, col, batch, S2, level_key(seed, step, 2))             # [B, S2]
    t.nodes1 = np.concatenate([batch[:, None], t.inner.astype(np.int64)], axis=1).ravel()        # [B (1 + S2)]
    t.outer = sample_neighbours(rowptr, col, t.nodes1, S1, level_key(seed, step, 1))           # [B (1 + S2), S1]
    x_self = _rows_or_zero(X, t.nodes1)
    x_mean = np.zeros_like(x_self)
    for j in range(S1):
        x_mean += _rows_or_zero(X, t.outer[:, j])
    x_mean /= S1
    t.C1 = np.concatenate([x_self, x_mean], axis=1)                                            # [.., 2 f]
    t.Z1 = t.C1 @ W1
    t.H1 = np.maximum(t.Z1, 0.0)
    h = t.H1.reshape(B, 1 + S2, -1)
    t.C2 = np.concatenate([h[:, 0, :], h[:, 1:, :].sum(axis=1) / S2], axis=1)                  # [B, 2 hidden]
    t.logits = t.C2 @ W2
    return t


def loss_acc(logits, labels):
    """Mean softmax cross-entropy over the batch, number of correct arg-max predictions (lowest index wins ties),
    and dLoss/dlogits."""
    logits = np.asarray(logits, dtype=np.float64)
    B = logits.shape[0]
    m = logits.max(axis=1, keepdims=True)
    e = np.exp(logits - m)
    s = e.sum(axis=1, keepdims=True)
    p = e / s
    lse = (m + np.log(s)).ravel()
    loss = float((lse - logits[np.arange(B), labels]).sum() / B)
    correct = int((logits.argmax(axis=1) == labels).sum())
    d = p.copy()
    d[np.arange(B), labels] -= 1.0
    return loss, correct, d / B


def backward(t: Trace, W2, labels, S2: int):
    """-> dW1, dW2.  The ReLU decision [Z1 > 0] is taken on the trace's own pre-activations."""
    W2 = np.asarray(W2, dtype=np.float64)
    B = t.logits.shape[0]
    hidden = t.H1.shape[1]
    t.loss, t.correct, t.dlogits = loss_acc(t.logits, labels)
    dW2 = t.C2.T @ t.dlogits
    dC2 = t.dlogits @ W2.T
    dH = np.empty((B, 1 + S2, hidden))
    dH[:, 0, :] = dC2[:, :hidden]
    dH[:, 1:, :] = (dC2[:, hidden:] / S2)[:, None, :]
    on = t.Z1 > 0.0
    t.dZ1 = dH.reshape(B * (1 + S2), hidden) * on
    dW1 = t.C1.T @ t.dZ1
    return dW1, dW2
