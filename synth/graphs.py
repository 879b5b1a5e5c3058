"""Seeded synthetic graphs with the shapes of the paper's workloads.

The paper trains on Reddit and Amazon2M (Table 1); neither dataset is available, so
these generators make stand-ins of the same shape: power-law degrees, planted
communities (the role METIS partitions and subreddit/product communities play),
and, for the partition workload, a few percent of extra boundary vertices that
carry approximated external information and are linked only to local vertices
(Section 3.1).  Output is always a *raw* adjacency in CSR form (rowptr int64,
col int32): structurally symmetric, no promise about self-loops or duplicates.
Nothing here computes any part of the GCN itself.
"""
from __future__ import annotations

import numpy as np

from . import rng


# --------------------------------------------------------------------------- CSR assembly
def pairs_to_csr(n: int, u: np.ndarray, v: np.ndarray):
    """Undirected pairs -> symmetric CSR of A (both directions stored, duplicate pairs
    collapsed, pairs with u == v dropped, columns ascending)."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    keep = u != v
    u, v = u[keep], v[keep]
    key = np.concatenate([u * n + v, v * n + u])
    key = np.unique(key)
    rows = key // n
    col = (key - rows * n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n), out=rowptr[1:])
    return rowptr, col


def unique_pair_count(n: int, u: np.ndarray, v: np.ndarray) -> int:
    lo = np.minimum(u, v)
    hi = np.maximum(u, v)
    k = (lo * n + hi)[lo != hi]
    return int(np.unique(k).size)


def messy_copy(n: int, rowptr: np.ndarray, col: np.ndarray, seed: int):
    """A raw CSR with the same adjacency but as untidy as the library must accept:
    about 1 row in 3 gets an explicit self-loop, about 1 entry in 8 is stored twice,
    and the order inside every row is scrambled."""
    deg = np.diff(rowptr)
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    c = col.astype(np.int64)
    dup = rng.uniform(seed, 101, c.size) < 0.125
    loops = np.nonzero(rng.uniform(seed, 102, n) < 1.0 / 3.0)[0]
    rows2 = np.concatenate([rows, rows[dup], loops, loops[::2]])
    cols2 = np.concatenate([c, c[dup], loops, loops[::2]])
    order = np.lexsort((rng.bits(seed, 103, rows2.size), rows2))
    rows2, cols2 = rows2[order], cols2[order]
    rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows2, minlength=n), out=rp[1:])
    return rp, cols2.astype(np.int32)


# --------------------------------------------------------------------------- samplers
class _Weighted:
    """Draw vertex ids with probability proportional to w, globally or inside a block
    of consecutive ids, by inverting the cumulative weights."""

    def __init__(self, w: np.ndarray):
        self.cum = np.concatenate([[0.0], np.cumsum(w, dtype=np.float64)])
        self.n = w.size

    def draw(self, unif: np.ndarray, lo: np.ndarray | int = 0, hi: np.ndarray | int | None = None):
        hi = self.n if hi is None else hi
        a = self.cum[lo]
        b = self.cum[hi]
        t = a + unif * (b - a)
        idx = np.searchsorted(self.cum, t, side="right") - 1
        return np.clip(idx, lo, np.asarray(hi) - 1)


def power_law_weights(n: int, exponent: float, cap: float | None, seed: int, stream: int):
    """Expected-degree weights w ~ rank^(-1/(exponent-1)) handed to vertices in a seeded
    random order, so heavy vertices are spread over all communities; optional cap."""
    ranks = rng.permutation(seed, stream, n).astype(np.float64)
    w = (ranks + 1.0 + 0.005 * n) ** (-1.0 / (exponent - 1.0))
    w /= w.mean()
    if cap is not None:
        w = np.minimum(w, cap)
        w /= w.mean()
    return w


# --------------------------------------------------------------------------- generators
def erdos_renyi_gnm(n: int, m: int, seed: int):
    """G(n, m): the first m distinct undirected pairs of a seeded stream of random pairs."""
    draws = int(m * 1.25) + 64
    u = rng.integers(seed, 1, draws, n)
    v = rng.integers(seed, 2, draws, n)
    lo, hi = np.minimum(u, v), np.maximum(u, v)
    ok = lo != hi
    key = (lo * n + hi)[ok]
    _, first = np.unique(key, return_index=True)
    first = np.sort(first)[:m]
    assert first.size == m, "not enough distinct pairs drawn"
    key = key[first]
    return pairs_to_csr(n, key // n, key % n)


def community_power_law(n_local: int, n_comm: int, avg_degree: float, exponent: float, seed: int,
                        p_intra: float, n_extra: int = 0, p_cut: float = 0.0, cap_sqrt: bool = True,
                        max_rounds: int = 16):
    """Chung-Lu-style graph over n_local vertices in n_comm blocks of consecutive ids.

    Each undirected edge draw picks its first endpoint u with probability ~ w_u.  With
    probability p_cut it is a cut edge and its far end is replaced by one of n_extra
    boundary vertices (ids n_local..), chosen uniformly; otherwise the second endpoint
    is drawn ~ w inside u's block with probability p_intra, else ~ w over all local
    vertices.  Draws repeat in seeded rounds until the number of distinct pairs gives
    the requested mean degree (stored entries per local vertex) to within 0.5 %.
    There are no edges between two boundary vertices.
    """
    n = n_local + n_extra
    target_entries = float(n_local) * avg_degree      # stored entries in the local rows
    cap = None
    if cap_sqrt:
        cap = np.sqrt(n_local * avg_degree) / avg_degree  # in units of the mean weight
    w = power_law_weights(n_local, exponent, cap, seed, 10)
    sampler = _Weighted(w)
    block = -(-n_local // n_comm)
    keys = np.empty(0, dtype=np.int64)

    def local_entries(k):
        # a local-local pair is stored in two local rows, a cut pair in one
        return 2 * k.size - int(np.count_nonzero(k % n >= n_local))

    for rnd in range(max_rounds):
        need = target_entries - local_entries(keys)
        if need <= 0.005 * target_entries:
            break
        per_pair = 2.0 - (p_cut if n_extra > 0 else 0.0)
        draws = int(need / per_pair * (1.10 if rnd == 0 else 1.6)) + 16
        s = 100 + 10 * rnd
        u = sampler.draw(rng.uniform(seed, s + 1, draws))
        kind = rng.uniform(seed, s + 2, draws)
        r2 = rng.uniform(seed, s + 3, draws)
        r3 = rng.uniform(seed, s + 4, draws)
        lo = (u // block) * block
        hi = np.minimum(lo + block, n_local)
        v_in = sampler.draw(r3, lo, hi)
        v_out = sampler.draw(r3)
        v = np.where(r2 < p_intra, v_in, v_out)
        if n_extra > 0 and p_cut > 0:
            cut = kind < p_cut
            v_cut = n_local + np.minimum((r3 * n_extra).astype(np.int64), n_extra - 1)
            v = np.where(cut, v_cut, v)
        a, b = np.minimum(u, v), np.maximum(u, v)
        k = (a * n + b)[a != b]
        new = np.setdiff1d(k, keys)                  # sorted, distinct, not seen before
        gain = local_entries(new)
        if gain > need:
            # thin the new pairs (seeded, uniform) so the total lands on the target
            take = int(new.size * need / gain)
            sel = rng.permutation(seed, s + 5, new.size)[:take]
            new = new[np.sort(sel)]
        keys = np.union1d(keys, new)
    rowptr, col = pairs_to_csr(n, keys // n, keys % n)
    comm = np.minimum(np.arange(n_local) // block, n_comm - 1).astype(np.int32)
    return rowptr, col, comm


def rmat(scale: int, n: int, n_pairs: int, a: float, b: float, c: float, seed: int, max_rounds: int = 8):
    """R-MAT: every edge picks one quadrant per bit level with probabilities (a, b, c, d);
    edges with an endpoint >= n are rejected; rounds repeat until n_pairs distinct
    undirected pairs exist (the last round is thinned to hit the count)."""
    keys = np.empty(0, dtype=np.int64)
    for rnd in range(max_rounds):
        need = n_pairs - keys.size
        if need <= 0:
            break
        draws = int(need * 1.35) + 1024
        u = np.zeros(draws, dtype=np.int64)
        v = np.zeros(draws, dtype=np.int64)
        for lvl in range(scale):
            r = rng.uniform(seed, 1000 * (rnd + 1) + lvl, draws)
            right = ((r >= a) & (r < a + b)) | (r >= a + b + c)
            down = r >= a + b
            u = (u << 1) | down
            v = (v << 1) | right
        ok = (u < n) & (v < n) & (u != v)
        lo, hi = np.minimum(u[ok], v[ok]), np.maximum(u[ok], v[ok])
        k = lo * n + hi
        new = np.setdiff1d(k, keys)
        if keys.size + new.size > n_pairs:
            sel = rng.permutation(seed, 1000 * (rnd + 1) + 999, new.size)[: n_pairs - keys.size]
            new = new[np.sort(sel)]
        keys = np.union1d(keys, new)
    return pairs_to_csr(n, keys // n, keys % n)


def relabel(n: int, rowptr: np.ndarray, col: np.ndarray, new_id: np.ndarray):
    """The same graph with vertex i renamed new_id[i] (a permutation of 0..n-1)."""
    deg = np.diff(rowptr)
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    return pairs_to_csr(n, new_id[rows], new_id[col.astype(np.int64)])
