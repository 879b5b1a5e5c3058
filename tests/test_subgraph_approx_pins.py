"""Pins for the oracle of Algorithm 1 (subgraph approximation) and the edge dropping that follows.  CPU only."""
import os

import numpy as np
import pytest

from oracle import subgraph_approx as SA
from synth import graphs, rng

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _random_partitioned_graph(n, p_edge, n_parts, seed):
    u = rng.uniform(seed, 1, n * n).reshape(n, n)
    a = np.triu(u < p_edge, 1)
    a = a | a.T
    part = rng.integers(seed, 2, n, n_parts).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    cols = []
    for i in range(n):
        cols.extend(np.nonzero(a[i])[0].tolist())
        rowptr[i + 1] = len(cols)
    return a, rowptr, np.array(cols, dtype=np.int32), part


def test_overlap_to_overhead_map_printed_in_the_paper():
    table = np.loadtxt(os.path.join(GOLD, "overlap_overhead.txt"), comments="#")
    n_p = 40_000
    for m, o_pct, share_pct, overhead_pct in table:
        m = int(m)
        nts = SA.vertices_to_sample(o_pct / 100.0, n_p, m)
        assert abs(100.0 * nts / n_p - share_pct) < 0.01
        overhead = 100.0 * (m - 1) * nts / (m * n_p)
        assert abs(overhead - overhead_pct) < 0.05        # Table 2 prints 3.3 for 3.33


def test_path_graph_by_hand():
    # 0-1-2 | 3-4-5 : partition 0 sees 3 at one hop, 4 at two, 5 at three
    n = 6
    rowptr, col = graphs.pairs_to_csr(n, np.arange(5), np.arange(1, 6))
    part = np.array([0, 0, 0, 1, 1, 1], dtype=np.int32)
    v, nl, lv = SA.augmented_partition(n, rowptr, col, part, 2, 0, 1.0, seed=1)       # nts = 3: whole other side
    assert v.tolist() == [0, 1, 2, 3, 4, 5] and nl == 3
    assert lv[1] == [{3}, {4}, {5}]
    v, nl, lv = SA.augmented_partition(n, rowptr, col, part, 2, 0, 0.67, seed=1)      # nts = 2: two levels
    assert v.tolist() == [0, 1, 2, 3, 4] and lv[1] == [{3}, {4}]
    v, nl, _ = SA.augmented_partition(n, rowptr, col, part, 2, 0, 0.0, seed=1)        # no overlap: nothing added
    assert v.tolist() == [0, 1, 2]
    rp, cl = SA.induced_subgraph(n, rowptr, col, np.array([0, 1, 2, 3, 4]))
    assert rp.tolist() == [0, 1, 3, 5, 7, 8] and cl.tolist() == [1, 0, 2, 1, 3, 2, 4, 3]   # edge 4-5 dropped


def test_random_choice_takes_the_smallest_keys():
    # star: centre 0 in partition 0, leaves 1..8 in partition 1; nts = 3 of the 8 leaves
    n = 9
    rowptr, col = graphs.pairs_to_csr(n, np.zeros(8, dtype=np.int64), np.arange(1, 9))
    part = np.array([0] + [1] * 8, dtype=np.int32)
    part0 = part.copy()
    # N_p = 1 would give nts = 0: give partition 0 three more isolated members so that nts = floor(0.75 * 4) = 3
    n2 = n + 3
    rowptr2 = np.concatenate([rowptr, [rowptr[-1]] * 3])
    part2 = np.concatenate([part0, [0, 0, 0]]).astype(np.int32)
    v, nl, lv = SA.augmented_partition(n2, rowptr2, col, part2, 2, 0, 0.75, seed=5)
    assert nl == 4 and lv[1] == [set(range(1, 9))]
    chosen = set(v[nl:].tolist())
    keys = {u: SA.sample_key(5, u) for u in range(1, 9)}
    assert chosen == set(sorted(keys, key=keys.get)[:3])
    v_other, _, _ = SA.augmented_partition(n2, rowptr2, col, part2, 2, 0, 0.75, seed=6)
    assert len(v_other) == len(v)                       # another seed: same count, (almost surely) another draw
    assert len(set(keys.values())) == 8                 # the key is injective: no ties to break


@pytest.mark.parametrize("n,p_edge,n_parts,overlap,seed", [(60, 0.06, 3, 0.3, 1), (90, 0.03, 4, 0.5, 2),
                                                            (70, 0.02, 2, 0.9, 3), (80, 0.10, 5, 0.1, 4)])
def test_levels_against_dense_boolean_algebra(n, p_edge, n_parts, overlap, seed):
    a, rowptr, col, part = _random_partitioned_graph(n, p_edge, n_parts, seed)
    for p in range(n_parts):
        v, nl, lv = SA.augmented_partition(n, rowptr, col, part, n_parts, p, overlap, seed)
        local = part == p
        assert v[:nl].tolist() == np.nonzero(local)[0].tolist()
        nts = int(np.floor(overlap * local.sum() / (n_parts - 1)))
        extra = v[nl:]
        assert np.all(np.diff(extra) > 0) and not np.any(local[extra])
        for op in range(n_parts):
            if op == p:
                continue
            # breadth-first levels inside op, by matrix-vector products on the dense 0/1 adjacency
            frontier, seen, levels = local.copy(), np.zeros(n, dtype=bool), []
            while True:
                lvl = (a[:, frontier].any(axis=1)) & (part == op) & ~seen
                if not lvl.any():
                    break
                levels.append(set(np.nonzero(lvl)[0].tolist()))
                seen |= lvl
                frontier = lvl
            taken = set(extra[part[extra] == op].tolist())
            reachable = set().union(*levels) if levels else set()
            assert len(taken) == min(nts, len(reachable))
            assert taken <= reachable
            # whole levels first, then part of one level
            left = nts
            for k, lvl in enumerate(levels):
                if left <= 0:
                    assert not (taken & lvl)
                elif len(lvl) <= left:
                    assert lvl <= taken
                    left -= len(lvl)
                else:
                    assert len(taken & lvl) == left
                    left = 0
            assert lv[op] == levels[:len(lv[op])]
        # induced subgraph: symmetric, exactly the edges inside the vertex set, local-local edges all kept
        rp, cl = SA.induced_subgraph(n, rowptr, col, v)
        sub = a[np.ix_(v, v)]
        got = np.zeros_like(sub)
        for i in range(len(v)):
            got[i, cl[rp[i]:rp[i + 1]]] = True
        np.testing.assert_array_equal(got, sub)


@pytest.mark.parametrize("n,p_edge,n_parts,overlap,seed", [(120, 0.05, 3, 0.4, 7), (150, 0.015, 4, 1.5, 8),
                                                            (100, 0.2, 5, 0.2, 9)])
def test_array_version_equals_set_version(n, p_edge, n_parts, overlap, seed):
    _, rowptr, col, part = _random_partitioned_graph(n, p_edge, n_parts, seed)
    for p in range(n_parts):
        v, nl, _ = SA.augmented_partition(n, rowptr, col, part, n_parts, p, overlap, seed)
        v2, nl2 = SA.augmented_partition_np(n, rowptr, col, part, n_parts, p, overlap, seed)
        assert nl == nl2
        np.testing.assert_array_equal(v, v2)
        rp, cl = SA.induced_subgraph(n, rowptr, col, v)
        rp2, cl2 = SA.induced_subgraph_np(n, rowptr, col, v2)
        np.testing.assert_array_equal(rp, rp2)
        np.testing.assert_array_equal(cl, cl2)
    for v in (0, 1, 77, 2 ** 31 - 1):
        assert int(SA.sample_keys_np(seed, np.array([v]))[0]) == SA.sample_key(seed, v)
