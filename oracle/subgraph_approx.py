"""CPU oracle for the paper's subgraph approximation (TEST INFRASTRUCTURE ONLY).

Builds the augmented partition P_o[p] of Algorithm 1 (the breadth-first random sampling
of Section 3.1) and then keeps only the edges with both ends in it (Section 4: cut edges
that the sampling did not bring in are discarded).
Plain Python sets and loops: for small graphs only.  Nothing here is shared with, or
imported by, the GPU package.

Reading of the algorithm (the listing is ambiguous in its recursive step, see the design notes):
  * nts = floor(O * N_p / (M - 1)) vertices are wanted from every other partition op
    (the sizing rule at the top of Algorithm 1; N_p counts the vertices of p).
  * Level 1 of op is every vertex of op adjacent to a vertex of p (`neighbors(p, op)`).
    Level k + 1 is every vertex of op adjacent to a level-k vertex and not in an earlier
    level (`neighbors(selection, op) \\ selection`).
  * Levels are taken whole, in order, while they fit into what is left of nts; from the
    first level that does not fit, exactly the missing number is drawn at random; an
    empty level ends the search.
  * "random(selection, k)": the paper names no generator.  Here: the k vertices of the
    level with the smallest key(v) = mix(mix(seed) ^ v), mix = SplitMix64's output
    function — a bijection on 64-bit words, so there are no ties and the draw does not
    depend on any processing order.
  * The result lists the vertices of p first (ascending id), then the sampled vertices
    (ascending id); new ids follow that order.  Kept edges: both ends in the result.
"""
from __future__ import annotations

import numpy as np

_M = (1 << 64) - 1


def _mix(z: int) -> int:
    z = (z + 0x9E3779B97F4A7C15) & _M
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M
    return z ^ (z >> 31)


def sample_key(seed: int, v: int) -> int:
    return _mix(_mix(seed & _M) ^ v)


def vertices_to_sample(overlap: float, n_p: int, n_parts: int) -> int:
    """nts, the sizing rule at the top of Algorithm 1 (a single partition has no other partition to sample from)."""
    if n_parts < 2:
        return 0
    return int(np.floor(overlap * n_p / (n_parts - 1)))


def augmented_partition(n: int, rowptr, col, part, n_parts: int, p: int, overlap: float, seed: int):
    """-> (vertices, n_local, levels) with `vertices` the old ids in new-id order and `levels` a dict
    {op: [set(level 1), set(level 2), ...]} of the levels that were looked at (for the tests)."""
    rowptr = np.asarray(rowptr)
    col = np.asarray(col)
    part = np.asarray(part)
    local = [v for v in range(n) if part[v] == p]
    nts = vertices_to_sample(overlap, len(local), n_parts)
    sampled = set()
    seen_levels = {}
    for op in range(n_parts):
        if op == p:
            continue
        need = nts
        frontier = set(local)
        visited = set()
        seen_levels[op] = []
        while need > 0:
            level = set()
            for v in frontier:
                for u in col[rowptr[v]:rowptr[v + 1]]:
                    u = int(u)
                    if part[u] == op and u not in visited:
                        level.add(u)
            if not level:
                break
            seen_levels[op].append(level)
            if len(level) >= need:
                chosen = sorted(level, key=lambda v: sample_key(seed, v))[:need]
                sampled.update(chosen)
                need = 0
            else:
                sampled.update(level)
                need -= len(level)
                visited |= level
                frontier = level
    vertices = np.array(local + sorted(sampled), dtype=np.int64)
    return vertices, len(local), seen_levels


def induced_subgraph(n: int, rowptr, col, vertices):
    """Edges with both ends in `vertices`, renamed to positions in `vertices`.  Raw CSR (row order of the
    input kept, no promise about sorting): -> (rowptr int64, col int32)."""
    rowptr = np.asarray(rowptr)
    col = np.asarray(col)
    new_id = -np.ones(n, dtype=np.int64)
    new_id[vertices] = np.arange(len(vertices))
    out_ptr = [0]
    out_col = []
    for v in vertices:
        for u in col[rowptr[v]:rowptr[v + 1]]:
            if new_id[u] >= 0:
                out_col.append(int(new_id[u]))
        out_ptr.append(len(out_col))
    return np.array(out_ptr, dtype=np.int64), np.array(out_col, dtype=np.int32)


# ---------------------------------------------------------------------------------------------------------
# The same reading with numpy arrays instead of Python sets, for graphs of full size (tens of millions of
# edges).  Checked against the set version above on small graphs by the CPU tests.
def _mix_np(z):
    z = z + np.uint64(0x9E3779B97F4A7C15)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def sample_keys_np(seed: int, v):
    with np.errstate(over="ignore"):
        k0 = _mix_np(np.array([seed & _M], dtype=np.uint64))[0]
        return _mix_np(k0 ^ np.asarray(v, dtype=np.uint64))


def _neighbours_of(rowptr, col, rows):
    """All column entries of the given rows (with repeats)."""
    lens = rowptr[rows + 1] - rowptr[rows]
    if lens.sum() == 0:
        return np.empty(0, dtype=np.int64)
    starts = np.repeat(rowptr[rows], lens)
    within = np.arange(lens.sum()) - np.repeat(np.cumsum(lens) - lens, lens)
    return col[starts + within].astype(np.int64)


def augmented_partition_np(n: int, rowptr, col, part, n_parts: int, p: int, overlap: float, seed: int):
    """-> (vertices, n_local), as augmented_partition."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col)
    part = np.asarray(part)
    local = np.nonzero(part == p)[0]
    nts = vertices_to_sample(overlap, len(local), n_parts)
    taken = np.zeros(n, dtype=bool)
    for op in range(n_parts):
        if op == p or nts == 0:
            continue
        need = nts
        frontier = local
        visited = np.zeros(n, dtype=bool)
        while need > 0:
            nb = _neighbours_of(rowptr, col, frontier)
            nb = nb[(part[nb] == op) & ~visited[nb]]
            level = np.unique(nb)
            if level.size == 0:
                break
            if level.size >= need:
                keys = sample_keys_np(seed, level)
                taken[level[np.argsort(keys, kind="stable")[:need]]] = True
                need = 0
            else:
                taken[level] = True
                visited[level] = True
                need -= level.size
                frontier = level
    return np.concatenate([local, np.nonzero(taken)[0]]).astype(np.int64), int(len(local))


def induced_subgraph_np(n: int, rowptr, col, vertices):
    """As induced_subgraph, vectorised."""
    rowptr = np.asarray(rowptr, dtype=np.int64)
    col = np.asarray(col)
    new_id = -np.ones(n, dtype=np.int64)
    new_id[vertices] = np.arange(len(vertices))
    lens = rowptr[vertices + 1] - rowptr[vertices]
    entries = _neighbours_of(rowptr, col, np.asarray(vertices, dtype=np.int64))
    owner = np.repeat(np.arange(len(vertices)), lens)
    ids = new_id[entries]
    keep = ids >= 0
    out_ptr = np.zeros(len(vertices) + 1, dtype=np.int64)
    np.cumsum(np.bincount(owner[keep], minlength=len(vertices)), out=out_ptr[1:])
    return out_ptr, ids[keep].astype(np.int32)
