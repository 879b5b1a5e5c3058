"""CPU oracle for the paper's subgraph approximation (TEST INFRASTRUCTURE ONLY).

Builds the augmented partition P_o[p] of Algorithm 1 ("breadth-first random sampling of
vertices", Section 3.1) and then drops every edge that does not have both ends in it
(Section 4: after the sampling "all other edges between the subgraphs are dropped").
Plain Python sets and loops: for small graphs only.  Nothing here is shared with, or
imported by, the GPU package.

Reading of the algorithm (the listing is ambiguous in its recursive step, see the design notes):
  * nts = floor(O * N_p / (M - 1)) vertices are wanted from every other partition op
    (line 2 of Algorithm 1; N_p counts the vertices of p).
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
    """nts of Algorithm 1, line 2 (a single partition has no other partition to sample from)."""
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
