"""CPU oracle of GAD-Partition's importance-based subgraph augmentation.  TEST INFRASTRUCTURE ONLY.

arXiv 2110.02987, Section 3.2.2: candidate replication nodes (Definition 2), Monte-Carlo importance I(v) (Eq. 3),
the number of walks from the Monte-Carlo error (Eq. 4), depth-first selection of whole walks (Algorithm 1).
Plain numpy / Python loops over an explicit CSR of the original graph; nothing here is shared with, imported by,
or imports the HIP path.  Random numbers come from a counter-based generator defined here (`draw`); the HIP path
implements the same definition on its side, so both walk the same paths.

Readings taken where the paper is silent or garbled:

* The walks run on the ORIGINAL graph (Algorithm 1: random_walk(step = l, graph = G)), start at a uniformly drawn
  boundary node, take l uniform steps (l = number of GCN layers, Property 1); a node without neighbours stays.
* RW_j(v) of Eq. 3 is an indicator: a node seen twice by one walk counts once for that walk.  Only nodes
  outside the partition are counted (Eq. 3: v not in v_i); the start node itself is never a candidate.
* First batch: d |B| walks with d the average degree of the boundary nodes, i.e. exactly sum_{v in B} deg(v).
* Algorithm 1 prints "prob.var(), prob.mean()" and n = (z_c sigma_x / (xbar E))^2 (Eq. 4 squared and solved for n).
  sigma_x and xbar are read as the population standard deviation and the mean of I(v) over the candidates the
  first batch has visited; with counts c_v, m visited candidates, S1 = sum c, S2 = sum c^2 this is
  n = ceil((z_c / E)^2 (m S2 - S1^2) / S1^2), z_c = 1.96, E = 0.05.  The total is max(first batch, n), capped by
  the caller.  n is an integer decided by a real number: it is evaluated exactly, (z_c / E)^2 = 38416 / 25 as a
  rational and the ceiling of an integer quotient, so that no rounding of an intermediate can move it.
* The score of a walk is the sum of I(v) over its l steps (positions outside the partition; a node met twice
  adds twice).  Walks are taken in descending score, ties by walk number; their nodes are added in step order
  until the budget is reached (Algorithm 1, the repeat loop), so every added node hangs on the partition through
  the earlier nodes of its walk.
* The budget n(g_i) = alpha (1 + d(g_i)) |v| is passed in by the caller (Eq. 6 prints |v|, Algorithm 1 |v_i|).
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

Z_C = 1.96
E_MC = 0.05
_M64 = (1 << 64) - 1


def draw(seed: int, walk: int, step: int) -> int:
    """32 random bits for (seed, walk, step): a splitmix64-style finaliser of the mixed counter."""
    x = (seed ^ (walk * 0x9E3779B97F4A7C15) ^ (step * 0xD1B54A32D192ED03)) & _M64
    x = (x + 0x9E3779B97F4A7C15) & _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return x >> 32


def below(r32: int, m: int) -> int:
    """Map 32 random bits to [0, m) by multiply-shift."""
    return (r32 * m) >> 32


def neighbours(rowptr, colidx, v):
    """Neighbours of v in a CSR of A + I (sorted columns, one self loop per row), without the self loop."""
    row = colidx[rowptr[v]:rowptr[v + 1]]
    return row[row != v]


def boundary(rowptr, colidx, part):
    """B(g_i): nodes of the partition with an edge leaving it (Definition 2), in the order of `part`."""
    inside = np.zeros(len(rowptr) - 1, dtype=bool)
    inside[part] = True
    return np.array([v for v in part if np.any(~inside[neighbours(rowptr, colidx, v)])], dtype=np.int64)


def walk(rowptr, colidx, B, l, seed, j):
    """Walk number j: [start, step 1, ..., step l]."""
    cur = int(B[below(draw(seed, j, 0), len(B))])
    seq = [cur]
    for t in range(1, l + 1):
        nb = neighbours(rowptr, colidx, cur)
        if len(nb):
            cur = int(nb[below(draw(seed, j, t), len(nb))])
        seq.append(cur)
    return seq


def mc_walk_count(counts) -> int:
    """Number of walks from Eq. 4 at E = 0.05, z_c = 1.96, given the visit counts of the first batch."""
    c = np.asarray([int(x) for x in counts if x > 0], dtype=object)
    if len(c) == 0:
        return 0
    m, s1, s2 = len(c), int(sum(c)), int(sum(x * x for x in c))
    q2 = (Fraction(str(Z_C)) / Fraction(str(E_MC))) ** 2               # 38416 / 25, exactly
    n = q2 * (m * s2 - s1 * s1) / (s1 * s1)                            # exact rational
    return -((-n.numerator) // n.denominator)                          # its ceiling


def augment(rowptr, colidx, part, l, budget, seed, max_walks=1 << 22):
    """Returns dict(halo = selected replication nodes in selection order, n_walks, counts, walks, boundary)."""
    rowptr = np.asarray(rowptr)
    colidx = np.asarray(colidx)
    part = np.asarray(part, dtype=np.int64)
    N = len(rowptr) - 1
    inside = np.zeros(N, dtype=bool)
    inside[part] = True
    B = boundary(rowptr, colidx, part)
    if len(B) == 0 or budget <= 0:
        return dict(halo=np.zeros(0, dtype=np.int64), n_walks=0, counts=np.zeros(N, dtype=np.int64), walks=[], boundary=B)
    n0 = int(sum(len(neighbours(rowptr, colidx, v)) for v in B))
    n0 = max(1, min(n0, max_walks))
    counts = np.zeros(N, dtype=np.int64)
    walks = []

    def run(j0, j1):
        for j in range(j0, j1):
            seq = walk(rowptr, colidx, B, l, seed, j)
            walks.append(seq)
            for v in set(seq[1:]):
                if not inside[v]:
                    counts[v] += 1

    run(0, n0)
    n_total = min(max(n0, mc_walk_count(counts)), max_walks)
    run(n0, n_total)
    score = [sum(int(counts[v]) for v in seq[1:] if not inside[v]) for seq in walks]
    order = sorted(range(n_total), key=lambda j: (-score[j], j))
    halo, seen = [], set()
    for j in order:
        for v in walks[j][1:]:
            if not inside[v] and v not in seen:
                if len(halo) == budget:
                    break
                seen.add(v)
                halo.append(v)
        if len(halo) == budget:
            break
    return dict(halo=np.asarray(halo, dtype=np.int64), n_walks=n_total, counts=counts, walks=walks, boundary=B)


def replica_budget(n_nodes, n_edges, n_total, alpha=0.01):
    """Eq. 5 and Eq. 6: d(g) = 2|e| / (|v| (|v| - 1)), n(g) = alpha (1 + d(g)) |v| with |v| = n_total."""
    d = 0.0 if n_nodes < 2 else 2.0 * n_edges / (n_nodes * (n_nodes - 1.0))
    return int(alpha * (1.0 + d) * n_total)
