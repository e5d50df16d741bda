"""Pins of the augmentation oracle (oracle/gad_augment.py) against what the paper and the mathematics fix:
Definition 2 (candidates lie within l hops of the boundary), Eq. 3 (Monte-Carlo importance converges to the
exact visit probabilities), Eq. 4 (walk count, by hand and through numpy's own std / mean), Eq. 5 / Eq. 6 (replica
budget by hand), and Algorithm 1's depth-first selection (no dangling nodes, walk order, budget)."""
import dataclasses

import numpy as np
import pytest
import scipy.sparse as sp

from oracle import gad_augment as AUG
from oracle import gad_csr as T1
from paper_2110_02987_amd import workloads as wl


def _whole_graph(n, avg, seed=0, max_degree=200):
    cfg = dataclasses.replace(wl.CONFIGS["products_small"], n_local=n, n_halo=0, global_factor=1, extra_edge_frac=0.0,
                              max_degree=max_degree, avg_degree=avg)
    gr = wl.make_graph(cfg, seed=seed)
    gr["local_ids"], gr["halo_ids"] = np.arange(n, dtype=np.int64), np.zeros(0, dtype=np.int64)
    return T1.build(**gr)


def _adj(G):
    A = sp.csr_matrix((np.ones(G.nnz), G.colidx, G.rowptr), shape=(G.n, G.n)).tolil()
    A.setdiag(0)
    return A.tocsr()


def test_generator_is_splitmix64_and_uniform():
    # splitmix64's published first output for state 0 is 0xE220A8397B1DCDAF; draw(0, 0, 0) is its upper half
    assert AUG.draw(0, 0, 0) == 0xE220A839
    # range reduction and uniformity: chi-square of 60,000 draws over 7 cells, separately for two steps
    for step in (0, 3):
        h = np.bincount([AUG.below(AUG.draw(12345, j, step), 7) for j in range(60_000)], minlength=7)
        assert ((h - 60_000 / 7) ** 2 / (60_000 / 7)).sum() < 30.0          # 6 degrees of freedom
    assert AUG.below(0xFFFFFFFF, 5) == 4 and AUG.below(0, 5) == 0
    # different steps of one walk are not copies of each other
    a = [AUG.draw(9, j, 1) for j in range(1000)]
    b = [AUG.draw(9, j, 2) for j in range(1000)]
    assert abs(np.corrcoef(a, b)[0, 1]) < 0.1


def test_walk_count_formula_eq4():
    assert AUG.mc_walk_count([1, 1, 1, 1, 0, 0]) == 0                        # equal importance: sigma = 0
    assert AUG.mc_walk_count([3, 1]) == 385                                  # (2*10 - 16)/16 * 1536.64 = 384.16
    rng = np.random.default_rng(1)
    c = rng.integers(0, 30, 500)
    x = c[c > 0] / 1000.0                                                    # I(v) after 1000 walks
    by_numpy = (AUG.Z_C * x.std() / (x.mean() * AUG.E_MC)) ** 2
    assert abs(AUG.mc_walk_count(c) - by_numpy) <= 1.0 + 1e-6 * by_numpy    # ceil of the same number


def test_replica_budget_eq5_eq6():
    # 4-cycle: density 2*4/(4*3) = 2/3; alpha (1 + 2/3) |v| with |v| = 3000 -> 50
    assert AUG.replica_budget(4, 4, 3000) == 50
    assert AUG.replica_budget(1000, 0, 100_000) == 1000                      # density 0: alpha |v|


def test_path_graph_depth_first_selection():
    """Path 0-1-2-3-4, partition {0, 1}: the boundary is {1}; node 3 can only be reached through node 2."""
    pairs = [(0, 1), (1, 2), (2, 3), (3, 4)]
    src = np.array([a for a, _ in pairs], dtype=np.int64)
    dst = np.array([b for _, b in pairs], dtype=np.int64)
    G = T1.build(src, dst, 5, np.arange(5, dtype=np.int64), np.zeros(0, dtype=np.int64))
    seen = set()
    for seed in range(40):
        r = AUG.augment(G.rowptr, G.colidx, [0, 1], 2, 5, seed)
        assert list(r["boundary"]) == [1]
        assert r["n_walks"] >= 2                                             # first batch: deg(1) = 2 walks
        halo = list(r["halo"])
        assert halo in ([], [2], [2, 3])                                     # 3 never without (or before) 2
        assert r["counts"][4] == 0 and r["counts"][0] == 0 and r["counts"][1] == 0   # 4 is three hops away
        assert list(AUG.augment(G.rowptr, G.colidx, [0, 1], 2, 1, seed)["halo"]) == halo[:1]
        seen.add(tuple(halo))
    assert (2, 3) in seen
    assert len(AUG.augment(G.rowptr, G.colidx, [0, 1, 2, 3, 4], 2, 3, 0)["halo"]) == 0     # no boundary, no halo


@pytest.mark.parametrize("l", [1, 2, 3])
def test_candidates_and_selection_invariants(l):
    G = _whole_graph(3000, 10.0, seed=l)
    A = _adj(G)
    part = np.arange(500, 1400)
    r = AUG.augment(G.rowptr, G.colidx, part, l, 120, seed=3)
    inside = np.zeros(G.n, dtype=bool)
    inside[part] = True
    B = r["boundary"]
    assert all(inside[B]) and all((A[b].toarray().ravel() > 0)[~inside].any() for b in B[:50])
    # Definition 2 / Property 1: every counted node is outside the partition and within l hops of the boundary
    reach = np.zeros(G.n, dtype=bool)
    front = np.zeros(G.n)
    front[B] = 1.0
    for _ in range(l):
        front = (A @ front > 0).astype(float)
        reach |= front > 0
    visited = np.nonzero(r["counts"])[0]
    assert not inside[visited].any() and reach[visited].all()
    # first batch = sum of boundary degrees; the total follows Eq. 4 on the first batch's counts
    n0 = int(np.asarray(A[B].sum()))
    assert r["n_walks"] >= n0 and len(r["walks"]) == r["n_walks"]
    # selection: distinct, outside, budget, and connected to the partition through earlier picks (no dangling node)
    halo = r["halo"]
    assert len(halo) == 120 and len(set(halo)) == 120 and not inside[halo].any()
    ok = inside.copy()
    for v in halo:
        assert (A[v].toarray().ravel() > 0)[ok].any(), v
        ok[v] = True
    # reproducible, and a different seed walks differently
    again = AUG.augment(G.rowptr, G.colidx, part, l, 120, seed=3)
    assert np.array_equal(again["halo"], halo) and again["n_walks"] == r["n_walks"]
    assert not np.array_equal(AUG.augment(G.rowptr, G.colidx, part, l, 120, seed=4)["halo"], halo)


def test_importance_converges_to_visit_probabilities():
    """Eq. 3: I(v) estimates the probability that a 2-step walk from a uniformly drawn boundary node meets v."""
    G = _whole_graph(400, 6.0, seed=5, max_degree=40)
    A = _adj(G).toarray()
    part = np.arange(0, 150)
    inside = np.zeros(G.n, dtype=bool)
    inside[part] = True
    r = AUG.augment(G.rowptr, G.colidx, part, 2, 10, seed=11, max_walks=200_000)
    B, n = r["boundary"], r["n_walks"]
    deg = A.sum(axis=1)
    P1 = A / np.maximum(deg, 1)[:, None]                                      # one uniform step
    # from boundary node b: v is met at step 1 (probability P1[b, v]) or, after a step to some u != v, at step 2;
    # without self loops P1[v, v] = 0, so the two events are disjoint and the u = v term vanishes
    exact = np.zeros(G.n)
    for b in B:
        exact += (P1[b] + P1[b] @ P1) / len(B)
    est = r["counts"] / n
    cand = ~inside
    sd = np.sqrt(np.maximum(exact * (1 - exact), 1e-12) / n)
    assert np.all(np.abs(est - exact)[cand] <= 5 * sd[cand] + 1e-9)
    assert est[cand].sum() > 0.2
