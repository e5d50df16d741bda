"""Importance-based augmentation (Algorithm 1) through the C ABI against the CPU oracle: the chosen replication
nodes, their order and the number of walks must match exactly (integer work; both sides implement the same
counter-based generator).  Then the whole load-time chain: augment -> build the augmented subgraph -> one GCN step."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import gad_augment as AUG
from oracle import gad_csr as T1
from paper_2110_02987_amd import workloads as wl
from tests.test_gpu_parity import assert_csr_equal, check_step, dev, gad  # noqa: F401

pytestmark = pytest.mark.gpu


def _whole_graph(gad, n, avg, seed=0, max_degree=300, graph="chung_lu"):
    cfg = dataclasses.replace(wl.CONFIGS["products_small"], n_local=n, n_halo=0, global_factor=1, extra_edge_frac=0.0,
                              max_degree=max_degree, avg_degree=avg, graph=graph)
    gr = wl.make_graph(cfg, seed=seed)
    gr["local_ids"], gr["halo_ids"] = np.arange(n, dtype=np.int64), np.zeros(0, dtype=np.int64)
    G = gad.build_subgraph(dev(gr["src"]), dev(gr["dst"]), gr["n_global"], dev(gr["local_ids"]), dev(gr["halo_ids"]))
    ref = T1.build(**gr)
    assert_csr_equal(G, ref)
    return gr, G, ref


@pytest.mark.parametrize("n,avg,l,part,budget,seed", [
    (3000, 10.0, 2, (500, 1400), 120, 3), (3000, 10.0, 1, (0, 700), 50, 1), (3000, 10.0, 3, (2000, 3000), 400, 9),
    (20_000, 25.0, 2, (0, 5000), 750, 2), (20_000, 25.0, 3, (7000, 9000), 10_000, 5), (500, 3.0, 4, (10, 40), 25, 0)])
def test_augment_matches_oracle(gad, n, avg, l, part, budget, seed):
    _, G, ref = _whole_graph(gad, n, avg, seed=seed)
    rng = np.random.default_rng(seed)
    rows = rng.permutation(np.arange(part[0], part[1])).astype(np.int64)      # the order of the list is part of the input
    exp = AUG.augment(ref.rowptr, ref.colidx, rows, l, budget, seed)
    halo, n_walks = gad.augment_subgraph(G, dev(rows), l, budget, seed)
    assert n_walks == exp["n_walks"]
    assert np.array_equal(halo.cpu().numpy(), exp["halo"])
    assert len(exp["halo"]) > 0
    # a cap on the walks below what Eq. 4 asks for is honoured identically
    cap = max(1, exp["n_walks"] // 3)
    exp2 = AUG.augment(ref.rowptr, ref.colidx, rows, l, budget, seed, max_walks=cap)
    halo2, n2 = gad.augment_subgraph(G, dev(rows), l, budget, seed, max_walks=cap)
    assert n2 == exp2["n_walks"] == cap and np.array_equal(halo2.cpu().numpy(), exp2["halo"])


@pytest.mark.parametrize("n_part", [601, 600, 130])
def test_augment_with_a_hub_row_inside_the_partition(gad, n_part):
    """A hub of 600 neighbours (its row spans several 128-entry chunks) on top of a ring: with rows 0..600 in the
    partition the hub is interior, with rows 0..599 its last chunk holds the one outside neighbour, with rows 0..129
    every chunk but the first does."""
    n = 1000
    hub = np.arange(1, 601, dtype=np.int64)
    ring = np.arange(1, n, dtype=np.int64)                       # the ring leaves the hub (node 0) out
    gr = dict(src=np.concatenate([np.zeros(600, dtype=np.int64), ring]), dst=np.concatenate([hub, ring % (n - 1) + 1]),
              n_global=n, local_ids=np.arange(n, dtype=np.int64), halo_ids=np.zeros(0, dtype=np.int64))
    G = gad.build_subgraph(dev(gr["src"]), dev(gr["dst"]), n, dev(gr["local_ids"]), dev(gr["halo_ids"]))
    ref = T1.build(**gr)
    assert_csr_equal(G, ref)
    rows = np.arange(n_part, dtype=np.int64)
    assert (0 in AUG.boundary(ref.rowptr, ref.colidx, rows)) == (n_part != 601)
    for seed in (0, 1):
        exp = AUG.augment(ref.rowptr, ref.colidx, rows, 3, 40, seed)
        halo, n_walks = gad.augment_subgraph(G, dev(rows), 3, 40, seed)
        assert n_walks == exp["n_walks"] and np.array_equal(halo.cpu().numpy(), exp["halo"])


def test_augment_degenerate_and_errors(gad):
    _, G, ref = _whole_graph(gad, 400, 4.0, seed=2)
    everything = torch.arange(400, dtype=torch.int64, device="cuda")
    halo, n_walks = gad.augment_subgraph(G, everything, 2, 10, 0)            # no boundary: nothing to replicate
    assert halo.numel() == 0 and n_walks == 0
    part = torch.arange(0, 100, dtype=torch.int64, device="cuda")
    halo, _ = gad.augment_subgraph(G, part, 2, 0, 0)                          # zero budget
    assert halo.numel() == 0
    for bad, status in ((torch.tensor([1, 2, 2], device="cuda"), -4), (torch.tensor([1, 400], device="cuda"), -3),
                        (torch.tensor([-1], device="cuda"), -3)):
        with pytest.raises(gad.GadError) as e:
            gad.augment_subgraph(G, bad.to(torch.int64), 2, 5, 0)
        assert e.value.status == status
    with pytest.raises(gad.GadError) as e:
        gad.augment_subgraph(G, part, 17, 5, 0)
    assert e.value.status == -2
    halo, _ = gad.augment_subgraph(G, part, 2, 5, 0)                          # still works after the errors
    assert np.array_equal(halo.cpu().numpy(), AUG.augment(ref.rowptr, ref.colidx, np.arange(100), 2, 5, 0)["halo"])


def test_partition_augment_build_train(gad):
    """The load-time chain of the paper for one processor: partition (here: a contiguous id range), augmentation by
    Algorithm 1 with the budget of Eq. 5 / Eq. 6, the augmented subgraph's CSR, and one GCN step on it."""
    n = 12_000
    gr, G, ref = _whole_graph(gad, n, 16.0, seed=4)
    part = np.arange(3000, 6000, dtype=np.int64)
    inside = np.zeros(n, dtype=bool)
    inside[part] = True
    A_rows = np.repeat(np.arange(n), np.diff(ref.rowptr))
    e_inside = int(((inside[A_rows] & inside[ref.colidx]).sum() - len(part)) // 2)       # edges of g_i (no self loops)
    budget = 5 * AUG.replica_budget(len(part), e_inside, n)                                 # alpha = 0.05
    assert budget > 100
    dims = (16, 24, 5)
    halo, n_walks = gad.augment_subgraph(G, dev(part), len(dims) - 1, budget, 77)
    exp = AUG.augment(ref.rowptr, ref.colidx, part, len(dims) - 1, budget, 77)
    assert np.array_equal(halo.cpu().numpy(), exp["halo"]) and halo.numel() == budget
    sub = dict(src=gr["src"], dst=gr["dst"], n_global=n, local_ids=part, halo_ids=exp["halo"])
    g = gad.build_subgraph(dev(sub["src"]), dev(sub["dst"]), n, dev(part), halo)
    sref = T1.build(**sub)
    assert_csr_equal(g, sref)
    assert (sref.deg[len(part):] > 0).all()                                 # every replica hangs on the subgraph
    X = wl.make_features(g.n, dims[0])
    Ws = wl.make_weights(dims)
    y = wl.make_labels(g.n, dims[-1])
    mask = np.r_[np.ones(len(part), dtype=np.uint8), np.zeros(budget, dtype=np.uint8)]
    check_step(gad, g, sref, X, Ws, y, mask, 1.0 / mask.sum(), dims)
