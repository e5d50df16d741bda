"""The synthetic workloads at their full sizes, in the launch configuration bench.py times:
CSR bit-exact against the oracle, one whole forward + backward against the float64 CSR oracle,
plus variance importance and weighted consensus where the workload asks for them.

Each test appends progress lines to a log in the run's output folder (generation and the float64 oracle take
tens of seconds on the large graphs).
"""
import time

import numpy as np
import pytest
import torch

from oracle import gad_csr as T1
from paper_2110_02987_amd import workloads as wl
from tests.conftest import progress
from tests.test_gpu_parity import (TOL, TOL_BF16, assert_csr_equal, bf16_dev, build_both, check_step, dev, gad,  # noqa: F401
                                   rel_err)

pytestmark = pytest.mark.gpu


def _step(gad, name, bf16=False):
    cfg = wl.CONFIGS[name]
    t0 = time.time()
    progress(f"[{name}] generating graph")
    gr = wl.make_graph(cfg)
    progress(f"[{name}] graph generated in {time.time() - t0:.1f}s, {len(gr['src'])} input pairs; building (gpu + oracle)")
    g, ref = build_both(gad, gr)
    assert_csr_equal(g, ref)
    progress(f"[{name}] CSR bit-exact: n={g.n} nnz={g.nnz} max_deg={int(ref.deg.max())}; forward/backward (gpu + float64 oracle)")
    dims = cfg.dims
    X = wl.make_features(cfg.n, dims[0])
    Ws = wl.make_weights(dims)
    y = wl.make_labels(cfg.n, dims[-1])
    mask = wl.make_mask(cfg)
    f = check_step(gad, g, ref, X, Ws, y, mask, 1.0 / mask.sum(), dims, bf16=bf16)
    progress(f"[{name}] step parity ok in {time.time() - t0:.1f}s, loss={f['loss']:.6f}, bf16={bf16}")
    spmm_fixed_point(gad, g, max(dims[1:-1]), bf16)
    progress(f"[{name}] standalone SpMM fixed point ok at width {max(dims[1:-1])}")
    return cfg, g, ref, X, f


def spmm_fixed_point(gad, g, width, bf16):
    """The standalone sparse product (the launch bench.py times, at the width it times): sqrt(1 + deg) is an
    eigenvector of A~ with eigenvalue 1, so a matrix whose columns are multiples of it must come back unchanged --
    a property of the definition that needs no oracle and holds at any size."""
    d = torch.sqrt(g.deg().to(torch.float64) + 1.0)
    T = (d[:, None] * (1.0 + torch.arange(width, device="cuda", dtype=torch.float64) / width)[None, :])
    Td = T.to(torch.bfloat16 if bf16 else torch.float32).contiguous()
    out = torch.empty_like(Td)
    gad.spmm(g, Td, out, width, 1 if bf16 else 0)
    torch.cuda.synchronize()
    err = ((out.to(torch.float64) - T).abs() / T).max().item()
    assert err < (1e-2 if bf16 else 1e-5), err


def test_reddit_shaped_partition(gad):
    cfg, g, ref, X, f = _step(gad, "reddit_part")
    assert g.n == 69_000 and g.n_local == 60_000
    assert 3.0e6 < g.nnz < 3.7e6                       # ~ n * (avg degree 50) after dropping repeats
    # per-pair reading of Eq. 14 over all 2.4e9 node pairs of the partition (41-dimensional node vectors: the
    # float64 double loop of the oracle takes about ten seconds on the host cores)
    V = wl.make_features(cfg.n, 41, sub=7)
    out2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    gad.pair_importance(g, dev(V), 1.0, out2)
    z = T1.zeta_pairs(ref, V, 1.0)
    assert abs(out2[0].item() - z) <= TOL * z
    progress(f"[reddit_part] pair importance ok: {out2[0].item():.6e}")


def test_pair_importance_beyond_2_32_threads(gad):
    """800,000 nodes = 1.95e7 pair tiles, more threads than one grid dimension holds: the tile grid is folded.
    No double loop finishes at this size; two node-vector patterns with a closed form stand in (a property that
    holds at any size: every pair is counted exactly once).  Identical vectors: zeta_pair = S_pp / beta (the paper's
    worked example).  Two values a, b by the parity of the row: the like pairs contribute
    (S_even^2 - Q_even + S_odd^2 - Q_odd) / (2 beta), the unlike pairs S_even S_odd / (||a - b|| + beta), with
    S = sum of p_i and Q = sum of p_i^2 over the rows of a parity."""
    import dataclasses
    n = 800_000
    cfg = dataclasses.replace(wl.CONFIGS["tiny"], n_local=n, n_halo=0, avg_degree=4.0)
    progress("[pairs_800k] generating graph")
    g, ref = build_both(gad, wl.make_graph(cfg))
    beta = 0.25
    out2 = torch.zeros(2, dtype=torch.float64, device="cuda")
    V = np.tile(np.linspace(-1.0, 2.0, 24, dtype=np.float32), (n, 1))
    gad.pair_importance(g, dev(V), beta, out2)
    spp = T1.zeta(ref, V, beta)[1]
    assert abs(out2[1].item() - spp) <= 1e-12
    assert abs(out2[0].item() - spp / beta) <= 1e-6 * spp / beta
    progress(f"[pairs_800k] identical vectors ok: {out2[0].item():.9e}")
    a, b = V[0].copy(), V[0][::-1].copy()
    V[1::2] = b
    gad.pair_importance(g, dev(V), beta, out2)
    p = ref.deg.astype(np.float64) / float(ref.deg.sum())
    se, so, qe, qo = p[0::2].sum(), p[1::2].sum(), (p[0::2] ** 2).sum(), (p[1::2] ** 2).sum()
    d = float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)))
    exp = (se * se - qe + so * so - qo) / (2 * beta) + se * so / (d + beta)
    assert abs(out2[0].item() - exp) <= TOL * exp
    progress(f"[pairs_800k] two-value vectors ok: {out2[0].item():.9e} vs {exp:.9e}")


@pytest.mark.parametrize("name", ["reddit_part", "products_part"])
def test_partitions_in_bf16_storage(gad, name):
    """The second and third workloads with bfloat16 storage of features and activations (bf16 matrix instruction for
    the GEMMs, float32 accumulation), whole step against the float64 oracle at the bf16 tolerance."""
    _step(gad, name, bf16=True)


def test_products_shaped_partition_with_variance_and_consensus(gad):
    cfg, g, ref, X, f = _step(gad, "products_part")
    assert g.n == 690_000 and 3.2e7 < g.nnz < 3.6e7
    # variance importance on the features and on the per-node gradients of the last layer
    out3 = torch.zeros(3, dtype=torch.float64, device="cuda")
    gad.subgraph_variance(g, dev(X), 1.0, out3)
    z = T1.zeta(ref, X, 1.0)
    got = out3.cpu().numpy()
    assert abs(got[0] - z[0]) <= TOL * z[0] and abs(got[1] - z[1]) <= 1e-12 and abs(got[2] - z[2]) <= TOL * z[2]
    # 4-way weighted consensus of parameter copies, zeta from four variance calls on differently seeded vectors
    zs_gpu, zs_ref = [], []
    for k in range(cfg.consensus_k):
        V = wl.make_features(cfg.n, 47, sub=20 + k) * (1.0 + 0.5 * k)
        gad.subgraph_variance(g, dev(V), 1.0, out3)
        zs_gpu.append(out3[0].item())
        zs_ref.append(T1.zeta(ref, V, 1.0)[0])
    copies = wl.make_param_copies(cfg.dims, cfg.consensus_k)
    out = torch.empty(cfg.n_params, device="cuda")
    gad.weighted_consensus([dev(c) for c in copies], zs_gpu, out)
    assert cfg.n_params == 103_168
    assert rel_err(out.cpu().numpy(), T1.weighted_consensus(copies, zs_ref)) < TOL
    progress("[products_part] variance + consensus ok")


def test_whole_graph_on_one_gpu(gad):
    cfg, g, ref, X, f = _step(gad, "whole_graph")
    assert g.n == 2_400_000 and g.n_local == g.n and 1.1e8 < g.nnz < 1.3e8


def test_rmat22_skew_stress_bf16(gad):
    """Fifth workload at full size (R-MAT scale 22, 4.2 M nodes, bf16 storage, GCN 128-512-512-512-64).

    The float64 oracle cannot hold the whole activation chain of this workload in host memory, so parity is
    checked (a) bit-exactly for the CSR, (b) layer by layer on sampled rows and columns that the oracle computes
    one by one from the kernel's own previous-layer tensors (teacher forcing): forward rows, the loss, the seed
    gradient, backward rows, and whole columns of every dW.  Full end-to-end parity of the same model runs on the
    down-scaled R-MAT in test_gpu_parity.py."""
    name = "rmat22"
    cfg = wl.CONFIGS[name]
    dims, L, n = cfg.dims, cfg.n_layers, cfg.n
    t0 = time.time()
    progress(f"[{name}] generating graph")
    gr = wl.make_graph(cfg)
    progress(f"[{name}] {len(gr['src'])} input pairs after {time.time() - t0:.1f}s; building (gpu + oracle)")
    g, ref = build_both(gad, gr)
    del gr
    assert_csr_equal(g, ref)
    iso = int((ref.deg == 0).sum())
    progress(f"[{name}] CSR bit-exact: n={g.n} nnz={g.nnz} max_deg={int(ref.deg.max())} isolated={iso}; gpu step")
    assert g.n == 1 << 22 and g.nnz <= 272_629_760 and ref.deg.max() > 50_000 and iso > n // 10

    rng = np.random.default_rng(5)
    rows = np.unique(np.r_[rng.integers(0, n, 1500), np.argsort(ref.deg)[-40:], np.nonzero(ref.deg == 0)[0][:40]])
    Xd, X = bf16_dev(wl.make_features(n, dims[0]))
    Ws = wl.make_weights(dims)
    y = wl.make_labels(n, dims[-1])
    mask = wl.make_mask(cfg)
    c = 1.0 / mask.sum()
    ws = gad.alloc_workspace(g, dims, 1)
    Wd = [dev(w) for w in Ws]
    logits = torch.empty((n, dims[-1]), device="cuda")
    loss = torch.zeros(1, dtype=torch.float64, device="cuda")
    dW = [torch.full_like(w, float("nan")) for w in Wd]
    Gd = [torch.empty((n, dims[l + 1]), device="cuda") for l in range(L)]
    gad.gcn_forward(g, Xd, dims, Wd, dev(y), dev(mask), c, ws, logits, loss, 1)
    Hd = [None] + [torch.empty((n, dims[l]), device="cuda") for l in range(1, L)]
    for l in range(1, L):
        gad.gcn_activation(g, ws, dims, l, Hd[l], 1)
    gad.gcn_backward(g, Xd, dims, Wd, ws, dW, Gd, 1)
    torch.cuda.synchronize()
    progress(f"[{name}] gpu forward+backward done at {time.time() - t0:.1f}s; checking forward rows")

    W64 = [w.astype(np.float64) for w in Ws]
    H_prev = X                                     # float32 host copy of the kernel's layer input
    for l in range(1, L + 1):
        P = T1.spmm_rows(ref, H_prev, rows) @ W64[l - 1]
        if l < L:
            H_l = Hd[l].cpu().numpy()
            assert rel_err(H_l[rows], np.maximum(P, 0.0)) < TOL_BF16, f"H[{l}]"
            H_prev = H_l
        else:
            Z = logits.cpu().numpy()
            assert rel_err(Z[rows], P) < TOL_BF16, "logits"
        progress(f"[{name}] forward layer {l} rows ok")
    # loss and seed gradient from the kernel's logits
    Z64 = Z.astype(np.float64)
    zmax = Z64.max(axis=1)
    lse = np.log(np.exp(Z64 - zmax[:, None]).sum(axis=1)) + zmax
    exp_loss = c * np.sum((lse - Z64[np.arange(n), y])[mask == 1])
    assert abs(loss.item() - exp_loss) <= 1e-5 * abs(exp_loss)
    yhat = np.exp(Z64[rows] - lse[rows, None])
    yhat[np.arange(rows.size), y[rows]] -= 1.0
    G_last = Gd[L - 1].cpu().numpy()
    assert rel_err(G_last[rows], c * yhat * mask[rows, None]) < TOL_BF16
    del Z64
    progress(f"[{name}] loss + seed gradient ok; checking backward")

    cols_rng = np.random.default_rng(6)
    G_l = G_last
    for l in range(L - 1, -1, -1):                 # G_l = dLoss/dP_{l+1}, kernel's own values
        H_in = X if l == 0 else Hd[l].cpu().numpy()
        # whole columns of dW[l] = (A~ H_l)^T G_l = H_l^T (A~ G_l)
        got = dW[l].cpu().numpy()
        for b in cols_rng.choice(dims[l + 1], 2, replace=False):
            s = T1.spmm(ref, G_l[:, b].astype(np.float64))[:, 0]
            col = np.zeros(dims[l])
            for r0 in range(0, n, 1 << 19):
                col += H_in[r0:r0 + (1 << 19)].astype(np.float64).T @ s[r0:r0 + (1 << 19)]
            assert rel_err(got[:, b], col) < TOL_BF16, f"dW[{l}][:, {b}]"
        progress(f"[{name}] dW[{l}] columns ok")
        if l > 0:
            G_prev = Gd[l - 1].cpu().numpy()
            exp = (T1.spmm_rows(ref, G_l, rows) @ W64[l].T) * (H_in[rows] > 0)
            assert rel_err(G_prev[rows], exp) < TOL_BF16, f"G[{l - 1}]"
            G_l = G_prev
            progress(f"[{name}] backward rows of layer {l} ok")
    spmm_fixed_point(gad, g, 512, True)
    progress(f"[{name}] standalone SpMM fixed point ok at width 512; done in {time.time() - t0:.1f}s")
