"""Seeded synthetic inputs for the GAD per-processor training step.

This module only *generates inputs* (edge lists, id lists, features, weights,
labels, parameter copies).  It holds none of the method's arithmetic: no
adjacency normalisation, no propagation, no variance, no averaging.  Both the
CPU oracle's tests and the HIP path's tests draw their inputs from here so that
the two sides see bit-identical arrays.

The paper trains on Cora, Pubmed, Flickr and Reddit (Table 1).  Those datasets
are not available; the workloads below stand in for their *shapes* only
(feature width, class count, average degree, nodes per partition on 4 GPUs).

Random streams: numpy PCG64 seeded with ``SeedSequence([seed, tag])`` so every
array has a stream of its own and can be regenerated independently.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

_TAGS = {"edges": 1, "perm": 2, "extra": 3, "features": 4, "weights": 5,
         "labels": 6, "copies": 7, "orient": 8, "zeta": 9, "rows": 10}


def _rng(seed: int, tag: str, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, _TAGS[tag], sub])))


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (shape of one augmented subgraph + model)."""
    name: str
    graph: str                      # "er" | "chung_lu" | "rmat"
    n_local: int
    n_halo: int
    dims: Tuple[int, ...]           # F_0 .. F_L
    dtype: str = "f32"              # storage type of X / activations: "f32" | "bf16"
    avg_degree: float = 8.0         # er / chung_lu
    max_degree: int = 0             # chung_lu clip (0 = none)
    n_draws: int = 0                # chung_lu: number of endpoint pairs drawn (0 = n*avg/2)
    gamma: float = 2.2              # chung_lu power-law exponent
    rmat_scale: int = 0
    rmat_edge_factor: int = 0
    rmat_abc: Tuple[float, float, float] = (0.57, 0.19, 0.19)
    global_factor: int = 1          # id space = global_factor * n  (2 => half the ids are outside g')
    extra_edge_frac: float = 0.0    # fraction of extra edges with an endpoint outside g'
    consensus_k: int = 0            # >0: weighted consensus over K parameter copies
    shuffle_rows: bool = True       # rows of the subgraph in a seeded random order of the generator's node numbers

    @property
    def n(self) -> int:
        return self.n_local + self.n_halo

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1

    @property
    def n_params(self) -> int:
        return sum(self.dims[l] * self.dims[l + 1] for l in range(self.n_layers))


CONFIGS: Dict[str, Workload] = {
    # configs[0]: oracle finishes in seconds
    "tiny": Workload("tiny", "er", 4096, 0, (128, 64, 16), avg_degree=8.0),
    # configs[1]: Reddit-shaped partition (602 features, 41 classes, avg degree ~50, 1/4 of the graph)
    "reddit_part": Workload("reddit_part", "chung_lu", 60_000, 9_000, (602, 256, 41),
                            avg_degree=50.0, max_degree=20_000, global_factor=2, extra_edge_frac=0.10),
    # configs[2]: products-shaped partition; roofline target
    "products_part": Workload("products_part", "chung_lu", 600_000, 90_000, (100, 256, 256, 47),
                              avg_degree=50.0, max_degree=20_000, global_factor=2, extra_edge_frac=0.10,
                              consensus_k=4),
    # configs[3]: whole graph on one GPU (k = 1, no halo)
    "whole_graph": Workload("whole_graph", "chung_lu", 2_400_000, 0, (100, 256, 256, 47),
                            avg_degree=51.7, max_degree=50_000, n_draws=62_000_000),
    # configs[4]: skew stress
    "rmat22": Workload("rmat22", "rmat", 1 << 22, 0, (128, 512, 512, 512, 64), dtype="bf16",
                       rmat_scale=22, rmat_edge_factor=32),
    # down-scaled variants used by parity tests that need the full oracle
    "rmat16": Workload("rmat16", "rmat", 1 << 16, 0, (128, 512, 512, 512, 64), dtype="bf16",
                       rmat_scale=16, rmat_edge_factor=32),
    "rmat18": Workload("rmat18", "rmat", 1 << 18, 0, (128, 512, 512, 512, 64), dtype="bf16",
                       rmat_scale=18, rmat_edge_factor=32),
    "products_small": Workload("products_small", "chung_lu", 20_000, 3_000, (100, 256, 256, 47),
                               avg_degree=50.0, max_degree=2_000, global_factor=2, extra_edge_frac=0.10,
                               consensus_k=4),
}


# --------------------------------------------------------------------------------------
# graphs: every generator returns raw endpoint pairs over node numbers 0..n-1; duplicates,
# reversed duplicates and self loops are left in on purpose (the CSR build must remove them).
# --------------------------------------------------------------------------------------

def _pairs_er(n: int, m: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    rng = _rng(seed, "edges")
    return rng.integers(0, n, m, dtype=np.int64), rng.integers(0, n, m, dtype=np.int64)


def chung_lu_weights(n: int, avg: float, max_deg: int, gamma: float) -> np.ndarray:
    """Expected-degree sequence w_i ~ (i+1)^(-1/(gamma-1)), mean `avg`, clipped at `max_deg`."""
    w = (np.arange(n, dtype=np.float64) + 1.0) ** (-1.0 / (gamma - 1.0))
    for _ in range(8):                       # rescale / clip until the mean settles
        w *= avg / w.mean()
        if max_deg > 0:
            np.minimum(w, float(max_deg), out=w)
    return w


def _pairs_chung_lu(n: int, avg: float, max_deg: int, gamma: float, m: int, seed: int):
    w = chung_lu_weights(n, avg, max_deg, gamma)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    rng = _rng(seed, "edges")
    out = []
    for _ in range(2):
        ends = np.empty(m, dtype=np.int64)
        step = 1 << 24
        for s in range(0, m, step):          # chunked to bound temporary memory
            e = min(m, s + step)
            ends[s:e] = np.searchsorted(cdf, rng.random(e - s), side="right")
        np.minimum(ends, n - 1, out=ends)
        out.append(ends)
    return out[0], out[1]


def _pairs_rmat(scale: int, edge_factor: int, abc, seed: int):
    a, b, c = abc
    m = edge_factor << scale
    src = np.zeros(m, dtype=np.int64)
    dst = np.zeros(m, dtype=np.int64)
    rng = _rng(seed, "edges")
    for _ in range(scale):
        r = rng.random(m, dtype=np.float32)
        sbit = r >= np.float32(a + b)                               # quadrants c, d
        dbit = ((r >= np.float32(a)) & ~sbit) | (r >= np.float32(a + b + c))   # quadrants b, d
        src <<= 1
        dst <<= 1
        src |= sbit
        dst |= dbit
    return src, dst


def make_graph(cfg: Workload, seed: int = 0) -> dict:
    """Raw input of the CSR build: directed endpoint pairs in *global* ids plus the id lists.

    Returns dict(src, dst [int64, E_in], n_global, local_ids [int64], halo_ids [int64]).
    Generator node u (0 <= u < n) is global id ``perm[u]``.  Row k of the subgraph is generator node ``order[k]``,
    a seeded shuffle: the generators number their nodes in a structured way (Chung-Lu: by falling expected degree;
    R-MAT: by bit pattern), and a real partition has no such row order.  The first n_local rows are the local nodes,
    the next n_halo the replicated (halo) nodes -- a random subset, listed after the locals.
    ``shuffle_rows=False`` keeps row k = generator node k (rows sorted by expected degree for Chung-Lu).
    """
    n = cfg.n
    if cfg.graph == "er":
        m = int(round(n * cfg.avg_degree / 2))
        u, v = _pairs_er(n, m, seed)
    elif cfg.graph == "chung_lu":
        m = cfg.n_draws or int(round(n * cfg.avg_degree / 2))
        u, v = _pairs_chung_lu(n, cfg.avg_degree, cfg.max_degree, cfg.gamma, m, seed)
    elif cfg.graph == "rmat":
        assert n == 1 << cfg.rmat_scale
        u, v = _pairs_rmat(cfg.rmat_scale, cfg.rmat_edge_factor, cfg.rmat_abc, seed)
    else:
        raise ValueError(cfg.graph)

    n_global = cfg.global_factor * n
    perm = _rng(seed, "perm").permutation(n_global).astype(np.int64)
    src = perm[u]
    dst = perm[v]
    del u, v
    if cfg.extra_edge_frac > 0 and n_global > n:
        # edges that leave the subgraph (one endpoint outside) or lie fully outside: must be dropped
        rng = _rng(seed, "extra")
        k = int(len(src) * cfg.extra_edge_frac)
        inside = perm[rng.integers(0, n, k)]
        outside = perm[rng.integers(n, n_global, k)]
        k2 = k // 10
        out_a = perm[rng.integers(n, n_global, k2)]
        out_b = perm[rng.integers(n, n_global, k2)]
        src = np.concatenate([src, inside[: k // 2], outside[k // 2:], out_a])
        dst = np.concatenate([dst, outside[: k // 2], inside[k // 2:], out_b])
        order = rng.permutation(len(src))
        src = src[order]
        dst = dst[order]
    order = _rng(seed, "rows").permutation(n) if cfg.shuffle_rows else np.arange(n)
    return dict(src=np.ascontiguousarray(src), dst=np.ascontiguousarray(dst), n_global=int(n_global),
                local_ids=np.ascontiguousarray(perm[order[: cfg.n_local]]),
                halo_ids=np.ascontiguousarray(perm[order[cfg.n_local: n]]))


# --------------------------------------------------------------------------------------
# model inputs
# --------------------------------------------------------------------------------------

def make_features(n: int, f: int, seed: int = 0, sub: int = 0) -> np.ndarray:
    """X ~ N(0,1), float32, row-major [n, f]."""
    return _rng(seed, "features", sub).standard_normal((n, f), dtype=np.float32)


def make_weights(dims, seed: int = 0):
    """Glorot-uniform U(+-sqrt(6/(F_in+F_out))) float32 [F_in, F_out] per layer."""
    out = []
    for l in range(len(dims) - 1):
        lim = np.sqrt(6.0 / (dims[l] + dims[l + 1]))
        out.append(_rng(seed, "weights", l).uniform(-lim, lim, (dims[l], dims[l + 1])).astype(np.float32))
    return out


def make_labels(n: int, n_classes: int, seed: int = 0) -> np.ndarray:
    return _rng(seed, "labels").integers(0, n_classes, n, dtype=np.int32)


def make_mask(cfg: Workload) -> np.ndarray:
    """Loss mask: 1 on local rows, 0 on halo rows (halo nodes only feed aggregation)."""
    m = np.zeros(cfg.n, dtype=np.uint8)
    m[: cfg.n_local] = 1
    return m


def make_param_copies(dims, k: int, seed: int = 0, sigma: float = 0.01):
    """K flat float32 parameter vectors: the Glorot weights plus N(0, sigma^2) noise per copy."""
    base = np.concatenate([w.ravel() for w in make_weights(dims, seed)])
    return [(base + sigma * _rng(seed, "copies", i).standard_normal(base.size)).astype(np.float32)
            for i in range(k)]


def to_bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (b.astype(np.uint32) << 16).view(np.float32)


def make_planted_labels(X: np.ndarray, n_classes: int, seed: int = 0) -> np.ndarray:
    """Labels a linear map of the features can explain (argmax of X R for a seeded random R): gives the training
    loop something to learn.  Input generation only."""
    R = _rng(seed, "labels", 1).standard_normal((X.shape[1], n_classes)).astype(np.float32)
    return np.argmax(X @ R, axis=1).astype(np.int32)
