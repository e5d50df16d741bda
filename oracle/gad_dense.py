"""Definition-level CPU oracle (tier T0) for GAD's per-processor GCN step.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64, explicit dense n x n matrices; meant for n up to a few thousand.
Nothing here is shared with, imported by, or imports the HIP path.  Only tests, the
smoke check and the benchmark's CPU-baseline leg may call it.

What it computes, and where the paper defines it (arXiv 2110.02987):

* augmented subgraph g' = (v + v', e + e')            -- Algorithm 1 (last step), Algorithm 2 (Require)
* layer forward  H^(l+1) = sigma(A~ H^(l) W^(l))      -- Section 3.3, Eq. 7 (sigma = ReLU)
* prediction     y^ = softmax(A~ sigma(A~ H W1) W2)    -- Eq. 8 (no bias, no activation on the last layer)
* loss and its gradient                                -- Eq. 9, Eq. 10
* plain consensus (mean of gradients)                  -- Definition 4, Eq. 11
* variance-based importance zeta(g')                   -- Section 3.4.1, Eq. 14 and its worked example
* weighted consensus                                   -- Section 3.4.2, Eq. 15

Readings taken where the paper is silent or garbled (each is pinned by tests/test_oracle_pins.py
unless marked "parity unpinned"):

* A~ is never defined in the paper; it is the renormalised adjacency of the GCN the paper builds
  on: A~ = D~^-1/2 (A + I) D~^-1/2 with D~ = diag(1 + deg).  Degrees are those *inside* g'.
* The subgraph is the induced simple undirected graph on local ++ halo nodes: an input pair counts
  iff both ends are in the node set; direction, multiplicity and self pairs are ignored.
  (Whether halo-halo edges are kept is not stated by the paper: parity unpinned, fixed by this
  definition.)
* Eq. 9 is printed in a two-class form although Eq. 8 uses a softmax over the classes and the
  datasets are single-label; it is read as softmax cross-entropy summed over the masked nodes and
  multiplied by a caller-supplied scale c.  Eq. 10 then collapses to c*(y^ - onehot(y)) w.r.t. the logits.
* ReLU'(0) = 0.
* Eq. 14 sums only the numerator and leaves i, j free in the denominator.  The worked example
  (d = 0; printed values 3.75 > 3.61 > 3.59) forces: p_i = deg_i / sum(deg), deg without self
  loop, all unordered pairs.  The denominator is read as ONE aggregate distance of the subgraph,
  D = sqrt(2 * var), var = mean_i ||v_i - mean(v)||^2 summed over feature dimensions ("each dimension
  separately"), which equals the root-mean-square Euclidean distance over all ordered pairs.
  zeta = S_pp / (D + beta).  (The choice aggregate-vs-per-pair distance is parity unpinned: the
  paper's only example has d = 0, where both agree.)
  The per-pair reading, sum_{i<j} p_i p_j / (||v_i - v_j|| + beta), is `zeta_pairs`.
* An edgeless subgraph (sum(deg) = 0) gets S_pp = 0 and zeta = 0 (convention; parity unpinned).
* Eq. 15 is printed with a spurious outer sum; read as sum_i zeta_i B_i / sum_j zeta_j.
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------- graph

def relabel(local_ids, halo_ids, n_global):
    """Global id -> row number (local nodes first, then halo nodes, in the given order); -1 = absent."""
    ids = np.concatenate([np.asarray(local_ids, dtype=np.int64), np.asarray(halo_ids, dtype=np.int64)])
    if ids.size and (ids.min() < 0 or ids.max() >= n_global):
        raise ValueError("id out of range")
    if np.unique(ids).size != ids.size:
        raise ValueError("duplicate id")
    lut = np.full(n_global, -1, dtype=np.int64)
    lut[ids] = np.arange(ids.size)
    return lut, ids.size


def adjacency_dense(src, dst, n_global, local_ids, halo_ids):
    """A in {0,1}^(n x n): symmetric, zero diagonal, induced on local ++ halo (Algorithm 1, last step)."""
    lut, n = relabel(local_ids, halo_ids, n_global)
    r = lut[np.asarray(src, dtype=np.int64)]
    c = lut[np.asarray(dst, dtype=np.int64)]
    keep = (r >= 0) & (c >= 0) & (r != c)
    A = np.zeros((n, n), dtype=np.float64)
    A[r[keep], c[keep]] = 1.0
    A[c[keep], r[keep]] = 1.0
    return A


def degrees(A):
    """deg_i = sum_j A_ij (no self loop)."""
    return A.sum(axis=1).astype(np.int64)


def normalized_adjacency(A):
    """A~ = D~^-1/2 (A + I) D~^-1/2, D~ = diag(1 + deg)   (A~ of Eq. 7)."""
    n = A.shape[0]
    dt = 1.0 + A.sum(axis=1)
    s = 1.0 / np.sqrt(dt)
    return s[:, None] * (A + np.eye(n)) * s[None, :]


def csr_of(A):
    """CSR of the pattern of A + I: rows in node order, columns strictly ascending."""
    n = A.shape[0]
    P = (A + np.eye(n)) > 0
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(P.sum(axis=1))
    colidx = np.nonzero(P)[1].astype(np.int32)      # row-major scan => ascending inside each row
    return rowptr, colidx


# ----------------------------------------------------------------------------- GCN step

def forward(At, X, Ws, labels, mask, c=1.0, slope=0.0):
    """Eq. 7-9.  Returns dict(Z, loss, H=[H_0..H_{L-1}], P=[P_1..P_L], yhat)."""
    H = [np.asarray(X, dtype=np.float64)]
    P = []
    L = len(Ws)
    for l in range(L):
        p = At @ H[l] @ np.asarray(Ws[l], dtype=np.float64)        # Eq. 7 argument
        P.append(p)
        if l < L - 1:
            H.append(np.where(p > 0, p, slope * p))                # sigma = ReLU (slope 0) or LeakyReLU
    Z = P[-1]
    zmax = Z.max(axis=1, keepdims=True)
    e = np.exp(Z - zmax)
    yhat = e / e.sum(axis=1, keepdims=True)                         # Eq. 8
    lse = np.log(e.sum(axis=1)) + zmax[:, 0]
    m = np.asarray(mask).astype(bool)
    idx = np.arange(Z.shape[0])
    if np.ndim(c) == 0:
        loss = c * np.sum((lse - Z[idx, labels])[m])                # Eq. 9 read as softmax-CE (sum)
    else:                                                           # per-node weights c_i
        loss = np.sum((np.asarray(c, dtype=np.float64) * (lse - Z[idx, labels]))[m])
    return dict(Z=Z, loss=float(loss), H=H, P=P, yhat=yhat)


def backward(At, Ws, fwd, labels, mask, c=1.0, relu_on=None, slope=0.0):
    """Chain rule of Eq. 7-10.  Returns (dW list, G list with G[l] = dLoss/dP_{l+1}).

    relu_on: optional list of boolean arrays (one per hidden layer) replacing the decisions [P_l > 0];
    used by callers that must take the decisions with |P_l| below float32 rounding in float32."""
    L = len(Ws)
    n, C = fwd["Z"].shape
    onehot = np.zeros((n, C))
    onehot[np.arange(n), labels] = 1.0
    cm = np.asarray(c, dtype=np.float64) * np.asarray(mask, dtype=np.float64)      # scalar or per-node weight
    G = (fwd["yhat"] - onehot) * (cm[:, None] if np.ndim(cm) else cm)                # Eq. 10 w.r.t. logits
    dW = [None] * L
    Gs = [None] * L
    for l in range(L - 1, -1, -1):
        Gs[l] = G
        dW[l] = (At @ fwd["H"][l]).T @ G
        if l > 0:
            on = fwd["P"][l - 1] > 0 if relu_on is None else relu_on[l - 1]
            G = (At.T @ G @ np.asarray(Ws[l], dtype=np.float64).T) * np.where(on, 1.0, slope)
    return dW, Gs


# ----------------------------------------------------------------------------- GAD-Optimizer

def pair_probability_sum(deg):
    """S_pp = sum over unordered pairs i<j of p_i p_j, p_i = deg_i / sum(deg)   (numerator of Eq. 14)."""
    deg = np.asarray(deg, dtype=np.float64)
    s = deg.sum()
    if s == 0:
        return 0.0
    p = deg / s
    tot = 0.0
    n = p.size
    if n <= 2048:                           # literal double sum
        for i in range(n):
            tot += p[i] * p[i + 1:].sum()
        return float(tot)
    return float((1.0 - np.sum(p * p)) / 2.0)


def aggregate_distance(V):
    """(var, D): var = mean_i ||v_i - vbar||^2 (summed over dimensions); D = sqrt(2 var)."""
    V = np.asarray(V, dtype=np.float64)
    vbar = V.mean(axis=0)
    r = ((V - vbar) ** 2).sum(axis=1)
    var = r.mean()
    return float(var), float(np.sqrt(2.0 * var)), r


def zeta(deg, V, beta=1.0):
    """Eq. 14 under the reading in the header.  Returns (zeta, S_pp, var, r_per_node)."""
    spp = pair_probability_sum(deg)
    var, D, r = aggregate_distance(V)
    return spp / (D + beta), spp, var, r


def zeta_pairs(deg, V, beta=1.0):
    """Eq. 14 under its other reading: the distance stays inside the sum, one term per unordered pair,
        zeta_pair = sum_{i<j} p_i p_j / (||v_i - v_j||_2 + beta),   p_i = deg_i / sum(deg).
    (The paper prints the sum over the numerator only and leaves i, j free in the denominator; with identical
    node vectors, as in its worked example, this and the aggregate reading of `zeta` coincide.)
    Literal double loop over the pairs, float64; O(n^2 F).  An edgeless subgraph gives 0."""
    deg = np.asarray(deg, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    s = deg.sum()
    if s == 0:
        return 0.0
    p = deg / s
    tot = 0.0
    for i in range(p.size - 1):
        d = np.sqrt(((V[i + 1:] - V[i]) ** 2).sum(axis=1))
        tot += p[i] * float(np.sum(p[i + 1:] / (d + beta)))
    return float(tot)


def weighted_consensus(bufs, zetas):
    """Eq. 15: sum_i zeta_i B_i / sum_j zeta_j."""
    z = np.asarray(zetas, dtype=np.float64)
    if z.size < 1 or not np.all(np.isfinite(z)) or np.any(z < 0) or z.sum() == 0:
        raise ValueError("bad zeta")
    w = z / z.sum()
    out = np.zeros_like(np.asarray(bufs[0], dtype=np.float64))
    for wi, b in zip(w, bufs):
        out += wi * np.asarray(b, dtype=np.float64)
    return out


def plain_consensus(bufs):
    """Definition 4 / Eq. 11: arithmetic mean."""
    return sum(np.asarray(b, dtype=np.float64) for b in bufs) / len(bufs)
