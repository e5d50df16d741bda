"""CSR-level CPU oracle (tier T1): ctypes wrapper over oracle/csr_oracle.c + numpy float64 matmuls.

TEST INFRASTRUCTURE ONLY -- called by tests, the smoke check and the benchmark's
CPU-baseline leg; never by the product path, with which it shares no code.

Same definitions and readings as oracle/gad_dense.py (see its header for the paper
citations: Eq. 7-10, Eq. 14-15 of arXiv 2110.02987), evaluated over a CSR so that it
scales to the large workloads.  The sparse product A~ T is the C routine `t1_spmm`;
dense products are numpy float64 matmuls; everything else is elementwise numpy.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csr_oracle.c")
_SO = os.path.join(_HERE, "libgad_oracle.so")
_lib = None


def build_library(force: bool = False) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _SO, "-lm"])
    return _SO


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build_library())
        _lib.t1_deviation.restype = C.c_double
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


class Graph:
    """CSR of A + I with int64 rowptr / int32 colidx, plus deg and float32 dinv."""

    def __init__(self, rowptr, colidx):
        self.rowptr = rowptr
        self.colidx = colidx
        self.n = rowptr.size - 1
        self.nnz = int(rowptr[-1])
        self.deg = np.empty(self.n, dtype=np.int32)
        self.dinv = np.empty(self.n, dtype=np.float32)
        lib().t1_degree(_p(rowptr, C.c_int64), C.c_int64(self.n), _p(self.deg, C.c_int32), _p(self.dinv, C.c_float))


def build(src, dst, n_global, local_ids, halo_ids) -> Graph:
    """Induced simple undirected graph on local ++ halo, self loops added (Algorithm 1 last step)."""
    src = np.ascontiguousarray(src, dtype=np.int64)
    dst = np.ascontiguousarray(dst, dtype=np.int64)
    local_ids = np.ascontiguousarray(local_ids, dtype=np.int64)
    halo_ids = np.ascontiguousarray(halo_ids, dtype=np.int64)
    n = local_ids.size + halo_ids.size
    rowptr = np.empty(n + 1, dtype=np.int64)
    colp = C.POINTER(C.c_int32)()
    nnz = C.c_int64(0)
    st = lib().t1_build(_p(src, C.c_int64), _p(dst, C.c_int64), C.c_int64(src.size), C.c_int64(n_global),
                        _p(local_ids, C.c_int64), C.c_int64(local_ids.size),
                        _p(halo_ids, C.c_int64), C.c_int64(halo_ids.size),
                        _p(rowptr, C.c_int64), C.byref(colp), C.byref(nnz))
    if st == -3:
        raise ValueError("id out of range")
    if st == -4:
        raise ValueError("duplicate id")
    if st != 0:
        raise MemoryError("t1_build failed")
    colidx = np.empty(nnz.value, dtype=np.int32)
    lib().t1_copy_colidx(colp, nnz, _p(colidx, C.c_int32))
    lib().t1_free(colp)
    return Graph(rowptr, colidx)


def spmm(g: Graph, T) -> np.ndarray:
    """A~ T in float64."""
    T = np.ascontiguousarray(T, dtype=np.float64)
    if T.ndim == 1:
        T = T[:, None]
    out = np.empty_like(T)
    lib().t1_spmm(_p(g.rowptr, C.c_int64), _p(g.colidx, C.c_int32), C.c_int64(g.n), C.c_int64(T.shape[1]),
                  _p(T, C.c_double), _p(out, C.c_double))
    return out


def spmm_rows(g: Graph, T32, rows, width=None) -> np.ndarray:
    """Rows `rows` of A~ T for a float32 T (leading dimension T32.shape[1]); float64 result."""
    T32 = np.ascontiguousarray(T32, dtype=np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    w = int(width or T32.shape[1])
    out = np.empty((rows.size, w), dtype=np.float64)
    lib().t1_spmm_rows_f32(_p(g.rowptr, C.c_int64), _p(g.colidx, C.c_int32), C.c_int64(w), C.c_int64(T32.shape[1]),
                           _p(T32, C.c_float), _p(rows, C.c_int64), C.c_int64(rows.size), _p(out, C.c_double))
    return out


def forward(g: Graph, X, Ws, labels, mask, c=1.0, slope=0.0):
    """Eq. 7-9.  Keeps AH[l] = A~ H_l for the backward.  sigma = ReLU (slope 0) or LeakyReLU (Eq. 7 names both).
    c: the scale of the loss, a scalar or one weight per node."""
    H = [np.asarray(X, dtype=np.float64)]
    AH, P = [], []
    L = len(Ws)
    for l in range(L):
        AH.append(spmm(g, H[l]))
        P.append(AH[l] @ np.asarray(Ws[l], dtype=np.float64))
        if l < L - 1:
            H.append(np.where(P[l] > 0, P[l], slope * P[l]))
    Z = P[-1]
    zmax = Z.max(axis=1, keepdims=True)
    e = np.exp(Z - zmax)
    se = e.sum(axis=1, keepdims=True)
    yhat = e / se
    lse = np.log(se[:, 0]) + zmax[:, 0]
    m = np.asarray(mask).astype(bool)
    if np.ndim(c) == 0:
        loss = c * np.sum((lse - Z[np.arange(Z.shape[0]), labels])[m])
    else:                                   # per-node weights c_i (e.g. the importance weights of Eq. 15 per block)
        loss = np.sum((np.asarray(c, dtype=np.float64) * (lse - Z[np.arange(Z.shape[0]), labels]))[m])
    return dict(Z=Z, loss=float(loss), H=H, P=P, AH=AH, yhat=yhat)


def backward(g: Graph, Ws, fwd, labels, mask, c=1.0, relu_on=None, slope=0.0):
    """dW_l = (A~ H_{l-1})^T G_l ;  G_{l-1} = (A~ G_l W_l^T) * [P_{l-1} > 0].

    relu_on: optional list of boolean arrays (one per hidden layer) replacing the decisions [P_l > 0].
    A caller comparing against float32 arithmetic uses it to take the decisions in that precision for
    the entries whose |P_l| lies below float32 rounding (ReLU'(0) = 0 otherwise)."""
    L = len(Ws)
    n, K = fwd["Z"].shape
    G = fwd["yhat"].copy()
    G[np.arange(n), labels] -= 1.0
    G *= (np.asarray(c, dtype=np.float64) * np.asarray(mask, dtype=np.float64))[:, None]
    dW = [None] * L
    Gs = [None] * L
    for l in range(L - 1, -1, -1):
        Gs[l] = G
        dW[l] = fwd["AH"][l].T @ G
        if l > 0:
            on = fwd["P"][l - 1] > 0 if relu_on is None else relu_on[l - 1]
            G = (spmm(g, G) @ np.asarray(Ws[l], dtype=np.float64).T) * np.where(on, 1.0, slope)
    return dW, Gs


def concat(graphs) -> Graph:
    """Block-diagonal union: the rows of graphs[k] follow those of graphs[0..k-1]; no edge joins two blocks."""
    rowptr, colidx, row_off, nnz_off = [np.zeros(1, dtype=np.int64)], [], 0, 0
    for g in graphs:
        rowptr.append(g.rowptr[1:] + nnz_off)
        colidx.append(g.colidx + np.int32(row_off))
        row_off += g.n
        nnz_off += g.nnz
    return Graph(np.concatenate(rowptr), np.concatenate(colidx).astype(np.int32))


def zeta(g: Graph, V, beta=1.0):
    """Eq. 14 (aggregate-distance reading).  Returns (zeta, S_pp, var, r_per_node)."""
    s = np.zeros(2, dtype=np.int64)
    lib().t1_degree_sums(_p(g.deg, C.c_int32), C.c_int64(g.n), _p(s, C.c_int64))
    s1, s2 = int(s[0]), int(s[1])
    spp = 0.0 if s1 == 0 else float((s1 * s1 - s2)) / float(2 * s1 * s1)   # python ints: exact numerator
    V = np.ascontiguousarray(V, dtype=np.float64)
    r = np.empty(V.shape[0], dtype=np.float64)
    var = lib().t1_deviation(_p(V, C.c_double), C.c_int64(V.shape[0]), C.c_int64(V.shape[1]), _p(r, C.c_double))
    D = float(np.sqrt(2.0 * var))
    return spp / (D + beta), spp, float(var), r


def zeta_pairs(g: Graph, V, beta=1.0):
    """Eq. 14, per-pair reading: sum_{i<j} p_i p_j / (||v_i - v_j|| + beta), p_i = deg_i / sum(deg).  O(n^2 F)."""
    s1 = int(g.deg.astype(np.int64).sum())
    if s1 == 0:
        return 0.0
    V = np.ascontiguousarray(V, dtype=np.float64)
    lib().t1_pair_sum.restype = C.c_double
    tot = lib().t1_pair_sum(_p(g.deg, C.c_int32), _p(V, C.c_double), C.c_int64(V.shape[0]), C.c_int64(V.shape[1]),
                            C.c_double(beta))
    return float(tot) / (float(s1) * float(s1))


def weighted_consensus(bufs, zetas):
    """Eq. 15."""
    z = np.asarray(zetas, dtype=np.float64)
    if z.size < 1 or not np.all(np.isfinite(z)) or np.any(z < 0) or z.sum() == 0:
        raise ValueError("bad zeta")
    w = z / z.sum()
    out = np.zeros(np.asarray(bufs[0]).shape, dtype=np.float64)
    for wi, b in zip(w, bufs):
        out += wi * np.asarray(b, dtype=np.float64)
    return out


def train_round(graphs, Xs, Ws, labels, masks, cs, zetas, eta, slope=0.0):
    """One synchronous round of Algorithm 2 with the K subgraphs as the K processors: every processor runs
    forward + backward with the same parameters (Eq. 7-10), the gradients are averaged with the importance
    weights (Eq. 15) and every processor applies W <- W - eta * grad_hat (Eq. 16 read as plain SGD).
    Returns (new weights, per-subgraph losses, averaged gradient)."""
    grads, losses = [], []
    for g, X, y, m, c in zip(graphs, Xs, labels, masks, cs):
        f = forward(g, X, Ws, y, m, c, slope)
        dW, _ = backward(g, Ws, f, y, m, c, slope=slope)
        grads.append(dW)
        losses.append(f["loss"])
    new_W, avg = [], []
    for l in range(len(Ws)):
        g_hat = weighted_consensus([gk[l] for gk in grads], zetas)
        avg.append(g_hat)
        new_W.append(np.asarray(Ws[l], dtype=np.float64) - eta * g_hat)
    return new_W, losses, avg
