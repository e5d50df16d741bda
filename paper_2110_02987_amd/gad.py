"""Thin ctypes binding over libgad.so (the C ABI declared in include/gad.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch is
used for device memory (`torch.Tensor.data_ptr()`) and for the current HIP stream, nothing else.
There is no fallback: if libgad.so is missing or a call fails, a GadError / OSError is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgad.so")

F32, BF16 = 0, 1
SYMBOLS = ["gad_last_error", "gad_build_subgraph", "gad_graph_info", "gad_graph_destroy", "gad_graph_concat", "gad_augment_subgraph",
           "gad_gcn_workspace_bytes", "gad_workspace_forget", "gad_gcn_forward", "gad_gcn_forward_cached", "gad_gcn_backward", "gad_gcn_layer_events", "gad_gcn_activation", "gad_spmm_workspace_bytes", "gad_spmm",
           "gad_gemm_workspace_bytes", "gad_gemm_w", "gad_gemm_tn",
           "gad_subgraph_variance", "gad_subgraph_variance_static", "gad_pair_importance_workspace_bytes", "gad_pair_importance",
           "gad_weighted_consensus", "gad_consensus_update", "gad_train_round", "gad_train_round_batched"]

_lib = None
_hip = None


class GadError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"libgad status {status}: {msg}")
        self.status = status


def lib() -> C.CDLL:
    """Load libgad.so (built in-tree by `python -m paper_2110_02987_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError(f"{LIB_PATH} not found: build it with `python -m paper_2110_02987_amd.build`")
        _lib = C.CDLL(LIB_PATH)
        _lib.gad_last_error.restype = C.c_char_p
        for name in SYMBOLS[1:]:
            getattr(_lib, name).restype = C.c_int
    return _lib


def _check(st: int) -> None:
    if st != 0:
        raise GadError(st, lib().gad_last_error().decode())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str) -> torch.Tensor:
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous {dtype} device tensor")
    return t


def _memcpy_d2d(dst: torch.Tensor, src_ptr: int, nbytes: int) -> None:
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
    if nbytes:
        rc = _hip.hipMemcpy(C.c_void_p(dst.data_ptr()), C.c_void_p(src_ptr), C.c_size_t(nbytes), C.c_int(3))
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed with {rc}")


class Graph:
    """Owner of a gad_graph handle."""

    def __init__(self, handle: C.c_void_p):
        self.handle = handle
        n, nl, nnz = C.c_int64(), C.c_int64(), C.c_int64()
        self._rowptr, self._colidx, self._deg, self._dinv = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
        _check(lib().gad_graph_info(handle, C.byref(n), C.byref(nl), C.byref(nnz), C.byref(self._rowptr),
                                    C.byref(self._colidx), C.byref(self._deg), C.byref(self._dinv)))
        self.n, self.n_local, self.nnz = n.value, nl.value, nnz.value

    def _copy(self, ptr, count, dtype):
        out = torch.empty(count, dtype=dtype, device="cuda")
        torch.cuda.synchronize()
        _memcpy_d2d(out, ptr.value, out.numel() * out.element_size())
        return out

    def rowptr(self): return self._copy(self._rowptr, self.n + 1, torch.int64)
    def colidx(self): return self._copy(self._colidx, self.nnz, torch.int32)
    def deg(self): return self._copy(self._deg, self.n, torch.int32)
    def dinv(self): return self._copy(self._dinv, self.n, torch.float32)

    def destroy(self):
        if self.handle:
            _check(lib().gad_graph_destroy(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def build_subgraph(src: torch.Tensor, dst: torch.Tensor, n_global: int, local_ids: torch.Tensor,
                   halo_ids: torch.Tensor) -> Graph:
    for name, t in (("src", src), ("dst", dst), ("local_ids", local_ids), ("halo_ids", halo_ids)):
        _dev(t, torch.int64, name)
    if src.numel() != dst.numel():
        raise ValueError("src and dst differ in length")
    h = C.c_void_p()
    _check(lib().gad_build_subgraph(_ptr(src if src.numel() else None), _ptr(dst if dst.numel() else None),
                                    C.c_int64(src.numel()), C.c_int64(n_global),
                                    _ptr(local_ids if local_ids.numel() else None), C.c_int64(local_ids.numel()),
                                    _ptr(halo_ids if halo_ids.numel() else None), C.c_int64(halo_ids.numel()),
                                    _stream(), C.byref(h)))
    return Graph(h)


def augment_subgraph(G: Graph, part_rows: torch.Tensor, walk_len: int, budget: int, seed: int,
                     max_walks: int = 1 << 22):
    """Replication nodes of one partition (Algorithm 1).  Returns (rows of G in selection order, number of walks)."""
    _dev(part_rows, torch.int64, "part_rows")
    out = torch.empty(max(budget, 1), dtype=torch.int64, device="cuda")
    n_halo, n_walks = C.c_int64(), C.c_int64()
    _check(lib().gad_augment_subgraph(G.handle, _ptr(part_rows), C.c_int64(part_rows.numel()), C.c_int32(walk_len),
                                      C.c_int64(budget), C.c_uint64(seed), C.c_int64(max_walks), _ptr(out),
                                      C.byref(n_halo), C.byref(n_walks), _stream()))
    return out[: n_halo.value], n_walks.value


def graph_concat(graphs: List[Graph]) -> Graph:
    """Block-diagonal union of the graphs (rows of graphs[k] follow those of graphs[0..k-1])."""
    gh = (C.c_void_p * len(graphs))(*[g.handle.value for g in graphs])
    h = C.c_void_p()
    _check(lib().gad_graph_concat(gh, C.c_int(len(graphs)), _stream(), C.byref(h)))
    return Graph(h)


def _dims(dims: Sequence[int]):
    return (C.c_int32 * len(dims))(*dims)


def _ptr_array(ts: Sequence[torch.Tensor]):
    return (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])


def gcn_workspace_bytes(g: Graph, dims: Sequence[int], dtype: int = F32) -> int:
    b = C.c_size_t()
    _check(lib().gad_gcn_workspace_bytes(g.handle, C.c_int(len(dims) - 1), _dims(dims), C.c_int(dtype), C.byref(b)))
    return b.value


def alloc_workspace(g: Graph, dims: Sequence[int], dtype: int = F32) -> torch.Tensor:
    return torch.empty(gcn_workspace_bytes(g, dims, dtype), dtype=torch.uint8, device="cuda")


def workspace_forget(workspace: torch.Tensor) -> None:
    """Call before the memory of a workspace is freed or reused for anything else."""
    _check(lib().gad_workspace_forget(_ptr(workspace)))


def gcn_forward(g: Graph, X: torch.Tensor, dims: Sequence[int], W: List[torch.Tensor], labels: torch.Tensor,
                mask: Optional[torch.Tensor], loss_scale: float, workspace: torch.Tensor,
                logits_out: Optional[torch.Tensor] = None, loss_out: Optional[torch.Tensor] = None,
                dtype: int = F32, negative_slope: float = 0.0, row_scale: Optional[torch.Tensor] = None,
                x_unchanged: bool = False) -> None:
    """x_unchanged: the caller vouches that X holds what it held at the last forward on this workspace
    (gad_gcn_forward_cached: the first layer's aggregate is then reused)."""
    _dev(X, torch.float32 if dtype == F32 else torch.bfloat16, "X")
    _dev(labels, torch.int32, "labels")
    if mask is not None:
        _dev(mask, torch.uint8, "mask")
    for w in W:
        _dev(w, torch.float32, "W")
    if logits_out is not None:
        _dev(logits_out, torch.float32, "logits_out")
    if loss_out is not None:
        _dev(loss_out, torch.float64, "loss_out")
    if row_scale is not None:
        _dev(row_scale, torch.float32, "row_scale")
    fn = lib().gad_gcn_forward_cached if x_unchanged else lib().gad_gcn_forward
    _check(fn(g.handle, _ptr(X), C.c_int(dtype), C.c_int(len(dims) - 1), _dims(dims), _ptr_array(W),
                                 _ptr(labels), _ptr(mask), C.c_float(loss_scale), _ptr(row_scale), C.c_float(negative_slope), _ptr(workspace),
                                 C.c_size_t(workspace.numel()), _ptr(logits_out), _ptr(loss_out), _stream()))


def gcn_backward(g: Graph, X: torch.Tensor, dims: Sequence[int], W: List[torch.Tensor], workspace: torch.Tensor,
                 dW: List[torch.Tensor], G_out: Optional[List[Optional[torch.Tensor]]] = None, dtype: int = F32,
                 negative_slope: float = 0.0) -> None:
    for w in dW:
        _dev(w, torch.float32, "dW")
    gp = None
    if G_out is not None:
        gp = (C.c_void_p * len(G_out))(*[0 if t is None else _dev(t, torch.float32, "G_out").data_ptr() for t in G_out])
    _check(lib().gad_gcn_backward(g.handle, _ptr(X), C.c_int(dtype), C.c_int(len(dims) - 1), _dims(dims), _ptr_array(W),
                                  C.c_float(negative_slope), _ptr(workspace), C.c_size_t(workspace.numel()), _ptr_array(dW),
                                  gp, _stream()))


def gcn_layer_events(events: Sequence[int]) -> None:
    """events: hipEvent_t handles (integers) for the layer boundaries of this thread's passes; empty = off."""
    arr = (C.c_void_p * max(len(events), 1))(*events)
    _check(lib().gad_gcn_layer_events(arr, C.c_int(len(events))))


def gcn_activation(g: Graph, workspace: torch.Tensor, dims: Sequence[int], layer: int, out: torch.Tensor,
                   dtype: int = F32) -> None:
    _dev(out, torch.float32, "out")
    _check(lib().gad_gcn_activation(g.handle, _ptr(workspace), C.c_size_t(workspace.numel()), C.c_int(len(dims) - 1),
                                    _dims(dims), C.c_int(dtype), C.c_int(layer), _ptr(out), _stream()))


def spmm_workspace(g: Graph, width: int) -> Optional[torch.Tensor]:
    b = C.c_size_t()
    _check(lib().gad_spmm_workspace_bytes(g.handle, C.c_int32(width), C.byref(b)))
    return torch.empty(b.value, dtype=torch.uint8, device="cuda") if b.value else None


def spmm(g: Graph, T: torch.Tensor, out: torch.Tensor, width: Optional[int] = None, dtype: int = F32,
         workspace: Optional[torch.Tensor] = None) -> None:
    """out = A~ T for 2-D row-major T, out (leading dimensions = their second sizes)."""
    width = int(width if width is not None else T.shape[1])
    ws = workspace if workspace is not None else spmm_workspace(g, width)
    _check(lib().gad_spmm(g.handle, _ptr(T), C.c_int64(T.shape[1]), _ptr(out), C.c_int64(out.shape[1]),
                          C.c_int32(width), C.c_int(dtype), _ptr(ws), C.c_size_t(0 if ws is None else ws.numel()),
                          _stream()))


def gemm_workspace(M: int, K: int, N: int) -> torch.Tensor:
    b = C.c_size_t()
    _check(lib().gad_gemm_workspace_bytes(C.c_int64(M), C.c_int32(K), C.c_int32(N), C.byref(b)))
    return torch.empty(max(b.value, 256), dtype=torch.uint8, device="cuda")


def gemm_w(A: torch.Tensor, W: torch.Tensor, out: torch.Tensor, transpose_w: bool = False,
           workspace: Optional[torch.Tensor] = None, K: Optional[int] = None) -> None:
    """out = A[:, :K] W  (or A[:, :K] W^T); A and out are 2-D row-major float32 or bfloat16 (the same type), W float32."""
    dtype = F32 if A.dtype == torch.float32 else BF16
    _dev(A, torch.float32 if dtype == F32 else torch.bfloat16, "A")
    _dev(out, A.dtype, "out")
    _dev(W, torch.float32, "W")
    k = W.shape[1] if transpose_w else W.shape[0]
    n = W.shape[0] if transpose_w else W.shape[1]
    ws = workspace if workspace is not None else gemm_workspace(A.shape[0], k, n)
    _check(lib().gad_gemm_w(_ptr(A), C.c_int64(A.shape[1]), _ptr(W), C.c_int32(W.shape[0]), C.c_int32(W.shape[1]),
                            C.c_int(1 if transpose_w else 0), _ptr(out), C.c_int64(out.shape[1]), C.c_int64(A.shape[0]),
                            C.c_int(dtype), _ptr(ws), C.c_size_t(ws.numel()), _stream()))


def gemm_tn(A: torch.Tensor, G: torch.Tensor, out: torch.Tensor, K: Optional[int] = None, N: Optional[int] = None,
            workspace: Optional[torch.Tensor] = None) -> None:
    """out[K x N] (float32) = A[:, :K]^T G[:, :N]; A and G are 2-D row-major float32 or bfloat16 (the same type)."""
    dtype = F32 if A.dtype == torch.float32 else BF16
    _dev(A, torch.float32 if dtype == F32 else torch.bfloat16, "A")
    _dev(G, A.dtype, "G")
    _dev(out, torch.float32, "out")
    k = int(K if K is not None else A.shape[1])
    n = int(N if N is not None else G.shape[1])
    ws = workspace if workspace is not None else gemm_workspace(A.shape[0], k, n)
    _check(lib().gad_gemm_tn(_ptr(A), C.c_int64(A.shape[1]), _ptr(G), C.c_int64(G.shape[1]), _ptr(out),
                             C.c_int64(A.shape[0]), C.c_int32(k), C.c_int32(n), C.c_int(dtype), _ptr(ws),
                             C.c_size_t(ws.numel()), _stream()))


def subgraph_variance(g: Graph, V: torch.Tensor, beta: float, out3: torch.Tensor,
                      per_node_out: Optional[torch.Tensor] = None) -> None:
    dtype = F32 if V.dtype == torch.float32 else BF16
    _dev(V, torch.float32 if dtype == F32 else torch.bfloat16, "V")
    _dev(out3, torch.float64, "out3")
    _check(lib().gad_subgraph_variance(g.handle, _ptr(V), C.c_int32(V.shape[1]), C.c_int(dtype), C.c_double(beta),
                                       _ptr(out3), _ptr(per_node_out), _stream()))


def subgraph_variance_static(g: Graph, V: torch.Tensor, beta: float, out3: torch.Tensor,
                             per_node_out: Optional[torch.Tensor] = None) -> None:
    """subgraph_variance with the reduction buffer in the library's fixed device array (allocates nothing)."""
    dtype = F32 if V.dtype == torch.float32 else BF16
    _dev(V, torch.float32 if dtype == F32 else torch.bfloat16, "V")
    _dev(out3, torch.float64, "out3")
    _check(lib().gad_subgraph_variance_static(g.handle, _ptr(V), C.c_int32(V.shape[1]), C.c_int(dtype),
                                              C.c_double(beta), _ptr(out3), _ptr(per_node_out), _stream()))


def pair_importance(g: Graph, V: torch.Tensor, beta: float, out2: torch.Tensor,
                    workspace: Optional[torch.Tensor] = None) -> None:
    """out2 = (zeta_pair, S_pp): Eq. 14 with the distance inside the pair sum.  O(n^2 F)."""
    dtype = F32 if V.dtype == torch.float32 else BF16
    _dev(V, torch.float32 if dtype == F32 else torch.bfloat16, "V")
    _dev(out2, torch.float64, "out2")
    if workspace is None:
        b = C.c_size_t()
        _check(lib().gad_pair_importance_workspace_bytes(g.handle, C.c_int32(V.shape[1]), C.byref(b)))
        workspace = torch.empty(b.value, dtype=torch.uint8, device="cuda")
    _check(lib().gad_pair_importance(g.handle, _ptr(V), C.c_int32(V.shape[1]), C.c_int(dtype), C.c_double(beta),
                                     _ptr(out2), _ptr(workspace), C.c_size_t(workspace.numel()), _stream()))


def weighted_consensus(bufs: List[torch.Tensor], zeta: Sequence[float], out: torch.Tensor) -> None:
    for b in bufs:
        _dev(b, torch.float32, "bufs")
    z = (C.c_double * len(zeta))(*[float(v) for v in zeta])
    _check(lib().gad_weighted_consensus(_ptr_array(bufs), C.c_int(len(bufs)), z, C.c_int64(out.numel()), _ptr(out),
                                        _stream()))


def consensus_update(grads: List[torch.Tensor], zeta: Sequence[float], eta: float, params: torch.Tensor,
                     avg_out: Optional[torch.Tensor] = None) -> None:
    for b in grads:
        _dev(b, torch.float32, "grads")
    _dev(params, torch.float32, "params")
    z = (C.c_double * len(zeta))(*[float(v) for v in zeta])
    _check(lib().gad_consensus_update(_ptr_array(grads), C.c_int(len(grads)), z, C.c_int64(params.numel()),
                                      C.c_float(eta), _ptr(params), _ptr(avg_out), _stream()))


def train_round(graphs: List[Graph], X: List[torch.Tensor], dims: Sequence[int], params: torch.Tensor,
                labels: List[torch.Tensor], masks: Optional[List[Optional[torch.Tensor]]], loss_scales: Sequence[float],
                workspaces: List[torch.Tensor], grads: torch.Tensor, zeta: Sequence[float], eta: float,
                losses: Optional[torch.Tensor] = None, dtype: int = F32, negative_slope: float = 0.0,
                x_unchanged: bool = False) -> None:
    K = len(graphs)
    _dev(params, torch.float32, "params")
    _dev(grads, torch.float32, "grads")
    if grads.numel() < K * params.numel():
        raise ValueError("grads must hold K * n_params floats")
    gh = (C.c_void_p * K)(*[g.handle.value for g in graphs])
    mk = None if masks is None else (C.c_void_p * K)(*[0 if m is None else m.data_ptr() for m in masks])
    ls = (C.c_float * K)(*[float(v) for v in loss_scales])
    wb = (C.c_size_t * K)(*[w.numel() for w in workspaces])
    z = (C.c_double * K)(*[float(v) for v in zeta])
    _check(lib().gad_train_round(C.c_int(K), gh, _ptr_array(X), C.c_int(dtype), C.c_int(len(dims) - 1), _dims(dims),
                                 _ptr(params), _ptr_array(labels), mk, ls, C.c_float(negative_slope), _ptr_array(workspaces), wb,
                                 _ptr(grads), z,
                                 C.c_float(eta), _ptr(losses), C.c_int(1 if x_unchanged else 0), _stream()))


def train_round_batched(g: Graph, X: torch.Tensor, dims: Sequence[int], params: torch.Tensor, labels: torch.Tensor,
                        mask: Optional[torch.Tensor], row_scale: torch.Tensor, workspace: torch.Tensor, grad: torch.Tensor,
                        eta: float, loss: Optional[torch.Tensor] = None, dtype: int = F32,
                        negative_slope: float = 0.0, x_unchanged: bool = False) -> None:
    _dev(params, torch.float32, "params")
    _dev(grad, torch.float32, "grad")
    _dev(row_scale, torch.float32, "row_scale")
    _dev(labels, torch.int32, "labels")
    _check(lib().gad_train_round_batched(g.handle, _ptr(X), C.c_int(dtype), C.c_int(len(dims) - 1), _dims(dims),
                                         _ptr(params), _ptr(labels), _ptr(mask), _ptr(row_scale),
                                         C.c_float(negative_slope), _ptr(workspace), C.c_size_t(workspace.numel()),
                                         _ptr(grad), C.c_float(eta), _ptr(loss), C.c_int(1 if x_unchanged else 0),
                                         _stream()))
