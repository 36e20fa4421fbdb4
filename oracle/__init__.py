"""ctypes front-end of the CPU oracle (oracle/knn_softmax_oracle.c, oracle/topk_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's CPU-baseline
leg.  The product package never imports this module, and this module never imports the product.
All arrays are numpy; floating-point results are fp64.
"""
from __future__ import annotations

import ctypes as ct
import os

import numpy as np

from .build import LIB, build as _build

_lib = None

ORC_OK, ORC_BAD_ARG, ORC_BAD_LABEL, ORC_BAD_GRAPH_ID = 0, 1, 2, 3


def lib():
    global _lib
    if _lib is None:
        # ORACLE_LIB_PATH: another build of the same sources (the sanitizer build of the oracle's own test)
        path = os.environ.get("ORACLE_LIB_PATH") or (_build(force=False) if not os.path.exists(LIB) else LIB)
        _lib = ct.CDLL(path)
        _lib.orc_num_threads.restype = ct.c_int
        for name in ("orc_graph_bruteforce", "orc_select_active", "orc_knn_softmax_fwd_bwd",
                     "orc_full_softmax_fwd_bwd", "orc_apply_weight_grad", "orc_normalize_rows", "orc_norm_backward",
                     "orc_apply_weight_grad_normalized", "orc_graph_compress", "orc_pad_draws",
                     "orc_select_active_csr", "orc_graph_update", "orc_softmax_node_stats",
                     "orc_softmax_node_bwd", "orc_topk_abs", "orc_topk_dc", "orc_topk_group"):
            getattr(_lib, name).restype = ct.c_int
    return _lib


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(ct.POINTER(typ))


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def graph_bruteforce(W, K: int, rows=None):
    """Exact K nearest neighbours (inner product, self excluded, ties to the lowest id) of `rows`
    (all rows when None).  Returns (graph int32 [n,K], sims fp64 [n,K])."""
    W = _f32(W)
    C, D = W.shape
    rows_a = None if rows is None else _i32(rows)
    n = C if rows is None else rows_a.shape[0]
    graph = np.empty((n, K), dtype=np.int32)
    sims = np.empty((n, K), dtype=np.float64)
    rc = lib().orc_graph_bruteforce(_p(W, ct.c_float), ct.c_int64(C), ct.c_int(D), ct.c_int(K),
                                    _p(rows_a, ct.c_int32), ct.c_int64(n), _p(graph, ct.c_int32),
                                    _p(sims, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_graph_bruteforce failed with code {rc}")
    return graph, sims


def select_active(labels, G, C: int, M: int):
    """Algorithm 1 without the random fill-up.  Returns (active int32 [M] padded with -1, n_active,
    target_pos int32 [B])."""
    labels = _i32(labels)
    G = _i32(G)
    B = labels.shape[0]
    K = G.shape[1] if G.ndim == 2 else 0
    active = np.empty(M, dtype=np.int32)
    n_active = ct.c_int32(0)
    target_pos = np.empty(B, dtype=np.int32)
    rc = lib().orc_select_active(_p(labels, ct.c_int32), ct.c_int(B), _p(G, ct.c_int32), ct.c_int64(C),
                                 ct.c_int(K), ct.c_int(M), _p(active, ct.c_int32), ct.byref(n_active),
                                 _p(target_pos, ct.c_int32))
    if rc != ORC_OK:
        raise ValueError(f"orc_select_active failed with code {rc}")
    return active, int(n_active.value), target_pos


def knn_softmax_fwd_bwd(W, X, active, target_pos, scale: float, grad_scale: float = 1.0,
                        want_P: bool = False):
    """Softmax/CE forward and backward on the active columns.  `active` holds exactly the A valid ids.
    Returns dict(loss_i [B], loss, dX [B,D], dWA [A,D], lse [B], P [B,A] or None), all fp64."""
    W, X = _f32(W), _f32(X)
    active, target_pos = _i32(active), _i32(target_pos)
    A, (B, D) = active.shape[0], X.shape
    loss_i = np.empty(B, dtype=np.float64)
    loss = ct.c_double(0.0)
    dX = np.empty((B, D), dtype=np.float64)
    dWA = np.empty((A, D), dtype=np.float64)
    lse = np.empty(B, dtype=np.float64)
    P = np.empty((B, A), dtype=np.float64) if want_P else None
    rc = lib().orc_knn_softmax_fwd_bwd(_p(W, ct.c_float), _p(X, ct.c_float), _p(active, ct.c_int32),
                                       ct.c_int(A), _p(target_pos, ct.c_int32), ct.c_int(B), ct.c_int(D),
                                       ct.c_double(scale), ct.c_double(grad_scale), _p(loss_i, ct.c_double),
                                       ct.byref(loss), _p(dX, ct.c_double), _p(dWA, ct.c_double),
                                       _p(P, ct.c_double), _p(lse, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_knn_softmax_fwd_bwd failed with code {rc}")
    return dict(loss_i=loss_i, loss=float(loss.value), dX=dX, dWA=dWA, lse=lse, P=P)


def full_softmax_fwd_bwd(W, X, labels, scale: float, grad_scale: float = 1.0):
    """Full softmax over all classes.  Returns dict(loss_i, loss, dX [B,D], dW [C,D]), fp64."""
    W, X, labels = _f32(W), _f32(X), _i32(labels)
    (C, D), B = W.shape, X.shape[0]
    loss_i = np.empty(B, dtype=np.float64)
    loss = ct.c_double(0.0)
    dX = np.empty((B, D), dtype=np.float64)
    dW = np.empty((C, D), dtype=np.float64)
    rc = lib().orc_full_softmax_fwd_bwd(_p(W, ct.c_float), _p(X, ct.c_float), _p(labels, ct.c_int32),
                                        ct.c_int64(C), ct.c_int(B), ct.c_int(D), ct.c_double(scale),
                                        ct.c_double(grad_scale), _p(loss_i, ct.c_double), ct.byref(loss),
                                        _p(dX, ct.c_double), _p(dW, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_full_softmax_fwd_bwd failed with code {rc}")
    return dict(loss_i=loss_i, loss=float(loss.value), dX=dX, dW=dW)


def apply_weight_grad(W_master, idx, dW, alpha: float, want_bf16: bool = True):
    """W[c] += alpha * sum of the rows of dW addressed to c.  Returns (new fp32 master copy, bf16 bit
    patterns uint16 of the touched rows written into a copy that is zero elsewhere, or None).  The input
    array is not modified."""
    Wm = _f32(W_master).copy()
    idx, dW = _i32(idx), _f32(dW)
    C, D = Wm.shape
    n = idx.shape[0]
    Wb = np.zeros((C, D), dtype=np.uint16) if want_bf16 else None
    rc = lib().orc_apply_weight_grad(_p(Wm, ct.c_float), _p(Wb, ct.c_uint16), _p(idx, ct.c_int32), ct.c_int(n),
                                     _p(dW, ct.c_float), ct.c_double(alpha), ct.c_int64(C), ct.c_int(D))
    if rc != ORC_OK:
        raise ValueError(f"orc_apply_weight_grad failed with code {rc}")
    return Wm, Wb


def normalize_rows(V, want_bf16: bool = True):
    """Rows divided by their L2 norm (zero rows stay zero).  Returns (V_hat fp32, bf16 bit patterns of V_hat or
    None, inv_norm fp32 [n])."""
    V = _f32(V)
    n, D = V.shape
    Vh = np.empty((n, D), dtype=np.float32)
    Vb = np.empty((n, D), dtype=np.uint16) if want_bf16 else None
    inv = np.empty(n, dtype=np.float32)
    rc = lib().orc_normalize_rows(_p(V, ct.c_float), ct.c_int64(n), ct.c_int(D), _p(Vh, ct.c_float),
                                  _p(Vb, ct.c_uint16), _p(inv, ct.c_float))
    if rc != ORC_OK:
        raise ValueError(f"orc_normalize_rows failed with code {rc}")
    return Vh, Vb, inv


def norm_backward(V, G):
    """Gradient with respect to the rows V given the gradient G (fp64) with respect to V / |V|."""
    V = _f32(V)
    G = np.ascontiguousarray(G, dtype=np.float64)
    n, D = V.shape
    assert G.shape == (n, D)
    out = np.empty((n, D), dtype=np.float64)
    rc = lib().orc_norm_backward(_p(V, ct.c_float), _p(G, ct.c_double), ct.c_int64(n), ct.c_int(D), _p(out, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_norm_backward failed with code {rc}")
    return out


def apply_weight_grad_normalized(W_master, idx, dW_hat, alpha: float):
    """Update of the un-normalised master rows from gradients with respect to their normalised copies.
    Returns (new fp32 master copy, bf16 bit patterns of the re-normalised touched rows in an array that is zero
    elsewhere, inv_norm fp32 [C] that is zero for untouched rows).  The input array is not modified."""
    Wm = _f32(W_master).copy()
    idx, dW_hat = _i32(idx), _f32(dW_hat)
    C, D = Wm.shape
    n = idx.shape[0]
    Wb = np.zeros((C, D), dtype=np.uint16)
    inv = np.zeros(C, dtype=np.float32)
    rc = lib().orc_apply_weight_grad_normalized(_p(Wm, ct.c_float), _p(Wb, ct.c_uint16), _p(inv, ct.c_float),
                                                _p(idx, ct.c_int32), ct.c_int(n), _p(dW_hat, ct.c_float),
                                                ct.c_double(alpha), ct.c_int64(C), ct.c_int(D))
    if rc != ORC_OK:
        raise ValueError(f"orc_apply_weight_grad_normalized failed with code {rc}")
    return Wm, Wb, inv


def graph_compress(G, c0: int, C_loc: int):
    """Compressed graph of the node that owns classes [c0, c0 + C_loc): (counts int32 [Cg], offsets int64 [Cg + 1],
    flat int32 [offsets[-1]] of local ids)."""
    G = _i32(G)
    Cg, K = G.shape
    counts = np.empty(Cg, dtype=np.int32)
    offsets = np.empty(Cg + 1, dtype=np.int64)
    args = (_p(G, ct.c_int32), ct.c_int64(Cg), ct.c_int(K), ct.c_int64(c0), ct.c_int64(C_loc), _p(counts, ct.c_int32),
            _p(offsets, ct.c_int64))
    rc = lib().orc_graph_compress(*args, None)
    if rc != ORC_OK:
        raise ValueError(f"orc_graph_compress failed with code {rc}")
    flat = np.empty(max(int(offsets[-1]), 1), dtype=np.int32)
    rc = lib().orc_graph_compress(*args, _p(flat, ct.c_int32))
    if rc != ORC_OK:
        raise ValueError(f"orc_graph_compress failed with code {rc}")
    return counts, offsets, flat[:int(offsets[-1])]


def pad_draws(C_loc: int, seed: int, n: int):
    """The first n draws of the fill-up order for a node with C_loc classes (values in [0, 2^b))."""
    out = np.empty(n, dtype=np.uint32)
    rc = lib().orc_pad_draws(ct.c_int64(C_loc), ct.c_uint64(seed), ct.c_int64(n), _p(out, ct.c_uint32))
    if rc != ORC_OK:
        raise ValueError(f"orc_pad_draws failed with code {rc}")
    return out


def select_active_csr(labels, counts, offsets, flat, c0: int, C_loc: int, M: int, pad: bool = False, seed: int = 0):
    """Algorithm 1 on one node's compressed graph.  Returns (active int32 [M] of local ids padded with -1, n_active,
    n_found, target_pos int32 [B] with -1 for labels the node does not own)."""
    labels, counts, flat = _i32(labels), _i32(counts), _i32(flat)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    B, Cg = labels.shape[0], counts.shape[0]
    if flat.shape[0] == 0:
        flat = np.zeros(1, dtype=np.int32)
    active = np.empty(M, dtype=np.int32)
    n_active, n_found = ct.c_int32(0), ct.c_int32(0)
    target_pos = np.empty(B, dtype=np.int32)
    rc = lib().orc_select_active_csr(_p(labels, ct.c_int32), ct.c_int(B), _p(counts, ct.c_int32), _p(offsets, ct.c_int64),
                                     _p(flat, ct.c_int32), ct.c_int64(Cg), ct.c_int64(c0), ct.c_int64(C_loc), ct.c_int(M),
                                     ct.c_int(int(pad)), ct.c_uint64(seed), _p(active, ct.c_int32), ct.byref(n_active),
                                     ct.byref(n_found), _p(target_pos, ct.c_int32))
    if rc != ORC_OK:
        raise ValueError(f"orc_select_active_csr failed with code {rc}")
    return active, int(n_active.value), int(n_found.value), target_pos


def graph_update(W_local, W_visit, local_offset: int, visit_offset: int, graph, sims):
    """One hop of the distributed graph build: merges the visiting rows into the lists (graph int32 [C_loc, K] of
    ids of the whole problem, -1 = empty; sims fp64 [C_loc, K]).  Returns new arrays; the inputs are not modified."""
    W_local, W_visit = _f32(W_local), _f32(W_visit)
    graph = _i32(graph).copy()
    sims = np.ascontiguousarray(sims, dtype=np.float64).copy()
    (C_loc, D), C_vis, K = W_local.shape, W_visit.shape[0], graph.shape[1]
    assert graph.shape == (C_loc, K) and sims.shape == (C_loc, K) and W_visit.shape[1] == D
    rc = lib().orc_graph_update(_p(W_local, ct.c_float), ct.c_int64(C_loc), _p(W_visit, ct.c_float), ct.c_int64(C_vis),
                                ct.c_int(D), ct.c_int(K), ct.c_int64(local_offset), ct.c_int64(visit_offset),
                                _p(graph, ct.c_int32), _p(sims, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_graph_update failed with code {rc}")
    return graph, sims


def softmax_node_stats(W, X, active, target_pos, scale: float):
    """One node's part of the distributed softmax: per sample (max, sum of exponentials relative to it, target logit
    or 0 when target_pos < 0) over the node's active columns.  fp64 arrays [B]."""
    W, X = _f32(W), _f32(X)
    active, target_pos = _i32(active), _i32(target_pos)
    A, (B, D) = active.shape[0], X.shape
    m, l, t = (np.empty(B, dtype=np.float64) for _ in range(3))
    rc = lib().orc_softmax_node_stats(_p(W, ct.c_float), _p(X, ct.c_float), _p(active, ct.c_int32), ct.c_int(A),
                                      _p(target_pos, ct.c_int32), ct.c_int(B), ct.c_int(D), ct.c_double(scale),
                                      _p(m, ct.c_double), _p(l, ct.c_double), _p(t, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_softmax_node_stats failed with code {rc}")
    return m, l, t


def softmax_node_bwd(W, X, active, target_pos, scale: float, grad_scale: float, Mg, Sg, Tg):
    """One node's backward pass given the statistics combined over all nodes.  Returns dict(loss_i, loss, dX (this
    node's contribution), dWA), fp64."""
    W, X = _f32(W), _f32(X)
    active, target_pos = _i32(active), _i32(target_pos)
    Mg, Sg, Tg = (np.ascontiguousarray(v, dtype=np.float64) for v in (Mg, Sg, Tg))
    A, (B, D) = active.shape[0], X.shape
    loss_i = np.empty(B, dtype=np.float64)
    loss = ct.c_double(0.0)
    dX = np.empty((B, D), dtype=np.float64)
    dWA = np.empty((A, D), dtype=np.float64)
    rc = lib().orc_softmax_node_bwd(_p(W, ct.c_float), _p(X, ct.c_float), _p(active, ct.c_int32), ct.c_int(A),
                                    _p(target_pos, ct.c_int32), ct.c_int(B), ct.c_int(D), ct.c_double(scale),
                                    ct.c_double(grad_scale), _p(Mg, ct.c_double), _p(Sg, ct.c_double), _p(Tg, ct.c_double),
                                    _p(loss_i, ct.c_double), ct.byref(loss), _p(dX, ct.c_double), _p(dWA, ct.c_double))
    if rc != ORC_OK:
        raise ValueError(f"orc_softmax_node_bwd failed with code {rc}")
    return dict(loss_i=loss_i, loss=float(loss.value), dX=dX, dWA=dWA)


def combine_node_stats(stats):
    """(M, S, T) over nodes from a list of (m, l, t): M = max m, S = sum l exp(m - M), T = sum t."""
    M = np.max([m for m, _, _ in stats], axis=0)
    S = np.sum([l * np.exp(m - M) for m, l, _ in stats], axis=0)
    T = np.sum([t for _, _, t in stats], axis=0)
    return M, S, T


def topk_abs(g, k: int):
    """The k elements of largest magnitude of a tensor (Section 3.3.2), by definition: descending magnitude, equal
    magnitudes in ascending index.  Returns (idx int32 [k], val fp32 [k])."""
    g = _f32(g).ravel()
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float32)
    rc = lib().orc_topk_abs(_p(g, ct.c_float), ct.c_int64(g.size), ct.c_int(k), _p(idx, ct.c_int32), _p(val, ct.c_float))
    if rc != ORC_OK:
        raise ValueError(f"orc_topk_abs: {rc}")
    return idx, val


def topk_dc(g, k: int, M: int):
    """The same selection by the paper's two steps: top-k of each of M chunks, then top-k of the survivors."""
    g = _f32(g).ravel()
    idx = np.empty(k, dtype=np.int32)
    val = np.empty(k, dtype=np.float32)
    rc = lib().orc_topk_dc(_p(g, ct.c_float), ct.c_int64(g.size), ct.c_int(k), ct.c_int(M), _p(idx, ct.c_int32),
                           _p(val, ct.c_float))
    if rc != ORC_OK:
        raise ValueError(f"orc_topk_dc: {rc}")
    return idx, val


def topk_group(g, offsets, k, M=None):
    """Layer-wise selection over tensors stored back to back; M=None: by definition, else chunks per tensor.
    Returns (idx int32 [sum k], val fp32 [sum k]); tensor t's part starts at sum(k[:t])."""
    g = _f32(g).ravel()
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    k = _i32(k)
    T = k.size
    Ma = None if M is None else _i32(M)
    total = int(k.sum())
    idx = np.empty(total, dtype=np.int32)
    val = np.empty(total, dtype=np.float32)
    rc = lib().orc_topk_group(_p(g, ct.c_float), _p(offsets, ct.c_int64), _p(k, ct.c_int32), _p(Ma, ct.c_int32), ct.c_int(T),
                              _p(idx, ct.c_int32), _p(val, ct.c_float))
    if rc != ORC_OK:
        raise ValueError(f"orc_topk_group: {rc}")
    return idx, val
