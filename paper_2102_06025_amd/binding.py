"""ctypes binding of libknnsoftmax.so.  Function names and arguments mirror include/knnsoftmax.h; outputs
and workspaces that the caller does not pass in are allocated here as torch tensors on the inputs' device.
Nothing is computed in Python, and there is no fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as ct
import os

import torch

KS_OK, KS_INVALID_ARG, KS_UNSUPPORTED, KS_WORKSPACE_TOO_SMALL, KS_HIP_ERROR = 0, 1, 2, 3, 4
KS_DEV_BAD_LABEL, KS_DEV_BAD_GRAPH_ID, KS_DEV_BAD_INDEX, KS_DEV_IDX_NOT_SORTED, KS_DEV_BAD_COUNT = 1, 2, 4, 8, 16
KS_DEV_RANGE = 32
FLAG_PAD_RANDOM = 2
_STATUS = {1: "KS_INVALID_ARG", 2: "KS_UNSUPPORTED", 3: "KS_WORKSPACE_TOO_SMALL", 4: "KS_HIP_ERROR"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTS = ("ks_version", "knn_graph_build_workspace", "knn_graph_build", "knn_graph_build_plan", "knn_select_workspace",
           "knn_select_active", "knn_select_active_static", "knn_gather_rows", "knn_softmax_workspace", "knn_softmax_fwd_bwd",
           "full_softmax_workspace", "full_softmax_fwd_bwd", "apply_weight_grad_workspace", "apply_weight_grad",
           "knn_normalize_rows", "knn_norm_backward_rows", "apply_weight_grad_normalized_workspace",
           "apply_weight_grad_normalized", "knn_graph_compress_workspace", "knn_graph_compress",
           "knn_select_active_csr_workspace", "knn_select_active_csr", "knn_graph_update_workspace", "knn_graph_update",
           "knn_softmax_split_workspace", "knn_softmax_fwd_stats", "knn_softmax_bwd_from_stats",
           "knn_softmax_fwd_bwd_update", "knn_softmax_selected_workspace", "knn_softmax_fwd_bwd_update_selected",
           "knn_softmax_selected_next_workspace", "knn_softmax_fwd_bwd_update_selected_next",
           "knn_softmax_split_next_workspace", "knn_softmax_bwd_from_stats_next",
           "ks_peak_mfma", "ks_peak_copy", "grad_topk_plan", "grad_topk_workspace", "grad_topk_select")


class KsError(RuntimeError):
    def __init__(self, fn: str, code: int):
        super().__init__(f"{fn} returned {_STATUS.get(code, code)}")
        self.code = code


def lib_path() -> str:
    return os.path.join(_HERE, "libknnsoftmax.so")


def lib():
    """The loaded shared library.  Raises if it has not been built (python -m paper_2102_06025_amd.build)."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2102_06025_amd.build` "
                               "(there is no fallback implementation)")
        L = ct.CDLL(path)
        L.ks_version.restype = ct.c_char_p
        for name in EXPORTS:
            if name.endswith("_workspace"):
                getattr(L, name).restype = ct.c_size_t
            elif name == "grad_topk_plan":
                L.grad_topk_plan.restype = ct.c_int64
            elif name != "ks_version":
                getattr(L, name).restype = ct.c_int
        _LIB = L
    return _LIB


def ks_version() -> str:
    return lib().ks_version().decode()


def _ptr(t):
    return ct.c_void_p(0) if t is None else ct.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ct.c_void_p(s.cuda_stream)


def _check(fn, rc):
    if rc != KS_OK:
        raise KsError(fn, rc)


def _need(t, dtype, name):
    if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise TypeError(f"{name} must be a contiguous device tensor of {dtype}")
    return t


def _dtype_code(t):
    return 0 if t.dtype == torch.bfloat16 else 1  # KS_DTYPE_BF16 / KS_DTYPE_FP32


def _ws(nbytes, device, ws):
    if ws is not None:
        return ws
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def _status(device, dev_status):
    return torch.zeros(1, dtype=torch.int32, device=device) if dev_status is None else dev_status


# ---------------------------------------------------------------------------------------------------
def knn_graph_build_workspace(C, D, K, dtype) -> int:
    return int(lib().knn_graph_build_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(K), ct.c_int(dtype)))


def knn_graph_build_plan(C, D, K, dtype, workgroup=None):
    """Host-only.  -> (n_workgroups, plan) of the pass that computes every similarity once; n_workgroups == 0 when the
    problem takes the plain pass; plan (12 ints, see the header) only when `workgroup` is given."""
    n = ct.c_int32(0)
    out = (ct.c_int32 * 12)() if workgroup is not None else None
    rc = lib().knn_graph_build_plan(ct.c_int64(C), ct.c_int(D), ct.c_int(K), ct.c_int(dtype),
                                    ct.c_int(0 if workgroup is None else workgroup), ct.byref(n), out)
    _check("knn_graph_build_plan", rc)
    return int(n.value), (list(out) if out is not None else None)


def knn_graph_build(W, K, want_sims=False, graph=None, sims=None, ws=None, dev_status=None, stream=None):
    """W [C, D] bf16 or fp32 device tensor -> graph int32 [C, K] (and sims fp32 [C, K] when want_sims)."""
    if W.dtype == torch.bfloat16:
        dtype = 0
    elif W.dtype == torch.float32:
        dtype = 1
    else:
        raise TypeError("W must be bfloat16 or float32")
    if not (W.is_cuda and W.is_contiguous() and W.dim() == 2):
        raise TypeError("W must be a contiguous 2-D device tensor")
    C, D = W.shape
    need = knn_graph_build_workspace(C, D, K, dtype)
    if graph is None:
        graph = torch.empty((C, K), dtype=torch.int32, device=W.device)
    if want_sims and sims is None:
        sims = torch.empty((C, K), dtype=torch.float32, device=W.device)
    ws = _ws(need, W.device, ws)
    dev_status = _status(W.device, dev_status)
    rc = lib().knn_graph_build(_ptr(W), ct.c_int(dtype), ct.c_int64(C), ct.c_int(D), ct.c_int(K), _ptr(graph),
                               _ptr(sims), _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_graph_build", rc)
    return (graph, sims) if want_sims else graph


def knn_select_workspace(C, B, K, M) -> int:
    return int(lib().knn_select_workspace(ct.c_int64(C), ct.c_int(B), ct.c_int(K), ct.c_int(M)))


def knn_select_active(labels, graph, C, M, ws=None, dev_status=None, stream=None):
    """-> (active_idx int32 [M], n_active int32 [1] on the device, target_pos int32 [B], dev_status)."""
    _need(labels, torch.int32, "labels")
    B = labels.numel()
    K = 0 if graph is None else graph.shape[1]
    if graph is not None:
        _need(graph, torch.int32, "graph")
    dev = labels.device
    active_idx = torch.empty(M, dtype=torch.int32, device=dev)
    n_active = torch.empty(1, dtype=torch.int32, device=dev)
    target_pos = torch.empty(B, dtype=torch.int32, device=dev)
    ws = _ws(knn_select_workspace(C, B, K, M), dev, ws)
    dev_status = _status(dev, dev_status)
    rc = lib().knn_select_active(_ptr(labels), _ptr(graph), ct.c_int64(C), ct.c_int(B), ct.c_int(K), ct.c_int(M),
                                 _ptr(active_idx), _ptr(n_active), _ptr(target_pos), _ptr(ws),
                                 ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_select_active", rc)
    return active_idx, n_active, target_pos, dev_status


KS_SELECT_STATIC_BYTES = 2 << 20


def knn_select_active_static(labels, graph, C, M, out=None, dev_status=None, stream=None):
    """knn_select_active without a workspace: the library's own static device array serves as scratch (sizes up to
    knn_select_workspace(...) <= KS_SELECT_STATIC_BYTES).  `out` = (active_idx [M], n_active [1], target_pos [B])
    are used as the outputs when given, so that the call allocates nothing at all."""
    _need(labels, torch.int32, "labels")
    B = labels.numel()
    K = 0 if graph is None else graph.shape[1]
    if graph is not None:
        _need(graph, torch.int32, "graph")
    dev = labels.device
    if out is None:
        out = (torch.empty(M, dtype=torch.int32, device=dev), torch.empty(1, dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev))
    active_idx, n_active, target_pos = out
    if active_idx.numel() < M or target_pos.numel() < B:
        raise ValueError("out = (active_idx [M], n_active [1], target_pos [B])")
    dev_status = _status(dev, dev_status)
    rc = lib().knn_select_active_static(_ptr(labels), _ptr(graph), ct.c_int64(C), ct.c_int(B), ct.c_int(K), ct.c_int(M),
                                        _ptr(active_idx), _ptr(n_active), _ptr(target_pos), _ptr(dev_status),
                                        _stream(stream))
    _check("knn_select_active_static", rc)
    return active_idx, n_active, target_pos, dev_status


def knn_gather_rows(W_bf16, active_idx, n_active, out=None, dev_status=None, stream=None):
    _need(W_bf16, torch.bfloat16, "W_bf16")
    C, D = W_bf16.shape
    M = active_idx.numel()
    if out is None:
        out = torch.empty((M, D), dtype=torch.bfloat16, device=W_bf16.device)
    dev_status = _status(W_bf16.device, dev_status)
    rc = lib().knn_gather_rows(_ptr(W_bf16), _ptr(active_idx), _ptr(n_active), ct.c_int(M), ct.c_int64(C),
                               ct.c_int(D), _ptr(out), _ptr(dev_status), _stream(stream))
    _check("knn_gather_rows", rc)
    return out


def knn_softmax_workspace(C, D, B, K, M) -> int:
    return int(lib().knn_softmax_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(K), ct.c_int(M)))


FLAG_UNIT_ROWS = 1  # KS_FLAG_UNIT_ROWS
FLAG_TRUSTED_LIST = 4  # KS_FLAG_TRUSTED_LIST


def knn_softmax_fwd_bwd(W_bf16, X_bf16, labels, graph, M, scale, grad_scale=1.0, out=None, ws=None,
                        dev_status=None, stream=None, unit_rows=False):
    """One forward+backward step.  Returns a dict of device tensors: active_idx [M], n_active [1],
    target_pos [B], loss_per_sample [B], loss_mean [1], dX [B, D], dW_active [M, D], dev_status [1].
    Pass the dict of a previous call as `out` (and `ws`) to reuse the buffers.  unit_rows=True passes
    KS_FLAG_UNIT_ROWS (the rows of W_bf16 and X_bf16 are L2-normalised)."""
    _need(W_bf16, torch.bfloat16, "W_bf16")
    _need(X_bf16, torch.bfloat16, "X_bf16")
    _need(labels, torch.int32, "labels")
    C, D = W_bf16.shape
    B = X_bf16.shape[0]
    K = 0 if graph is None else graph.shape[1]
    if graph is not None:
        _need(graph, torch.int32, "graph")
    dev = W_bf16.device
    if out is None:
        out = dict(active_idx=torch.empty(M, dtype=torch.int32, device=dev),
                   n_active=torch.empty(1, dtype=torch.int32, device=dev),
                   target_pos=torch.empty(B, dtype=torch.int32, device=dev),
                   loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
                   loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
                   dX=torch.empty((B, D), dtype=torch.float32, device=dev),
                   dW_active=torch.empty((M, D), dtype=torch.float32, device=dev))
    ws = _ws(knn_softmax_workspace(C, D, B, K, M), dev, ws)
    dev_status = _status(dev, dev_status if dev_status is not None else out.get("dev_status"))
    out["dev_status"] = dev_status
    out["ws"] = ws
    rc = lib().knn_softmax_fwd_bwd(_ptr(W_bf16), _ptr(X_bf16), _ptr(labels), _ptr(graph), ct.c_int64(C), ct.c_int(D),
                                   ct.c_int(B), ct.c_int(K), ct.c_int(M), ct.c_float(scale), ct.c_float(grad_scale),
                                   ct.c_uint32(FLAG_UNIT_ROWS if unit_rows else 0), _ptr(out["active_idx"]), _ptr(out["n_active"]), _ptr(out["target_pos"]),
                                   _ptr(out["loss_per_sample"]), _ptr(out["loss_mean"]), _ptr(out["dX"]),
                                   _ptr(out["dW_active"]), _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status),
                                   _stream(stream))
    _check("knn_softmax_fwd_bwd", rc)
    return out


def knn_softmax_fwd_bwd_update(W_master, W_bf16, X_bf16, labels, graph, M, scale, grad_scale, alpha, out=None, ws=None,
                               dev_status=None, stream=None, unit_rows=False, want_dW=False):
    """The whole step in one call: forward+backward and the in-place update of W_master (fp32) and W_bf16.
    Returns the dict of knn_softmax_fwd_bwd; dW_active is None unless want_dW (or D % 64 != 0, where it is needed)."""
    _need(W_master, torch.float32, "W_master")
    _need(W_bf16, torch.bfloat16, "W_bf16")
    _need(X_bf16, torch.bfloat16, "X_bf16")
    _need(labels, torch.int32, "labels")
    C, D = W_bf16.shape
    if tuple(W_master.shape) != (C, D):
        raise ValueError("W_master and W_bf16 must have the same shape")
    B = X_bf16.shape[0]
    K = 0 if graph is None else graph.shape[1]
    if graph is not None:
        _need(graph, torch.int32, "graph")
    dev = W_bf16.device
    if out is None:
        out = dict(active_idx=torch.empty(M, dtype=torch.int32, device=dev),
                   n_active=torch.empty(1, dtype=torch.int32, device=dev),
                   target_pos=torch.empty(B, dtype=torch.int32, device=dev),
                   loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
                   loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
                   dX=torch.empty((B, D), dtype=torch.float32, device=dev),
                   dW_active=torch.empty((M, D), dtype=torch.float32, device=dev) if (want_dW or D % 64) else None)
    ws = _ws(knn_softmax_workspace(C, D, B, K, M), dev, ws)
    dev_status = _status(dev, dev_status if dev_status is not None else out.get("dev_status"))
    out["dev_status"] = dev_status
    out["ws"] = ws
    rc = lib().knn_softmax_fwd_bwd_update(_ptr(W_master), _ptr(W_bf16), _ptr(X_bf16), _ptr(labels), _ptr(graph),
                                          ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(K), ct.c_int(M), ct.c_float(scale),
                                          ct.c_float(grad_scale), ct.c_float(alpha),
                                          ct.c_uint32(FLAG_UNIT_ROWS if unit_rows else 0), _ptr(out["active_idx"]),
                                          _ptr(out["n_active"]), _ptr(out["target_pos"]), _ptr(out["loss_per_sample"]),
                                          _ptr(out["loss_mean"]), _ptr(out["dX"]), _ptr(out.get("dW_active")), _ptr(ws),
                                          ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_softmax_fwd_bwd_update", rc)
    return out


def knn_softmax_selected_workspace(C, D, B, M) -> int:
    return int(lib().knn_softmax_selected_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(M)))


def knn_softmax_fwd_bwd_update_selected(W_master, W_bf16, X_bf16, active_idx, n_active, target_pos, scale, grad_scale, alpha,
                                        out=None, ws=None, dev_status=None, stream=None, unit_rows=False, want_dW=False,
                                        trusted_list=False):
    """The step on a selection computed earlier by knn_select_active (W_master may be None: no update, dW_active is
    then returned).  Returns dict(loss_per_sample, loss_mean, dX, dW_active or None, dev_status, ws)."""
    _need(W_bf16, torch.bfloat16, "W_bf16")
    _need(X_bf16, torch.bfloat16, "X_bf16")
    _need(active_idx, torch.int32, "active_idx")
    _need(target_pos, torch.int32, "target_pos")
    if W_master is not None:
        _need(W_master, torch.float32, "W_master")
    C, D = W_bf16.shape
    B, M = X_bf16.shape[0], active_idx.numel()
    dev = W_bf16.device
    need_dW = want_dW or W_master is None or D % 64 != 0
    if out is None:
        out = dict(loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
                   loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
                   dX=torch.empty((B, D), dtype=torch.float32, device=dev),
                   dW_active=torch.empty((M, D), dtype=torch.float32, device=dev) if need_dW else None)
    ws = _ws(knn_softmax_selected_workspace(C, D, B, M), dev, ws)
    dev_status = _status(dev, dev_status if dev_status is not None else out.get("dev_status"))
    out["dev_status"], out["ws"] = dev_status, ws
    rc = lib().knn_softmax_fwd_bwd_update_selected(_ptr(W_master), _ptr(W_bf16), _ptr(X_bf16), _ptr(active_idx), _ptr(n_active),
                                                   _ptr(target_pos), ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(M),
                                                   ct.c_float(scale), ct.c_float(grad_scale), ct.c_float(alpha),
                                                   ct.c_uint32((FLAG_UNIT_ROWS if unit_rows else 0) | (FLAG_TRUSTED_LIST if trusted_list else 0)),
                                                   _ptr(out["loss_per_sample"]),
                                                   _ptr(out["loss_mean"]), _ptr(out["dX"]), _ptr(out.get("dW_active")), _ptr(ws),
                                                   ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_softmax_fwd_bwd_update_selected", rc)
    return out


def knn_softmax_selected_next_workspace(C, D, B, K, M) -> int:
    return int(lib().knn_softmax_selected_next_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(K), ct.c_int(M)))


def knn_softmax_fwd_bwd_update_selected_next(W_master, W_bf16, X_bf16, active_idx, n_active, target_pos, labels_next, graph,
                                             scale, grad_scale, alpha, next_out=None, out=None, ws=None, dev_status=None,
                                             stream=None, unit_rows=False, want_dW=False, trusted_list=False):
    """The step on a given selection, and in the same launches the selection of the next batch (labels_next).
    next_out: dict(active_idx, n_active, target_pos) to write the next selection to (None: this call's own list
    buffers are reused; not with trusted_list, which reads the list in place).  Returns (out, next_out)."""
    _need(W_bf16, torch.bfloat16, "W_bf16")
    _need(X_bf16, torch.bfloat16, "X_bf16")
    _need(active_idx, torch.int32, "active_idx")
    _need(target_pos, torch.int32, "target_pos")
    _need(labels_next, torch.int32, "labels_next")
    _need(graph, torch.int32, "graph")
    if W_master is not None:
        _need(W_master, torch.float32, "W_master")
    C, D = W_bf16.shape
    B, M, K = X_bf16.shape[0], active_idx.numel(), graph.shape[1]
    dev = W_bf16.device
    need_dW = want_dW or W_master is None or D % 64 != 0
    if out is None:
        out = dict(loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
                   loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
                   dX=torch.empty((B, D), dtype=torch.float32, device=dev),
                   dW_active=torch.empty((M, D), dtype=torch.float32, device=dev) if need_dW else None)
    if next_out is None:
        next_out = dict(active_idx=active_idx, n_active=n_active, target_pos=target_pos)
    ws = _ws(knn_softmax_selected_next_workspace(C, D, B, K, M), dev, ws)
    dev_status = _status(dev, dev_status if dev_status is not None else out.get("dev_status"))
    out["dev_status"], out["ws"] = dev_status, ws
    rc = lib().knn_softmax_fwd_bwd_update_selected_next(
        _ptr(W_master), _ptr(W_bf16), _ptr(X_bf16), _ptr(active_idx), _ptr(n_active), _ptr(target_pos), ct.c_int64(C),
        ct.c_int(D), ct.c_int(B), ct.c_int(M), ct.c_float(scale), ct.c_float(grad_scale), ct.c_float(alpha),
        ct.c_uint32((FLAG_UNIT_ROWS if unit_rows else 0) | (FLAG_TRUSTED_LIST if trusted_list else 0)),
        _ptr(out["loss_per_sample"]), _ptr(out["loss_mean"]), _ptr(out["dX"]),
        _ptr(out.get("dW_active")), _ptr(labels_next), _ptr(graph), ct.c_int(K), _ptr(next_out["active_idx"]),
        _ptr(next_out["n_active"]), _ptr(next_out["target_pos"]), _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status),
        _stream(stream))
    _check("knn_softmax_fwd_bwd_update_selected_next", rc)
    return out, next_out


def full_softmax_workspace(C, D, B) -> int:
    return int(lib().full_softmax_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(B)))


def full_softmax_fwd_bwd(W_bf16, X_bf16, labels, scale, grad_scale=1.0, out=None, ws=None, dev_status=None,
                         stream=None, unit_rows=False):
    """Full softmax over all classes.  Returns dict(loss_per_sample, loss_mean, dX, dW [C, D], dev_status)."""
    _need(W_bf16, torch.bfloat16, "W_bf16")
    _need(X_bf16, torch.bfloat16, "X_bf16")
    _need(labels, torch.int32, "labels")
    C, D = W_bf16.shape
    B = X_bf16.shape[0]
    dev = W_bf16.device
    if out is None:
        out = dict(loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
                   loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
                   dX=torch.empty((B, D), dtype=torch.float32, device=dev),
                   dW=torch.empty((C, D), dtype=torch.float32, device=dev))
    ws = _ws(full_softmax_workspace(C, D, B), dev, ws)
    dev_status = _status(dev, dev_status if dev_status is not None else out.get("dev_status"))
    out["dev_status"] = dev_status
    out["ws"] = ws
    rc = lib().full_softmax_fwd_bwd(_ptr(W_bf16), _ptr(X_bf16), _ptr(labels), ct.c_int64(C), ct.c_int(D), ct.c_int(B),
                                    ct.c_float(scale), ct.c_float(grad_scale), ct.c_uint32(FLAG_UNIT_ROWS if unit_rows else 0),
                                    _ptr(out["loss_per_sample"]),
                                    _ptr(out["loss_mean"]), _ptr(out["dX"]), _ptr(out["dW"]), _ptr(ws),
                                    ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("full_softmax_fwd_bwd", rc)
    return out


def apply_weight_grad_workspace(C, D, n_max, idx_sorted_unique) -> int:
    return int(lib().apply_weight_grad_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(n_max),
                                                 ct.c_int(int(idx_sorted_unique))))


def apply_weight_grad(W_master, W_bf16, idx, n, dW, alpha, idx_sorted_unique=False, ws=None, dev_status=None,
                      stream=None):
    """In-place update of W_master (fp32) and W_bf16 (may be None).  `n` is a device int32 scalar or None."""
    _need(W_master, torch.float32, "W_master")
    _need(idx, torch.int32, "idx")
    _need(dW, torch.float32, "dW")
    if W_bf16 is not None:
        _need(W_bf16, torch.bfloat16, "W_bf16")
    C, D = W_master.shape
    n_max = idx.numel()
    if dW.shape[0] < n_max or dW.shape[1] != D:
        raise ValueError("dW must be [n_max, D]")
    ws = _ws(apply_weight_grad_workspace(C, D, n_max, idx_sorted_unique), W_master.device, ws)
    dev_status = _status(W_master.device, dev_status)
    rc = lib().apply_weight_grad(_ptr(W_master), _ptr(W_bf16), _ptr(idx), _ptr(n), ct.c_int(n_max), _ptr(dW),
                                 ct.c_float(alpha), ct.c_int64(C), ct.c_int(D), ct.c_int(int(idx_sorted_unique)),
                                 _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("apply_weight_grad", rc)
    return dev_status


def knn_normalize_rows(V, want_bf16=True, want_inv_norm=True, out_bf16=None, out_inv_norm=None, stream=None):
    """Rows of V (bf16 or fp32) divided by their L2 norm.  Returns (V_hat bf16 or None, inv_norm fp32 or None);
    `out_bf16` / `out_inv_norm` are used as the outputs when given."""
    if V.dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("V must be bfloat16 or float32")
    _need(V, V.dtype, "V")
    n, D = V.shape
    Vh = out_bf16 if out_bf16 is not None else (
        torch.empty((n, D), dtype=torch.bfloat16, device=V.device) if want_bf16 else None)
    inv = out_inv_norm if out_inv_norm is not None else (
        torch.empty(n, dtype=torch.float32, device=V.device) if want_inv_norm else None)
    if Vh is not None and (_need(Vh, torch.bfloat16, "out_bf16").numel() != n * D):
        raise ValueError("out_bf16 must be [n, D]")
    if inv is not None and (_need(inv, torch.float32, "out_inv_norm").numel() != n):
        raise ValueError("out_inv_norm must be [n]")
    rc = lib().knn_normalize_rows(_ptr(V), ct.c_int(_dtype_code(V)), ct.c_int64(n), ct.c_int(D), _ptr(Vh), _ptr(inv),
                                  _stream(stream))
    _check("knn_normalize_rows", rc)
    return Vh, inv


def knn_norm_backward_rows(V, G, out=None, stream=None):
    """Gradient with respect to the rows of V from the gradient G (fp32) with respect to V / |V|."""
    if V.dtype not in (torch.bfloat16, torch.float32):
        raise TypeError("V must be bfloat16 or float32")
    _need(V, V.dtype, "V")
    _need(G, torch.float32, "G")
    n, D = V.shape
    if tuple(G.shape) != (n, D):
        raise ValueError("G must be [n, D]")
    if out is None:
        out = torch.empty_like(G)
    _need(out, torch.float32, "out")
    rc = lib().knn_norm_backward_rows(_ptr(V), ct.c_int(_dtype_code(V)), _ptr(G), ct.c_int64(n), ct.c_int(D), _ptr(out),
                                      _stream(stream))
    _check("knn_norm_backward_rows", rc)
    return out


def apply_weight_grad_normalized_workspace(C, D, n_max, idx_sorted_unique) -> int:
    return int(lib().apply_weight_grad_normalized_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(n_max),
                                                            ct.c_int(int(idx_sorted_unique))))


def apply_weight_grad_normalized(W_master, W_hat_bf16, inv_norm, idx, n, dW_hat, alpha, idx_sorted_unique=False, ws=None,
                                 dev_status=None, stream=None):
    """In-place update of W_master (fp32), of the normalised copy W_hat_bf16 and of inv_norm (either may be None)
    from gradients with respect to the normalised rows."""
    _need(W_master, torch.float32, "W_master")
    _need(idx, torch.int32, "idx")
    _need(dW_hat, torch.float32, "dW_hat")
    if W_hat_bf16 is not None:
        _need(W_hat_bf16, torch.bfloat16, "W_hat_bf16")
    if inv_norm is not None:
        _need(inv_norm, torch.float32, "inv_norm")
    C, D = W_master.shape
    n_max = idx.numel()
    if dW_hat.shape[0] < n_max or dW_hat.shape[1] != D:
        raise ValueError("dW_hat must be [n_max, D]")
    ws = _ws(apply_weight_grad_normalized_workspace(C, D, n_max, idx_sorted_unique), W_master.device, ws)
    dev_status = _status(W_master.device, dev_status)
    rc = lib().apply_weight_grad_normalized(_ptr(W_master), _ptr(W_hat_bf16), _ptr(inv_norm), _ptr(idx), _ptr(n),
                                            ct.c_int(n_max), _ptr(dW_hat), ct.c_float(alpha), ct.c_int64(C), ct.c_int(D),
                                            ct.c_int(int(idx_sorted_unique)), _ptr(ws), ct.c_size_t(ws.numel()),
                                            _ptr(dev_status), _stream(stream))
    _check("apply_weight_grad_normalized", rc)
    return dev_status


def knn_graph_compress(graph, c0, C_loc, dev_status=None, stream=None):
    """Compressed graph of the node that owns classes [c0, c0 + C_loc) of the dense graph [Cg, K] (global ids).
    Returns (counts int32 [Cg], offsets int64 [Cg + 1], flat int32 [total] of local ids, dev_status).  Two calls of
    the library (lengths first, then the lists) with one read-back of the total in between."""
    _need(graph, torch.int32, "graph")
    Cg, K = graph.shape
    dev = graph.device
    counts = torch.empty(Cg, dtype=torch.int32, device=dev)
    offsets = torch.empty(Cg + 1, dtype=torch.int64, device=dev)
    ws = _ws(int(lib().knn_graph_compress_workspace(ct.c_int64(Cg), ct.c_int(K))), dev, None)
    dev_status = _status(dev, dev_status)

    def call(flat, cap):
        rc = lib().knn_graph_compress(_ptr(graph), ct.c_int64(Cg), ct.c_int(K), ct.c_int64(c0), ct.c_int64(C_loc),
                                      _ptr(counts), _ptr(offsets), _ptr(flat), ct.c_int64(cap), _ptr(ws),
                                      ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
        _check("knn_graph_compress", rc)

    call(None, 0)
    total = int(offsets[Cg].item())
    flat = torch.empty(max(total, 1), dtype=torch.int32, device=dev)
    call(flat, total)
    return counts, offsets, flat[:total], dev_status


def knn_select_active_csr_workspace(C_loc, B, K_max, M) -> int:
    return int(lib().knn_select_active_csr_workspace(ct.c_int64(C_loc), ct.c_int(B), ct.c_int(K_max), ct.c_int(M)))


def knn_select_active_csr(labels, counts, offsets, flat, c0, C_loc, K_max, M, pad_random=False, pad_seed=0, ws=None,
                          dev_status=None, stream=None):
    """Algorithm 1 on one node's compressed graph.  Returns dict(active_idx [M] local ids, n_active [1], n_found [1],
    target_pos [B] with -1 for labels of other nodes' classes, dev_status)."""
    _need(labels, torch.int32, "labels")
    _need(counts, torch.int32, "counts")
    _need(offsets, torch.int64, "offsets")
    if flat.numel():
        _need(flat, torch.int32, "flat")
    dev = labels.device
    B, Cg = labels.numel(), counts.numel()
    if offsets.numel() != Cg + 1:
        raise ValueError("offsets must be [Cg + 1]")
    out = dict(active_idx=torch.empty(M, dtype=torch.int32, device=dev),
               n_active=torch.empty(1, dtype=torch.int32, device=dev),
               n_found=torch.empty(1, dtype=torch.int32, device=dev),
               target_pos=torch.empty(B, dtype=torch.int32, device=dev))
    ws = _ws(knn_select_active_csr_workspace(C_loc, B, K_max, M), dev, ws)
    dev_status = _status(dev, dev_status)
    out["dev_status"] = dev_status
    rc = lib().knn_select_active_csr(_ptr(labels), _ptr(counts), _ptr(offsets), _ptr(flat if flat.numel() else None),
                                     ct.c_int64(flat.numel()), ct.c_int64(Cg), ct.c_int64(c0), ct.c_int64(C_loc),
                                     ct.c_int(B), ct.c_int(K_max), ct.c_int(M),
                                     ct.c_uint32(FLAG_PAD_RANDOM if pad_random else 0), ct.c_uint64(pad_seed),
                                     _ptr(out["active_idx"]), _ptr(out["n_active"]), _ptr(out["n_found"]),
                                     _ptr(out["target_pos"]), _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status),
                                     _stream(stream))
    _check("knn_select_active_csr", rc)
    return out


def knn_graph_update_workspace(C_loc, C_vis, D, K, dtype) -> int:
    return int(lib().knn_graph_update_workspace(ct.c_int64(C_loc), ct.c_int64(C_vis), ct.c_int(D), ct.c_int(K),
                                                ct.c_int(dtype)))


def knn_graph_update(W_local, W_visit, local_offset, visit_offset, graph, sims, ws=None, dev_status=None, stream=None):
    """One hop of the distributed graph build: merges the visiting shard into graph (int32 [C_loc, K], -1 = empty) and
    sims (float64 [C_loc, K]) in place."""
    if W_local.dtype not in (torch.bfloat16, torch.float32) or W_visit.dtype != W_local.dtype:
        raise TypeError("W_local and W_visit must both be bfloat16 or both float32")
    _need(W_local, W_local.dtype, "W_local")
    _need(W_visit, W_visit.dtype, "W_visit")
    _need(graph, torch.int32, "graph")
    _need(sims, torch.float64, "sims")
    (C_loc, D), C_vis, K = W_local.shape, W_visit.shape[0], graph.shape[1]
    if W_visit.shape[1] != D or tuple(graph.shape) != (C_loc, K) or tuple(sims.shape) != (C_loc, K):
        raise ValueError("shapes: W_visit [C_vis, D], graph and sims [C_loc, K]")
    dtype = _dtype_code(W_local)
    ws = _ws(knn_graph_update_workspace(C_loc, C_vis, D, K, dtype), W_local.device, ws)
    dev_status = _status(W_local.device, dev_status)
    rc = lib().knn_graph_update(_ptr(W_local), _ptr(W_visit), ct.c_int(dtype), ct.c_int64(C_loc), ct.c_int64(C_vis),
                                ct.c_int(D), ct.c_int(K), ct.c_int64(local_offset), ct.c_int64(visit_offset), _ptr(graph),
                                _ptr(sims), _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_graph_update", rc)
    return dev_status


def knn_softmax_split_workspace(C, D, B, M) -> int:
    return int(lib().knn_softmax_split_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(M)))


def knn_softmax_fwd_stats(W_bf16, X_bf16, active_idx, n_active, target_pos, scale, unit_rows=False, ws=None,
                          dev_status=None, stream=None, trusted_list=False, out=None):
    """First call of the softmax split over nodes.  Returns dict(row_max, row_sumexp, target_logit [B] fp32, ws,
    dev_status); pass the same `ws` to knn_softmax_bwd_from_stats."""
    _need(W_bf16, torch.bfloat16, "W_bf16")
    _need(X_bf16, torch.bfloat16, "X_bf16")
    _need(active_idx, torch.int32, "active_idx")
    _need(target_pos, torch.int32, "target_pos")
    (C, D), B, M = W_bf16.shape, X_bf16.shape[0], active_idx.numel()
    dev = W_bf16.device
    if out is None:
        out = dict(row_max=torch.empty(B, dtype=torch.float32, device=dev),
                   row_sumexp=torch.empty(B, dtype=torch.float32, device=dev),
                   target_logit=torch.empty(B, dtype=torch.float32, device=dev))
    ws = _ws(knn_softmax_split_workspace(C, D, B, M), dev, ws)
    dev_status = _status(dev, dev_status)
    out["ws"], out["dev_status"] = ws, dev_status
    rc = lib().knn_softmax_fwd_stats(_ptr(W_bf16), _ptr(X_bf16), _ptr(active_idx), _ptr(n_active), _ptr(target_pos),
                                     ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(M), ct.c_float(scale),
                                     ct.c_uint32((FLAG_UNIT_ROWS if unit_rows else 0) | (FLAG_TRUSTED_LIST if trusted_list else 0)),
                                     _ptr(out["row_max"]),
                                     _ptr(out["row_sumexp"]), _ptr(out["target_logit"]), _ptr(ws), ct.c_size_t(ws.numel()),
                                     _ptr(dev_status), _stream(stream))
    _check("knn_softmax_fwd_stats", rc)
    return out


def knn_softmax_split_next_workspace(C, D, B, K_max, M) -> int:
    return int(lib().knn_softmax_split_next_workspace(ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(K_max), ct.c_int(M)))


def knn_softmax_bwd_from_stats_next(W_bf16, X_bf16, active_idx, n_active, target_pos, global_max, global_sumexp,
                                    global_target_logit, scale, grad_scale, ws, labels_next, counts, offsets, flat, c0, K_max,
                                    next_out=None, pad_random=False, pad_seed=0, unit_rows=False, trusted_list=False,
                                    dev_status=None, stream=None, out=None):
    """knn_softmax_bwd_from_stats, and in the same launches knn_select_active_csr for the next batch (labels_next).
    `ws` (knn_softmax_split_next_workspace) is the first call's.  next_out: dict(active_idx, n_active, n_found,
    target_pos) for the next list (None: this call's own list buffers, not with trusted_list).  Returns (out, next_out)."""
    for t, name in ((global_max, "global_max"), (global_sumexp, "global_sumexp"), (global_target_logit, "global_target_logit")):
        _need(t, torch.float32, name)
    _need(labels_next, torch.int32, "labels_next")
    _need(counts, torch.int32, "counts")
    _need(offsets, torch.int64, "offsets")
    _need(flat, torch.int32, "flat")
    (C, D), B, M = W_bf16.shape, X_bf16.shape[0], active_idx.numel()
    dev = W_bf16.device
    if out is None:
        out = dict(loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
                   loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
                   dX=torch.empty((B, D), dtype=torch.float32, device=dev),
                   dW_active=torch.empty((M, D), dtype=torch.float32, device=dev))
    if next_out is None:
        next_out = dict(active_idx=active_idx, n_active=n_active, n_found=None, target_pos=target_pos)
    dev_status = _status(dev, dev_status if dev_status is not None else out.get("dev_status"))
    out["dev_status"] = dev_status
    flags = (FLAG_UNIT_ROWS if unit_rows else 0) | (FLAG_TRUSTED_LIST if trusted_list else 0)
    rc = lib().knn_softmax_bwd_from_stats_next(
        _ptr(W_bf16), _ptr(X_bf16), _ptr(active_idx), _ptr(n_active), _ptr(target_pos), _ptr(global_max), _ptr(global_sumexp),
        _ptr(global_target_logit), ct.c_int64(C), ct.c_int(D), ct.c_int(B), ct.c_int(M), ct.c_float(scale), ct.c_float(grad_scale),
        ct.c_uint32(flags), _ptr(out["loss_per_sample"]), _ptr(out["loss_mean"]), _ptr(out["dX"]), _ptr(out["dW_active"]),
        _ptr(labels_next), _ptr(counts), _ptr(offsets), _ptr(flat), ct.c_int64(flat.numel()), ct.c_int64(counts.numel()),
        ct.c_int64(c0), ct.c_int(K_max), ct.c_uint32(FLAG_PAD_RANDOM if pad_random else 0), ct.c_uint64(pad_seed),
        _ptr(next_out["active_idx"]), _ptr(next_out["n_active"]), _ptr(next_out.get("n_found")), _ptr(next_out["target_pos"]),
        _ptr(ws), ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_softmax_bwd_from_stats_next", rc)
    return out, next_out


def knn_softmax_bwd_from_stats(W_bf16, X_bf16, active_idx, n_active, target_pos, global_max, global_sumexp,
                               global_target_logit, scale, grad_scale, ws, unit_rows=False, dev_status=None, stream=None,
                               trusted_list=False):
    """Second call of the softmax split over nodes (`ws` is the first call's).  Returns dict(loss_per_sample,
    loss_mean, dX (this node's contribution), dW_active, dev_status)."""
    for t, name in ((global_max, "global_max"), (global_sumexp, "global_sumexp"), (global_target_logit, "global_target_logit")):
        _need(t, torch.float32, name)
    (C, D), B, M = W_bf16.shape, X_bf16.shape[0], active_idx.numel()
    dev = W_bf16.device
    out = dict(loss_per_sample=torch.empty(B, dtype=torch.float32, device=dev),
               loss_mean=torch.empty(1, dtype=torch.float32, device=dev),
               dX=torch.empty((B, D), dtype=torch.float32, device=dev),
               dW_active=torch.empty((M, D), dtype=torch.float32, device=dev))
    dev_status = _status(dev, dev_status)
    out["dev_status"] = dev_status
    rc = lib().knn_softmax_bwd_from_stats(_ptr(W_bf16), _ptr(X_bf16), _ptr(active_idx), _ptr(n_active), _ptr(target_pos),
                                          _ptr(global_max), _ptr(global_sumexp), _ptr(global_target_logit), ct.c_int64(C),
                                          ct.c_int(D), ct.c_int(B), ct.c_int(M), ct.c_float(scale), ct.c_float(grad_scale),
                                          ct.c_uint32((FLAG_UNIT_ROWS if unit_rows else 0) | (FLAG_TRUSTED_LIST if trusted_list else 0)),
                                          _ptr(out["loss_per_sample"]),
                                          _ptr(out["loss_mean"]), _ptr(out["dX"]), _ptr(out["dW_active"]), _ptr(ws),
                                          ct.c_size_t(ws.numel()), _ptr(dev_status), _stream(stream))
    _check("knn_softmax_bwd_from_stats", rc)
    return out


# ---------------------------------------------------------------------------------------------------
# layer-wise top-k selection for gradient sparsification (include/grad_topk.h)
# ---------------------------------------------------------------------------------------------------
class GradTopkPlan:
    """Plan of grad_topk_select for a group of tensors: the host words and their copy in device memory."""

    def __init__(self, host, device):
        self.host = host        # numpy int64, the words written by grad_topk_plan
        self.dev = torch.from_numpy(host).to(device)
        self.T = int(host[1])
        self.n_workgroups = int(host[2])   # selection steps over all levels
        self.n_out = int(host[4])
        self.n_levels = int(host[6])       # levels of the plan
        self.n_filtered_chunks = int(host[29])  # chunks on the sampled path (a launch of their own)
        self.n_launches = sum(1 for lev in range(self.n_levels)
                              if int(host[9 + 2 * lev]) - (self.n_filtered_chunks if lev == 1 else 0) > 0) + (self.n_filtered_chunks > 0)
        self.ws_bytes = int(lib().grad_topk_workspace(host.ctypes.data_as(ct.c_void_p)))

    def chunks(self):
        """Chunks of every tensor (the paper's M)."""
        return [int(self.host[32 + 4 * t + 2]) for t in range(self.T)]

    def steps(self):
        """Selection steps every tensor goes through (1 = a single chunk; 2 = the paper's chunks + final selection;
        3 = threshold from a sample, filtered chunks, final selection, or a deeper tree of selections)."""
        return [int(self.host[32 + 4 * t + 3]) for t in range(self.T)]


def grad_topk_plan(offsets, k, chunks=0, device="cuda") -> GradTopkPlan:
    import numpy as np
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    k = np.ascontiguousarray(k, dtype=np.int32)
    T = int(k.size)
    if offsets.size != T + 1:
        raise ValueError("offsets must have one more entry than k")
    args = (offsets.ctypes.data_as(ct.c_void_p), k.ctypes.data_as(ct.c_void_p), ct.c_int(T), ct.c_int(chunks))
    words = int(lib().grad_topk_plan(*args, ct.c_void_p(0), ct.c_int64(0)))
    if words < 0:
        raise KsError("grad_topk_plan", -words)
    host = np.zeros(words, dtype=np.int64)
    got = int(lib().grad_topk_plan(*args, host.ctypes.data_as(ct.c_void_p), ct.c_int64(words)))
    if got != words:
        raise KsError("grad_topk_plan", -got if got < 0 else KS_INVALID_ARG)
    return GradTopkPlan(host, device)


def grad_topk_select(g, plan: GradTopkPlan, out_idx=None, out_val=None, ws=None, stream=None):
    """Top-k by magnitude of every tensor of the group (one launch per level of the plan).  Returns (idx int32 [sum k], val fp32 [sum k])."""
    _need(g, torch.float32, "g")
    if out_idx is None:
        out_idx = torch.empty(plan.n_out, dtype=torch.int32, device=g.device)
    if out_val is None:
        out_val = torch.empty(plan.n_out, dtype=torch.float32, device=g.device)
    _need(out_idx, torch.int32, "out_idx")
    _need(out_val, torch.float32, "out_val")
    if g.numel() < int(plan.host[5]) or out_idx.numel() < plan.n_out or out_val.numel() < plan.n_out:
        raise ValueError("g, out_idx or out_val is smaller than the plan requires")
    ws = _ws(plan.ws_bytes, g.device, ws)
    _check("grad_topk_select", lib().grad_topk_select(_ptr(g), _ptr(plan.dev), plan.host.ctypes.data_as(ct.c_void_p),
                                                      _ptr(out_idx), _ptr(out_val), _ptr(ws), ct.c_size_t(ws.numel()),
                                                      _stream(stream)))
    return out_idx, out_val
