"""Python binding of libgsr.so, the MI355X (gfx950) GSR-GNN training-step library.

Argument marshalling only: every function has the name of the C entry point it calls
(include/gsr.h) and does no arithmetic of its own.  PyTorch provides device memory and the
current HIP stream, nothing else.  If the compiled library is missing the import of the
package still works (so the input generators in `synth` stay usable on a CPU-only box) but
every call raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# GSR_LIB names another build of the library (kernel variants under measurement); default: the one built in-tree
LIB_PATH = os.environ.get("GSR_LIB") or os.path.join(_HERE, "libgsr.so")

GSR_OK, GSR_ERR_INVALID_ARG, GSR_ERR_BAD_CSR, GSR_ERR_UNSUPPORTED, GSR_ERR_WORKSPACE_TOO_SMALL, GSR_ERR_HIP = range(6)
GSR_F32, GSR_BF16 = 0, 1
GSR_NORM_NONE, GSR_NORM_RMS = 0, 1
GSR_LAYOUT_ROW_MAJOR, GSR_LAYOUT_GROUP_PLANAR = 0, 1
GSR_GRAPH_SYMMETRISE, GSR_GRAPH_ADD_SELF_LOOPS, GSR_GRAPH_GCN_NORM, GSR_GRAPH_ROWPTR_I64 = 1, 2, 4, 8
GSR_ADJ_UNIT, GSR_ADJ_GCN_SYM = 0, 1

EXPORTED = [
    "gsr_last_error", "gsr_version", "gsr_set_option", "gsr_profile_read", "gsr_profile_reset",
    "gsr_profile_class_name", "gsr_graph_create", "gsr_graph_normalize", "gsr_graph_info",
    "gsr_graph_export", "gsr_graph_destroy", "gsr_group_sparse", "gsr_spmm", "gsr_spmm_noalloc",
    "gsr_spmm_compressed_workspace",
    "gsr_spmm_compressed", "gsr_workspace_size", "gsr_layer_forward", "gsr_layer_inverse", "gsr_layer_backward",
    "gsr_step", "gsr_step_tie_stats", "gsr_step_tie_export", "gsr_walkthrough_workspace", "gsr_slot_block", "gsr_alg1_layer_forward", "gsr_alg2_layer_backward",
    "gsr_sgd_update", "gsr_adam_update",
]


class GsrError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"gsr status {status}: {message}")
        self.status = status


def gsr_last_error() -> str:
    """Message of the last call that returned a status other than GSR_OK."""
    return lib().gsr_last_error().decode()


class gsr_config_t(C.Structure):
    _fields_ = [("n", C.c_int64), ("d", C.c_int32), ("c", C.c_int32), ("l", C.c_int32), ("k", C.c_int32),
                ("dtype", C.c_int32), ("norm", C.c_int32), ("eps", C.c_float), ("layout", C.c_int32),
                ("save_indices", C.c_int32), ("tie_tol", C.c_float), ("tie_capacity", C.c_int32)]


_lib = None


def lib():
    """The loaded libgsr.so.  Raises if it has not been built (python -m paper_2603_27156_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise GsrError(-1, f"{LIB_PATH} is missing: build it with `python -m paper_2603_27156_amd.build`; "
                               "there is no CPU fallback")
        l = C.CDLL(LIB_PATH)
        l.gsr_last_error.restype = C.c_char_p
        l.gsr_version.restype = C.c_char_p
        l.gsr_profile_class_name.restype = C.c_char_p
        l.gsr_spmm_compressed_workspace.restype = C.c_size_t
        l.gsr_spmm_compressed_workspace.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        l.gsr_walkthrough_workspace.restype = C.c_size_t
        l.gsr_walkthrough_workspace.argtypes = [C.c_void_p, C.c_int32]
        _lib = l
    return _lib


def _check(st: int):
    if st != GSR_OK:
        raise GsrError(st, lib().gsr_last_error().decode())


def _stream() -> C.c_void_p:
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dp(t) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _np(a) -> C.c_void_p:
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def gsr_version() -> str:
    return lib().gsr_version().decode()


def gsr_set_option(key: str, value: int) -> None:
    _check(lib().gsr_set_option(key.encode(), C.c_int64(value)))


KERNEL_CLASSES = 11


def gsr_profile_reset() -> None:
    _check(lib().gsr_profile_reset())


def gsr_profile_read(kernel_class: int) -> Tuple[float, int]:
    """(summed milliseconds, launches) of one kernel class since the last reset."""
    ms, cnt = C.c_double(), C.c_int64()
    _check(lib().gsr_profile_read(C.c_int32(kernel_class), C.byref(ms), C.byref(cnt)))
    return ms.value, cnt.value


def gsr_profile_class_name(kernel_class: int) -> str:
    return lib().gsr_profile_class_name(C.c_int32(kernel_class)).decode()


@dataclass
class Config:
    n: int
    d: int
    c: int
    k: int
    l: int = 1
    dtype: int = GSR_F32
    norm: int = GSR_NORM_NONE
    eps: float = 1e-5
    layout: int = GSR_LAYOUT_ROW_MAJOR
    save_indices: int = 0
    tie_tol: float = 2.0 ** -12
    tie_capacity: int = 0

    @property
    def dg(self) -> int:
        return self.d // self.c

    def c_struct(self) -> gsr_config_t:
        return gsr_config_t(self.n, self.d, self.c, self.l, self.k, self.dtype, self.norm, self.eps, self.layout,
                            self.save_indices, self.tie_tol, self.tie_capacity)


class Graph:
    """Owner of a gsr_graph_t*."""

    def __init__(self, ptr: int):
        self.ptr = C.c_void_p(ptr)

    def destroy(self):
        if self.ptr:
            lib().gsr_graph_destroy(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def gsr_graph_create(rowptr: np.ndarray, colidx: np.ndarray, vals: Optional[np.ndarray] = None,
                     flags: int = GSR_GRAPH_SYMMETRISE | GSR_GRAPH_ADD_SELF_LOOPS | GSR_GRAPH_GCN_NORM,
                     n: Optional[int] = None, nnz: Optional[int] = None) -> Graph:
    """Host CSR (numpy) -> device graph.  rowptr int32 or int64 (flag set automatically)."""
    rowptr = np.ascontiguousarray(rowptr)
    if rowptr.dtype == np.int64:
        flags |= GSR_GRAPH_ROWPTR_I64
    elif rowptr.dtype == np.int32:
        flags &= ~GSR_GRAPH_ROWPTR_I64
    else:
        raise TypeError("rowptr must be int32 or int64")
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    if vals is not None:
        vals = np.ascontiguousarray(vals, dtype=np.float32)
    n = len(rowptr) - 1 if n is None else n
    nnz = len(colidx) if nnz is None else nnz
    out = C.c_void_p()
    _check(lib().gsr_graph_create(C.byref(out), C.c_int64(n), C.c_int64(nnz), _np(rowptr), _np(colidx), _np(vals),
                                  C.c_uint32(flags), _stream() if _has_cuda() else None))
    return Graph(out.value)


def _has_cuda() -> bool:
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def gsr_graph_normalize(g: Graph, mode: int) -> None:
    _check(lib().gsr_graph_normalize(g.ptr, C.c_int32(mode), _stream()))


def gsr_graph_info(g: Graph) -> dict:
    n, nnz, md, nh = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib().gsr_graph_info(g.ptr, C.byref(n), C.byref(nnz), C.byref(md), C.byref(nh)))
    return dict(n=n.value, nnz=nnz.value, max_degree=md.value, n_hub_rows=nh.value)


def gsr_graph_export(g: Graph) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    info = gsr_graph_info(g)
    rp = np.zeros(info["n"] + 1, dtype=np.int64)
    ci = np.zeros(max(1, info["nnz"]), dtype=np.int32)
    av = np.zeros(max(1, info["nnz"]), dtype=np.float32)
    _check(lib().gsr_graph_export(g.ptr, _np(rp), _np(ci), _np(av)))
    return rp, ci[:info["nnz"]], av[:info["nnz"]]


def _dtype_of(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return GSR_F32
    if t.dtype == torch.bfloat16:
        return GSR_BF16
    raise TypeError(f"unsupported tensor dtype {t.dtype}")


def gsr_group_sparse(x, k: int, norm: int = GSR_NORM_NONE, eps: float = 1e-5):
    """GS(X, k) -> (V [n,k] of x.dtype, I [n,k] int32).  x: device tensor [n, dg], last dim contiguous."""
    import torch
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1
    n, dg = x.shape
    vals = torch.empty((n, k), dtype=x.dtype, device=x.device)
    idx = torch.empty((n, k), dtype=torch.int32, device=x.device)
    _check(lib().gsr_group_sparse(_dp(x), C.c_int64(n), C.c_int32(dg), C.c_int64(x.stride(0) if n > 1 else dg),
                                  C.c_int32(k), C.c_int32(_dtype_of(x)), C.c_int32(norm), C.c_float(eps), _dp(vals),
                                  _dp(idx), _stream()))
    return vals, idx


def gsr_spmm(g: Graph, x, transpose: bool = False):
    import torch
    assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1
    n, width = x.shape
    y = torch.empty((n, width), dtype=torch.float32, device=x.device)
    _check(lib().gsr_spmm(g.ptr, _dp(x), C.c_int64(x.stride(0) if n > 1 else width), C.c_int32(width), _dp(y),
                          C.c_int64(width), C.c_int32(1 if transpose else 0), _stream()))
    return y


def gsr_spmm_noalloc(g: Graph, x, y, transpose: bool = False) -> None:
    """gsr_spmm into the caller's y, with the library's scratch in a fixed device array: nothing is allocated."""
    import torch
    for t in (x, y):
        assert t.is_cuda and t.dtype == torch.float32 and t.dim() == 2 and t.stride(1) == 1
    assert x.shape == y.shape
    n, width = x.shape
    _check(lib().gsr_spmm_noalloc(g.ptr, _dp(x), C.c_int64(x.stride(0) if n > 1 else width), C.c_int32(width), _dp(y),
                                  C.c_int64(y.stride(0) if n > 1 else width), C.c_int32(1 if transpose else 0), _stream()))


def _walkthrough_ws(g: Graph, k: int, device):
    import torch
    nbytes = lib().gsr_walkthrough_workspace(g.ptr, C.c_int32(k))
    return torch.empty(max(1, nbytes), dtype=torch.uint8, device=device), nbytes


def gsr_slot_block(g: Graph, vals, idx, dg: int, transpose: bool = False):
    """The block of the Section 4.3 / 4.4 walk-throughs: out[i, idx[i,t]] = sum_j a_ij vals[j,t] -> float32 [n, dg]."""
    import torch
    assert vals.is_cuda and idx.is_cuda and vals.dtype == torch.float32 and idx.dtype == torch.int32
    assert vals.is_contiguous() and idx.is_contiguous()
    n, k = vals.shape
    out = torch.empty((n, dg), dtype=torch.float32, device=vals.device)
    ws, nbytes = _walkthrough_ws(g, k, vals.device)
    _check(lib().gsr_slot_block(g.ptr, _dp(vals), _dp(idx), C.c_int32(k), C.c_int32(dg), C.c_int32(1 if transpose else 0),
                                _dp(out), C.c_int64(dg), _dp(ws), C.c_size_t(nbytes), _stream()))
    return out


def gsr_alg1_layer_forward(g: Graph, x1, x2, k: int):
    """One pass of the loop body of Algorithm 1 on the planes x1, x2 (float32 [n, dg], updated in place)."""
    import torch
    for x in (x1, x2):
        assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1
    assert x1.shape == x2.shape and x1.stride(0) == x2.stride(0)
    n, dg = x1.shape
    ws, nbytes = _walkthrough_ws(g, k, x1.device)
    _check(lib().gsr_alg1_layer_forward(g.ptr, C.c_int32(dg), C.c_int32(k), _dp(x1), _dp(x2),
                                        C.c_int64(x1.stride(0) if n > 1 else dg), _dp(ws), C.c_size_t(nbytes), _stream()))


def gsr_alg2_layer_backward(g: Graph, g1, g2, k: int):
    """One pass of the loop body of Algorithm 2 on the gradient planes g1, g2 (float32 [n, dg], in place)."""
    import torch
    for x in (g1, g2):
        assert x.is_cuda and x.dtype == torch.float32 and x.dim() == 2 and x.stride(1) == 1
    assert g1.shape == g2.shape and g1.stride(0) == g2.stride(0)
    n, dg = g1.shape
    ws, nbytes = _walkthrough_ws(g, k, g1.device)
    _check(lib().gsr_alg2_layer_backward(g.ptr, C.c_int32(dg), C.c_int32(k), _dp(g1), _dp(g2),
                                         C.c_int64(g1.stride(0) if n > 1 else dg), _dp(ws), C.c_size_t(nbytes), _stream()))


def gsr_sgd_update(w, dw, lr: float, weight_decay: float = 0.0):
    """w <- w - lr * (dw + weight_decay * w), in place (float32 device tensors of one shape)."""
    import torch
    assert w.is_cuda and dw.is_cuda and w.dtype == dw.dtype == torch.float32 and w.is_contiguous() and dw.is_contiguous()
    assert w.numel() == dw.numel()
    _check(lib().gsr_sgd_update(_dp(w), _dp(dw), C.c_int64(w.numel()), C.c_float(lr), C.c_float(weight_decay), _stream()))


def gsr_adam_update(w, dw, m, v, t: int, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                    weight_decay: float = 0.0):
    """One Adam step with bias correction, in place; m, v: state tensors (zero before t = 1)."""
    import torch
    for x in (w, dw, m, v):
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.numel() == w.numel()
    _check(lib().gsr_adam_update(_dp(w), _dp(dw), _dp(m), _dp(v), C.c_int64(w.numel()), C.c_int64(t), C.c_float(lr),
                                 C.c_float(beta1), C.c_float(beta2), C.c_float(eps), C.c_float(weight_decay), _stream()))


def gsr_spmm_compressed(g: Graph, vals, idx, dg: int):
    """A * scatter(V, I) -> dense float32 [n, dg]."""
    import torch
    assert vals.is_cuda and idx.is_cuda and idx.dtype == torch.int32 and vals.is_contiguous() and idx.is_contiguous()
    n, k = vals.shape
    h = torch.empty((n, dg), dtype=torch.float32, device=vals.device)
    nbytes = lib().gsr_spmm_compressed_workspace(g.ptr, C.c_int32(k), C.c_int32(dg))
    ws = torch.empty(max(1, nbytes), dtype=torch.uint8, device=vals.device)
    _check(lib().gsr_spmm_compressed(g.ptr, _dp(vals), _dp(idx), C.c_int32(k), C.c_int32(dg),
                                     C.c_int32(_dtype_of(vals)), _dp(h), _dp(ws), C.c_size_t(nbytes), _stream()))
    return h


def gsr_workspace_size(g: Graph, cfg: Config) -> Tuple[int, int]:
    """(bytes for the layer calls, bytes for gsr_step)."""
    lb, sb = C.c_size_t(), C.c_size_t()
    cs = cfg.c_struct()
    _check(lib().gsr_workspace_size(C.byref(cs), g.ptr, C.byref(lb), C.byref(sb)))
    return lb.value, sb.value


def _workspace(g: Graph, cfg: Config, workspace, step: bool, device):
    import torch
    need = gsr_workspace_size(g, cfg)[1 if step else 0]
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, workspace.numel() * workspace.element_size()


def gsr_layer_forward(g: Graph, cfg: Config, w, x_inout, workspace=None) -> None:
    ws, nb = _workspace(g, cfg, workspace, False, x_inout.device)
    cs = cfg.c_struct()
    _check(lib().gsr_layer_forward(g.ptr, C.byref(cs), _dp(w), _dp(x_inout), _dp(ws), C.c_size_t(nb), _stream()))


def gsr_layer_inverse(g: Graph, cfg: Config, w, y_inout, workspace=None) -> None:
    ws, nb = _workspace(g, cfg, workspace, False, y_inout.device)
    cs = cfg.c_struct()
    _check(lib().gsr_layer_inverse(g.ptr, C.byref(cs), _dp(w), _dp(y_inout), _dp(ws), C.c_size_t(nb), _stream()))


def gsr_layer_backward(g: Graph, cfg: Config, w, y_inout, dy_inout, dw_out, workspace=None) -> None:
    ws, nb = _workspace(g, cfg, workspace, False, y_inout.device)
    cs = cfg.c_struct()
    _check(lib().gsr_layer_backward(g.ptr, C.byref(cs), _dp(w), _dp(y_inout), _dp(dy_inout), _dp(dw_out), _dp(ws),
                                    C.c_size_t(nb), _stream()))


def gsr_step(g: Graph, cfg: Config, x0, w_all, w_out, b_out, target, loss_out, dw_all, dw_out, db_out,
             yhat_out=None, dx0_out=None, x0_rebuilt_out=None, xl_out=None, workspace=None) -> None:
    """All tensors are caller-allocated device tensors (see include/gsr.h for shapes)."""
    ws, nb = _workspace(g, cfg, workspace, True, x0.device)
    cs = cfg.c_struct()
    _check(lib().gsr_step(g.ptr, C.byref(cs), _dp(x0), _dp(w_all), _dp(w_out), _dp(b_out), _dp(target), _dp(loss_out),
                          _dp(yhat_out), _dp(dw_all), _dp(dw_out), _dp(db_out), _dp(dx0_out), _dp(x0_rebuilt_out),
                          _dp(xl_out), _dp(ws), C.c_size_t(nb), _stream()))


def gsr_step_tie_stats(g: Graph, cfg: Config, workspace) -> dict:
    """Counts of the last gsr_step with save_indices == 2 in `workspace`: rows kept, most per block, rows dropped."""
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    cs = cfg.c_struct()
    _check(lib().gsr_step_tie_stats(g.ptr, C.byref(cs), _dp(workspace), C.byref(a), C.byref(b), C.byref(c), _stream()))
    return dict(listed=a.value, max_per_block=b.value, dropped=c.value)


def gsr_step_tie_export(g: Graph, cfg: Config, workspace, layer: int, block: int):
    """(rows int32 [m], masks uint64 [m]) kept by the last save_indices == 2 step for the input of `block` of `layer`."""
    cap = cfg.tie_capacity if cfg.tie_capacity > 0 else cfg.n // 32 + 1024
    cap = (cap + 15) // 16 * 16                    # the library keeps sixteen sub-lists of cap / 16 places, rounded up
    rows = np.zeros(cap, dtype=np.int32)
    masks = np.zeros(cap, dtype=np.uint64)
    cnt = C.c_int64()
    cs = cfg.c_struct()
    _check(lib().gsr_step_tie_export(g.ptr, C.byref(cs), _dp(workspace), C.c_int32(layer), C.c_int32(block), _np(rows),
                                     _np(masks), C.byref(cnt), _stream()))
    return rows[:cnt.value].copy(), masks[:cnt.value].copy()
