"""ctypes front-end of the CPU oracle (oracle/gsr_oracle.c).  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this package: only tests/, the smoke check and
the cpu_baseline leg of bench.py do.  It has no code in common with the HIP library.
Every array crossing into C is float64 / int64 / int32 / float32 numpy, C-contiguous.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gsr_oracle.c")
_LIB = os.path.join(_HERE, "libgsr_oracle.so")

NORM_NONE, NORM_RMS = 0, 1
STORE_F64, STORE_F32, STORE_BF16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over rows, no fused multiply-add)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_graph_build.restype = C.c_int64
        _lib.orc_round_store.restype = C.c_double
        _lib.orc_round_store.argtypes = [C.c_double, C.c_int]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


@dataclass
class Graph:
    """Normalised adjacency in CSR plus its transpose."""
    n: int
    rp: np.ndarray
    ci: np.ndarray
    av: np.ndarray
    trp: np.ndarray
    tci: np.ndarray
    tav: np.ndarray

    @property
    def nnz(self) -> int:
        return int(self.rp[-1])


def graph_from_csr(rp, ci, av) -> Graph:
    """Wrap a ready CSR (any values, e.g. the paper's unnormalised 4x4 example)."""
    rp = np.ascontiguousarray(rp, dtype=np.int64)
    ci = np.ascontiguousarray(ci, dtype=np.int32)
    av = np.ascontiguousarray(av, dtype=np.float32)
    n = len(rp) - 1
    trp = np.zeros(n + 1, dtype=np.int64)
    tci = np.zeros(max(1, len(ci)), dtype=np.int32)
    tav = np.zeros(max(1, len(ci)), dtype=np.float32)
    lib().orc_transpose(C.c_int64(n), _p(rp), _p(ci), _p(av), _p(trp), _p(tci), _p(tav))
    return Graph(n, rp, ci, av, trp, tci[:len(ci)], tav[:len(ci)])


def graph_build(rowptr, colidx) -> Graph:
    """Symmetrise + self-loops + GCN symmetric normalisation of a directed CSR."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    n = len(rowptr) - 1
    cap = 2 * len(colidx) + n
    rp = np.zeros(n + 1, dtype=np.int64)
    ci = np.zeros(max(1, cap), dtype=np.int32)
    av = np.zeros(max(1, cap), dtype=np.float32)
    nnz = lib().orc_graph_build(C.c_int64(n), _p(rowptr), _p(colidx), _p(rp), _p(ci), _p(av))
    if nnz < 0:
        raise ValueError("malformed CSR")
    return graph_from_csr(rp, ci[:nnz].copy(), av[:nnz].copy())


def spmm(g: Graph, X, transpose: bool = False):
    X = _f64(X)
    n, width = X.shape
    Y = np.zeros_like(X)
    rp, ci, av = (g.trp, g.tci, g.tav) if transpose else (g.rp, g.ci, g.av)
    lib().orc_spmm(C.c_int64(n), _p(rp), _p(ci), _p(av), _p(X), C.c_int64(width), C.c_int(width),
                   _p(Y), C.c_int64(width))
    return Y


def gs(Z, k: int, norm: int = NORM_NONE, eps: float = 1e-5, sm: int = STORE_F64):
    """GS(Z, k) -> (V [n,k] float64, I [n,k] int32 ascending, r [n])."""
    Z = _f64(Z)
    n, dg = Z.shape
    V = np.zeros((n, k), dtype=np.float64)
    I = np.zeros((n, k), dtype=np.int32)
    r = np.zeros(n, dtype=np.float64)
    lib().orc_gs(_p(Z), C.c_int64(dg), C.c_int64(n), C.c_int(dg), C.c_int(k), C.c_int(norm),
                 C.c_double(eps), C.c_int(sm), _p(V), _p(I), _p(r))
    return V, I, r


def gs_near_tie(Z, k: int, tol: float):
    """Rows whose top-k boundary is a near-tie: v_k - v_(k+1) <= tol * max|row| in float32 -> bool [n]."""
    Z = _f64(Z)
    n, dg = Z.shape
    out = np.zeros(n, dtype=np.uint8)
    lib().orc_gs_near_tie(_p(Z), C.c_int64(dg), C.c_int64(n), C.c_int(dg), C.c_int(k), C.c_float(tol), _p(out))
    return out.astype(bool)


def aggregate(g: Graph, V, I, dg: int):
    """A * scatter(V, I) -> [n, dg]."""
    V = _f64(V)
    I = np.ascontiguousarray(I, dtype=np.int32)
    n, k = V.shape
    H = np.zeros((n, dg), dtype=np.float64)
    lib().orc_aggregate(C.c_int64(n), _p(g.rp), _p(g.ci), _p(g.av), _p(V), _p(I), C.c_int(k),
                        C.c_int(dg), _p(H))
    return H


@dataclass
class Cfg:
    d: int
    c: int
    k: int
    norm: int = NORM_NONE
    eps: float = 1e-5
    sm: int = STORE_F64

    @property
    def dg(self):
        return self.d // self.c


def _cfg_args(cfg: Cfg):
    return (C.c_int(cfg.d), C.c_int(cfg.c), C.c_int(cfg.k), C.c_int(cfg.norm), C.c_double(cfg.eps),
            C.c_int(cfg.sm))


def layer_forward(g: Graph, cfg: Cfg, W, X):
    """eq. (6): returns Y [n, D].  W: [C, dg, dg]."""
    Y = _f64(X).copy()
    W = _f64(W)
    lib().orc_layer_forward(C.c_int64(g.n), _p(g.rp), _p(g.ci), _p(g.av), *_cfg_args(cfg), _p(W), _p(Y),
                            None, None, None, None, None, C.c_float(0.0))
    return Y


def layer_inverse(g: Graph, cfg: Cfg, W, Y):
    """eq. (7): returns X [n, D]."""
    X = _f64(Y).copy()
    W = _f64(W)
    lib().orc_layer_inverse(C.c_int64(g.n), _p(g.rp), _p(g.ci), _p(g.av), *_cfg_args(cfg), _p(W), _p(X))
    return X


def layer_backward(g: Graph, cfg: Cfg, W, Y, dY, I_saved=None, listed=None):
    """Inverse interleaved with backward.  Returns (X, dX, dW[C,dg,dg]).  I_saved [C, n, k]
    int32: indices kept from the forward pass, used instead of selecting again; with listed
    [C, n] (bool) only by the listed rows."""
    X = _f64(Y).copy()
    dX = _f64(dY).copy()
    W = _f64(W)
    dW = np.zeros((cfg.c, cfg.dg, cfg.dg), dtype=np.float64)
    lib().orc_layer_backward(C.c_int64(g.n), _p(g.rp), _p(g.ci), _p(g.av), _p(g.trp), _p(g.tci), _p(g.tav),
                             *_cfg_args(cfg), _p(W), _p(X), _p(dX), _p(dW),
                             _p(np.ascontiguousarray(I_saved, dtype=np.int32)) if I_saved is not None else None,
                             _p(np.ascontiguousarray(listed, dtype=np.uint8)) if listed is not None else None)
    return X, dX, dW


def layer_backward_stored(g: Graph, cfg: Cfg, W, X, dY):
    """Plain back-propagation from the stored layer input.  Returns (dX, dW)."""
    X = _f64(X)
    dX = _f64(dY).copy()
    W = _f64(W)
    dW = np.zeros((cfg.c, cfg.dg, cfg.dg), dtype=np.float64)
    lib().orc_layer_backward_stored(C.c_int64(g.n), _p(g.rp), _p(g.ci), _p(g.av), _p(g.trp), _p(g.tci),
                                    _p(g.tav), *_cfg_args(cfg), _p(W), _p(X), _p(dX), _p(dW))
    return dX, dW


def head(X, w, b, target, sm: int = STORE_F64):
    """Returns dict(loss, yhat, dX, dw, db)."""
    X = _f64(X)
    n, d = X.shape
    w = _f64(w)
    target = _f64(target)
    loss = C.c_double(0.0)
    db = C.c_double(0.0)
    yhat = np.zeros(n, dtype=np.float64)
    dX = np.zeros_like(X)
    dw = np.zeros(d, dtype=np.float64)
    lib().orc_head(C.c_int64(n), C.c_int(d), C.c_int(sm), _p(X), _p(w), C.c_double(b), _p(target),
                   C.byref(loss), _p(yhat), _p(dX), _p(dw), C.byref(db))
    return dict(loss=loss.value, yhat=yhat, dX=dX, dw=dw, db=db.value)


def step(g: Graph, cfg: Cfg, L: int, X0, W, w_out, b_out, target, variant: int = 0,
         want=("yhat", "XL", "X0rec", "dW", "dwout", "dX0"), tie_tol: float = 0.0):
    """One training step.  variant 0: inverse interleaved with backward; 1: stored activations;
    2: as 0 with the indices of the forward sweep kept and reused (Section 4.2); 3: as 2 for the
    rows that selected at a near-tie (gs_near_tie with tie_tol) only.
    Returns dict(loss, yhat, XL, X0rec, dW [L,C,dg,dg], dwout, dbout, dX0, n_listed); with "ties" / "I" in want also
    the near-tie flags [L,C,n] (variant 3) and the indices of the forward sweep [L,C,n,k] (variants 2, 3)."""
    X0 = _f64(X0)
    n, d = X0.shape
    W = _f64(W)
    assert W.shape[0] >= L
    W = np.ascontiguousarray(W[:L])
    w_out = _f64(w_out)
    target = _f64(target)
    out = dict(
        yhat=np.zeros(n) if "yhat" in want else None,
        XL=np.zeros((n, d)) if "XL" in want else None,
        X0rec=np.zeros((n, d)) if "X0rec" in want else None,
        dW=np.zeros((L, cfg.c, cfg.dg, cfg.dg)) if "dW" in want else None,
        dwout=np.zeros(d) if "dwout" in want else None,
        dX0=np.zeros((n, d)) if "dX0" in want else None,
        ties=np.zeros((L, cfg.c, n), dtype=np.uint8) if "ties" in want else None,
        I=np.zeros((L, cfg.c, n, cfg.k), dtype=np.int32) if "I" in want else None,
    )
    loss = C.c_double(0.0)
    db = C.c_double(0.0)
    n_listed = C.c_int64(0)
    rc = lib().orc_step(C.c_int64(n), _p(g.rp), _p(g.ci), _p(g.av), C.c_int(cfg.d), C.c_int(cfg.c),
                        C.c_int(L), C.c_int(cfg.k), C.c_int(cfg.norm), C.c_double(cfg.eps), C.c_int(cfg.sm),
                        _p(X0), _p(W), _p(w_out), C.c_double(b_out), _p(target), C.c_int(variant),
                        C.c_float(tie_tol), C.byref(n_listed), _p(out["ties"]), _p(out["I"]), C.byref(loss), _p(out["yhat"]), _p(out["XL"]), _p(out["X0rec"]), _p(out["dW"]),
                        _p(out["dwout"]), C.byref(db), _p(out["dX0"]))
    if rc != 0:
        raise MemoryError("orc_step failed")
    out["loss"] = loss.value
    out["dbout"] = db.value
    out["n_listed"] = n_listed.value
    return out


def num_threads() -> int:
    return int(lib().orc_num_threads())


def round_store(x, sm: int):
    """Elementwise rounding to the storage precision, as the oracle applies at stores."""
    x = np.asarray(x, dtype=np.float64)
    if sm == STORE_F64:
        return x.copy()
    if sm == STORE_F32:
        return x.astype(np.float32).astype(np.float64)
    f = np.vectorize(lambda v: lib().orc_round_store(float(v), sm), otypes=[np.float64])
    return f(x)
