"""Shared helpers of the GPU parity tests: build the same workload for the oracle and for the
HIP library, and compare tensors at the stated tolerance."""
from __future__ import annotations

import numpy as np

import oracle
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth

# float32 bar of the parity tests: |gpu - ref| <= ATOL * min(1, rms(ref)) + RTOL * |ref|.
# Never looser than rtol 1e-4 / atol 1e-5; the atol term shrinks with the tensor's scale so that
# gradients of magnitude 1e-7 (loss averaged over 1e6 nodes) are still compared meaningfully.
RTOL, ATOL = 1e-4, 1e-5
# bf16 storage: 1e-2 relative in norm per tensor
BF16_REL = 1e-2


def violations(gpu: np.ndarray, ref: np.ndarray, rtol=RTOL, atol=ATOL):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
    tol = atol * min(1.0, rms) + rtol * np.abs(ref)
    err = np.abs(gpu - ref)
    bad = err > tol
    worst = float((err / np.maximum(tol, 1e-300)).max()) if ref.size else 0.0
    return bad, worst


def assert_close(name, gpu, ref, rtol=RTOL, atol=ATOL, allow_rows=None):
    """allow_rows: boolean mask over the first axis of rows excluded from the comparison
    (rows a proven near-tie of the top-k selection has touched)."""
    bad, worst = violations(gpu, ref, rtol, atol)
    if allow_rows is not None:
        bad = bad & ~allow_rows.reshape((-1,) + (1,) * (bad.ndim - 1))
    assert not bad.any(), f"{name}: {int(bad.sum())} of {bad.size} elements outside tolerance (worst {worst:.2f}x)"


def rel_norm(gpu, ref):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(gpu - ref) / max(np.linalg.norm(ref), 1e-300))


NORM = {"none": (oracle.NORM_NONE, gsr.GSR_NORM_NONE), "rms": (oracle.NORM_RMS, gsr.GSR_NORM_RMS)}


class Case:
    """One workload instantiated on both sides."""

    def __init__(self, w: synth.GsrWorkload, seed: int = 0, layout=gsr.GSR_LAYOUT_ROW_MAJOR):
        import torch
        self.w = w
        self.inp = synth.make_inputs(w, seed)
        self.og = oracle.graph_build(self.inp.rowptr, self.inp.colidx)
        self.gg = gsr.gsr_graph_create(self.inp.rowptr, self.inp.colidx)
        sm = oracle.STORE_BF16 if w.dtype == "bf16" else oracle.STORE_F32
        self.ocfg = oracle.Cfg(w.d, w.c, w.k, NORM[w.norm][0], 1e-5, sm)
        self.gcfg = gsr.Config(n=w.n, d=w.d, c=w.c, k=w.k, l=w.l,
                               dtype=gsr.GSR_BF16 if w.dtype == "bf16" else gsr.GSR_F32,
                               norm=NORM[w.norm][1], eps=1e-5, layout=layout)
        self.tdtype = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.dev = torch.device("cuda:0")

    # --- layout helpers: the oracle always works on N x D row-major
    def to_dev(self, x_rowmajor: np.ndarray):
        import torch
        t = torch.from_numpy(np.ascontiguousarray(x_rowmajor, dtype=np.float32)).to(self.dev).to(self.tdtype)
        if self.gcfg.layout == gsr.GSR_LAYOUT_GROUP_PLANAR:
            n, d = t.shape
            t = t.view(n, self.w.c, self.w.dg).permute(1, 0, 2).contiguous()
        return t

    def to_host(self, t) -> np.ndarray:
        import torch
        if self.gcfg.layout == gsr.GSR_LAYOUT_GROUP_PLANAR:
            t = t.permute(1, 0, 2).reshape(self.w.n, self.w.d)
        return t.to(torch.float32).cpu().numpy().astype(np.float64)

    def x0_on_grid(self) -> np.ndarray:
        """X0 as the storage type holds it (float32, or rounded to bf16)."""
        x = self.inp.x0
        return (synth.to_bf16_grid(x) if self.w.dtype == "bf16" else x).astype(np.float64)


def near_tie_rows(Z: np.ndarray, k: int, tau: float) -> np.ndarray:
    """Rows of Z whose top-k boundary is a near-tie: gap between the k-th kept and the best
    rejected value <= tau * max|row|.  Only such rows may legitimately select differently when
    Z itself differs by rounding."""
    if k >= Z.shape[1]:
        return np.zeros(Z.shape[0], dtype=bool)
    s = -np.sort(-Z, axis=1)
    gap = s[:, k - 1] - s[:, k]
    return gap <= tau * np.abs(Z).max(axis=1)
