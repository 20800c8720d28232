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


# ---------------------------------------------------------------------------------------------------------------
# Audits at sizes where the two sides cannot be expected to take every top-k decision alike.
#
# GS is a discontinuous function of its input: where the k-th and (k+1)-th largest entries of a row differ by less
# than the rounding difference between the two sides' versions of that row, the sides may keep different columns, and
# both selections are valid.  The audits never allow a fraction of rows to be wrong: every row that leaves the bar
# must be explained by such a provable near-tie, and in the backward the oracle is handed the other side's selection
# for exactly those rows, after which everything must agree element by element.

def f32_bar(gpu, ref):
    """Elements outside the float32 bar of the parity tests."""
    return violations(gpu, ref)[0]


def bf16_bar(gpu, ref, steps=1.0):
    """Elements outside the bar for planes stored as bf16.  The two sides round sums that differ in their last
    float32 bits, which moves a stored value by one bf16 step; a block output formed from such inputs moves by that
    step times a_ij W, on every column of the row, however small the column's own value is.  Bar: two bf16 steps of
    the reference value plus one step of the row's largest entry (times `steps` where rows are sums of more terms)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rowmax = np.abs(ref).max(axis=1, keepdims=True) if ref.ndim > 1 else np.abs(ref).max()
    return np.abs(gpu - ref) > steps * (2.0 ** -7 * np.abs(ref) + 2.0 ** -8 * rowmax)


def adjacency_pattern(og):
    import scipy.sparse as sp
    n = og.n
    return sp.csr_matrix((np.ones(len(og.ci), dtype=np.int32), og.ci, og.rp), shape=(n, n))


def row_gap(z, k):
    """Gap between the k-th and (k+1)-th largest entry of every row."""
    if k >= z.shape[1]:
        return np.full(z.shape[0], np.inf)
    s = -np.sort(-z, axis=1)
    return s[:, k - 1] - s[:, k]


def group_sum_as_the_kernel(X, C, dg, bf16=False):
    """Y_0 = sum_{j >= 2} X_j the way the kernels form it: float32, planes added in order, rounded to storage."""
    from paper_2603_27156_amd import synth as _synth
    z = X[:, dg:2 * dg].astype(np.float32)
    for j in range(2, C):
        z = z + X[:, j * dg:(j + 1) * dg].astype(np.float32)
    if bf16:
        z = _synth.to_bf16_grid(z)
    return z.astype(np.float64)


def audit_layer_forward(c: Case, X, Y, Y_ref, tag, bar=f32_bar, max_reachable=5e-2):
    """Element-wise comparison of a layer output with the oracle's, group by group.

    Group i is X_i + f_i(Y_{i-1}).  A row of Y_{i-1} can select different columns on the two sides only if its two
    versions differ by at least half its top-k gap; a row of group i can leave the bar only if it aggregates such a
    row, or a row of group i-1 that already left it.  Every other row must agree.  Returns the fraction of rows
    outside the bar; asserts that each of them is explained and that the rows a flip can reach stay few."""
    w = c.w
    dg, C = w.dg, w.c
    A = adjacency_pattern(c.og)
    bf16 = w.dtype == "bf16"
    if C > 2:
        z_gpu = group_sum_as_the_kernel(X, C, dg, bf16)
        z_ref = oracle.round_store(X[:, dg:].reshape(w.n, C - 1, dg).sum(axis=1), c.ocfg.sm) if not bf16 else \
            synth.to_bf16_grid(X[:, dg:].reshape(w.n, C - 1, dg).sum(axis=1).astype(np.float32)).astype(np.float64)
    else:
        z_gpu = z_ref = X[:, dg:2 * dg]
    prev_bad = np.zeros(w.n, dtype=bool)
    total_bad = np.zeros(w.n, dtype=bool)
    for i in range(C):
        dev = np.abs(z_gpu - z_ref).max(axis=1)
        may_flip = (row_gap(z_ref, w.k) <= 2.0 * dev) & (dev > 0)
        allowed = (A @ (may_flip | prev_bad).astype(np.int32)) > 0
        sl = slice(i * dg, (i + 1) * dg)
        rows = bar(Y[:, sl], Y_ref[:, sl]).any(axis=1)
        print(f"[{tag}] group {i}: rows that may flip {int(may_flip.sum())}, reachable {int(allowed.sum())}, "
              f"outside the bar {int(rows.sum())}, unexplained {int((rows & ~allowed).sum())}", flush=True)
        for r in np.flatnonzero(rows & ~allowed)[:4]:          # what an unexplained row looks like
            e = np.abs(Y[r, sl] - Y_ref[r, sl])
            col = int(e.argmax())
            nb = A.indices[A.indptr[r]:A.indptr[r + 1]]
            print(f"[{tag}] unexplained row {r}: degree {len(nb)}, worst column {col}: gpu {Y[r, sl][col]:.6g} ref {Y_ref[r, sl][col]:.6g}, "
                  f"row max {np.abs(Y_ref[r, sl]).max():.3g}, neighbours whose input differs {int((dev[nb] > 0).sum())}, "
                  f"largest such difference {dev[nb].max():.3g}", flush=True)
        assert not (rows & ~allowed).any(), f"group {i}: rows outside the bar that no flipped selection explains"
        assert allowed.mean() < max_reachable
        prev_bad = rows
        total_bad |= rows
        z_gpu, z_ref = Y[:, sl], Y_ref[:, sl]
    return float(total_bad.mean())


def audit_layer_backward(c: Case, W, Y, dY, tag, bar=f32_bar, dw_rtol=1e-4, max_flips=1e-3):
    """gsr_layer_backward against the oracle on the same (Y, dY), every element of the rebuilt X, of dX and of dW.

    Both sides are given the same Y, so blocks C..2 select on identical rows.  Block 1 selects on Y_0, which each side
    forms from its own rebuilt X_2..X_C: where the two Y_0 differ by rounding a row may select differently.  Each such
    row must be a provable near-tie (its gap at most twice the difference of the two versions); the oracle is then
    run again with the GPU's selection for exactly those rows (the listed-rows form of its backward), and everything
    is compared with no row set aside.  Returns the number of rows handed over."""
    import torch
    w = c.w
    dg, C, k = w.dg, w.c, w.k
    bf16 = w.dtype == "bf16"
    yb, dyb = c.to_dev(Y), c.to_dev(dY)
    dW = torch.empty((C, dg, dg), dtype=torch.float32, device=c.dev)
    gsr.gsr_layer_backward(c.gg, c.gcfg, torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).to(c.dev), yb, dyb, dW)
    Xg, dXg, dWg = c.to_host(yb), c.to_host(dyb), dW.cpu().numpy().astype(np.float64)
    Xr, dXr, dWr = oracle.layer_backward(c.og, c.ocfg, W, Y, dY)
    if C > 2:
        z_gpu = group_sum_as_the_kernel(Xg, C, dg, bf16)
        z_ref = oracle.round_store(Xr[:, dg:].reshape(w.n, C - 1, dg).sum(axis=1), oracle.STORE_F32) if not bf16 else \
            synth.to_bf16_grid(Xr[:, dg:].reshape(w.n, C - 1, dg).sum(axis=1).astype(np.float32)).astype(np.float64)
    else:
        z_gpu, z_ref = Xg[:, dg:2 * dg], Xr[:, dg:2 * dg]
    I_gpu, I_ref = oracle.gs(z_gpu, k)[1], oracle.gs(z_ref, k)[1]
    flips = (I_gpu != I_ref).any(axis=1)
    dev = np.abs(z_gpu - z_ref).max(axis=1)
    provable = row_gap(z_ref, k) <= 2.0 * dev
    print(f"[{tag}] block 1 selects differently on {int(flips.sum())} of {w.n} rows, all provable near-ties: "
          f"{bool(provable[flips].all())}", flush=True)
    assert provable[flips].all(), "a row selected differently although its two versions differ by less than half its gap"
    assert flips.mean() <= max_flips
    if flips.any():
        saved = np.zeros((C, w.n, k), dtype=np.int32)
        saved[0] = I_gpu
        listed = np.zeros((C, w.n), dtype=bool)
        listed[0] = flips
        Xr, dXr, dWr = oracle.layer_backward(c.og, c.ocfg, W, Y, dY, I_saved=saved, listed=listed)
    for name, got, ref in (("X rebuilt", Xg, Xr), ("dX", dXg, dXr)):
        bad = bar(got, ref)
        print(f"[{tag}] {name}: elements outside the bar {int(bad.sum())}, rel {rel_norm(got, ref):.2e}", flush=True)
        assert not bad.any(), name
    # dW sums n products per entry in float32 (per-wave partial sums, then a fixed tree)
    err = np.abs(dWg - dWr).max(axis=(1, 2)) / np.abs(dWr).max(axis=(1, 2))
    shown = ", ".join(f"{e:.2e}" for e in err)
    print(f"[{tag}] dW: max error per block relative to its largest entry {shown}", flush=True)
    assert (err <= dw_rtol).all()
    return int(flips.sum())
