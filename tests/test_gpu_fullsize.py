"""GPU parity at the full size of the benchmarked workloads, in the launch configuration the
benchmark times (persistent grids over all compute units, hub rows split in two passes).

The top-k selection of GS is a discontinuous function of its input: where the k-th and (k+1)-th
largest entries of a row differ by less than the rounding difference between float32 accumulation
(GPU) and float64 accumulation rounded to float32 (oracle), the two sides may keep different
columns, and both selections are valid.  Such a row changes the rows that aggregate it.  The tests
therefore compare every element at the float32 bar outside the rows such a flip can reach
(a flip needs a deviation of at least half the row's top-k gap), and bound how many rows lie
inside."""
import time

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth
from gpu_util import Case, violations, rel_norm, BF16_REL
from test_gpu_layer import run_step

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

PLANAR = gsr.GSR_LAYOUT_GROUP_PLANAR
_cases = {}


def case(name) -> Case:
    if name not in _cases:
        t = time.time()
        if name == "cfg1":
            w = synth.workload(1)
        elif name == "cfg2":
            w = synth.workload(2)
        elif name == "cfg2-bf16":
            w = synth.workload(2, dtype="bf16")
        _cases[name] = Case(w, 0, PLANAR)
        print(f"[case] {name} n={w.n} D={w.d} C={w.c} k={w.k} built in {time.time() - t:.1f}s", flush=True)
    return _cases[name]


def adjacency(c: Case):
    n = c.w.n
    return sp.csr_matrix((np.ones(len(c.og.ci), dtype=np.int32), c.og.ci, c.og.rp), shape=(n, n))


def row_gap(z, k):
    """Gap between the k-th and (k+1)-th largest entry of every row."""
    if k >= z.shape[1]:
        return np.full(z.shape[0], np.inf)
    s = -np.sort(-z, axis=1)
    return s[:, k - 1] - s[:, k]


def audit_layer_forward(c: Case, X, Y, Y_ref, tag):
    """Element-wise comparison of a layer output with the oracle's, group by group.

    Group i is X_i + f_i(Y_{i-1}).  A row of Y_{i-1} can select different columns on the two
    sides only if its two versions differ by at least half its top-k gap; a row of group i can
    leave the tolerance only if it aggregates such a row, or a row of group i-1 that already left
    it.  Every other row must agree at the float32 bar.  Returns the fraction of rows outside the
    tolerance; asserts that each of them is explained."""
    w = c.w
    dg, C = w.dg, w.c
    A = adjacency(c)
    if C > 2:
        # Y_0 as the kernel forms it (float32, planes added in order) and as the oracle does
        z_gpu = X[:, dg:2 * dg].astype(np.float32)
        for j in range(2, C):
            z_gpu = z_gpu + X[:, j * dg:(j + 1) * dg].astype(np.float32)
        z_gpu = z_gpu.astype(np.float64)
        z_ref = oracle.round_store(X[:, dg:].reshape(w.n, C - 1, dg).sum(axis=1), c.ocfg.sm)
    else:
        z_gpu = z_ref = X[:, dg:2 * dg]
    prev_bad = np.zeros(w.n, dtype=bool)
    total_bad = np.zeros(w.n, dtype=bool)
    for i in range(C):
        dev = np.abs(z_gpu - z_ref).max(axis=1)
        may_flip = row_gap(z_ref, w.k) <= 2.0 * dev + 1e-30 * (dev > 0)
        may_flip &= dev > 0
        allowed = (A @ (may_flip | prev_bad).astype(np.int32)) > 0
        sl = slice(i * dg, (i + 1) * dg)
        bad, worst = violations(Y[:, sl], Y_ref[:, sl])
        rows = bad.any(axis=1)
        print(f"[{tag}] group {i}: rows that may flip {int(may_flip.sum())}, reachable {int(allowed.sum())}, "
              f"outside tolerance {int(rows.sum())}, unexplained {int((rows & ~allowed).sum())}", flush=True)
        assert not (rows & ~allowed).any(), f"group {i}: rows outside tolerance that no flipped selection explains"
        assert allowed.mean() < 2e-2
        prev_bad = rows
        total_bad |= rows
        z_gpu, z_ref = Y[:, sl], Y_ref[:, sl]
    return float(total_bad.mean())


def test_cfg1_full_size_layer():
    c = case("cfg1")
    w = c.w
    X = c.x0_on_grid()
    for l in range(2):
        X = oracle.layer_forward(c.og, c.ocfg, c.inp.weights[l], X)
    W = c.inp.weights[2]
    Wd = torch.from_numpy(W).to(c.dev)
    Y_ref = oracle.layer_forward(c.og, c.ocfg, W, X)
    y = c.to_dev(X)
    gsr.gsr_layer_forward(c.gg, c.gcfg, Wd, y)
    frac = audit_layer_forward(c, X, c.to_host(y), Y_ref, "cfg1 fwd")
    assert frac < 1e-3

    rng = np.random.default_rng(5)
    dY = (rng.standard_normal((w.n, w.d)) * 1e-3).astype(np.float32).astype(np.float64)
    Xb_ref, dX_ref, dW_ref = oracle.layer_backward(c.og, c.ocfg, W, Y_ref, dY)
    yb, dyb = c.to_dev(Y_ref), c.to_dev(dY)
    dW = torch.empty((w.c, w.dg, w.dg), dtype=torch.float32, device=c.dev)
    gsr.gsr_layer_backward(c.gg, c.gcfg, Wd, yb, dyb, dW)
    for name, got, ref in (("X rebuilt", c.to_host(yb), Xb_ref), ("dX", c.to_host(dyb), dX_ref)):
        bad, worst = violations(got, ref)
        print(f"[cfg1 bwd] {name}: bad rows {int(bad.any(axis=1).sum())} of {w.n}, worst {worst:.2f}, "
              f"rel {rel_norm(got, ref):.2e}", flush=True)
        assert bad.any(axis=1).mean() < 2e-3
        assert rel_norm(got, ref) < 1e-3
    print(f"[cfg1 bwd] dW rel {rel_norm(dW.cpu().numpy(), dW_ref):.2e}", flush=True)
    assert rel_norm(dW.cpu().numpy(), dW_ref) < 1e-4


def test_cfg2_full_size_layer_forward_and_properties():
    c = case("cfg2")
    w = c.w
    X = c.x0_on_grid()
    W = c.inp.weights[0]
    Wd = torch.from_numpy(W).to(c.dev)
    t = time.time()
    Y_ref = oracle.layer_forward(c.og, c.ocfg, W, X)
    print(f"[cfg2] oracle layer forward {time.time() - t:.1f}s", flush=True)
    y = c.to_dev(X)
    gsr.gsr_layer_forward(c.gg, c.gcfg, Wd, y)
    Y = c.to_host(y)
    frac = audit_layer_forward(c, X, Y, Y_ref, "cfg2 fwd")
    assert frac < 5e-3
    assert rel_norm(Y, Y_ref) < 1e-3

    # bit-identical reruns, and inverse(forward(X)) returns X outside the rows a recomputed
    # selection flipped
    y2 = c.to_dev(X)
    gsr.gsr_layer_forward(c.gg, c.gcfg, Wd, y2)
    assert torch.equal(y, y2)
    gsr.gsr_layer_inverse(c.gg, c.gcfg, Wd, y2)
    Xr = c.to_host(y2)
    bad, worst = violations(Xr, X, rtol=1e-4, atol=1e-4)
    print(f"[cfg2] inverse(forward(X)): bad rows {int(bad.any(axis=1).sum())}, worst {worst:.2f}", flush=True)
    assert bad.any(axis=1).mean() < 5e-3

    # backward fused with the inverse, from the oracle's Y: the inverse recomputes GS on rebuilt
    # activations, so a few selections flip on either side; bounded in count and in norm
    rng = np.random.default_rng(5)
    dY = (rng.standard_normal((w.n, w.d)) * 1e-3).astype(np.float32).astype(np.float64)
    Xb_ref, dX_ref, dW_ref = oracle.layer_backward(c.og, c.ocfg, W, Y_ref, dY)
    yb, dyb = c.to_dev(Y_ref), c.to_dev(dY)
    dW = torch.empty((w.c, w.dg, w.dg), dtype=torch.float32, device=c.dev)
    gsr.gsr_layer_backward(c.gg, c.gcfg, Wd, yb, dyb, dW)
    for name, got, ref, frac, rel in (("X rebuilt", c.to_host(yb), Xb_ref, 5e-3, 1e-3),
                                      ("dX", c.to_host(dyb), dX_ref, 2e-2, 1e-2)):
        bad, worst = violations(got, ref)
        print(f"[cfg2 bwd] {name}: bad rows {int(bad.any(axis=1).sum())} of {w.n}, rel {rel_norm(got, ref):.2e}",
              flush=True)
        assert bad.any(axis=1).mean() < frac, name
        assert rel_norm(got, ref) < rel, name
    print(f"[cfg2 bwd] dW rel {rel_norm(dW.cpu().numpy(), dW_ref):.2e}", flush=True)
    assert rel_norm(dW.cpu().numpy(), dW_ref) < 1e-3


def test_cfg2_full_size_step_equals_chain_of_layers():
    c = case("cfg2")
    w = c.w
    L = 2
    a = run_step(c, l=L, raw=True)
    b = run_step(c, l=L, raw=True)
    for key in a:
        assert torch.equal(a[key], b[key]), key
    x = c.to_dev(c.inp.x0)
    Wd = torch.from_numpy(np.ascontiguousarray(c.inp.weights[:L])).to(c.dev)
    for l in range(L):
        gsr.gsr_layer_forward(c.gg, c.gcfg, Wd[l], x)
    assert torch.equal(x, a["XL"])
    yh = a["yhat"].cpu().numpy().astype(np.float32)
    gy = (np.float32(2.0) * (yh - c.inp.target) / np.float32(w.n)).astype(np.float32)
    dy = c.to_dev((gy[:, None] * c.inp.w_out[None, :]).astype(np.float32))
    dW = torch.empty_like(Wd)
    for l in reversed(range(L)):
        gsr.gsr_layer_backward(c.gg, c.gcfg, Wd[l], x, dy, dW[l])
    assert torch.equal(x, a["X0rec"]) and torch.equal(dW, a["dW"]) and torch.equal(dy, a["dX0"])
    # the head against the oracle's head on the same X^L is covered at small size; here the loss
    # only has to be finite and the rebuilt input close to X0 for all but flipped rows
    assert np.isfinite(float(a["loss"].item()))
    bad, worst = violations(c.to_host(a["X0rec"]), c.x0_on_grid(), rtol=1e-4, atol=1e-4)
    print(f"[cfg2 step L={L}] X0 rebuilt: bad rows {int(bad.any(axis=1).sum())}, worst {worst:.2f}", flush=True)
    assert bad.any(axis=1).mean() < 2e-2


def test_cfg1_full_size_step():
    c = case("cfg1")
    w = c.w
    L = 6
    t = time.time()
    ref = oracle.step(c.og, c.ocfg, L, c.x0_on_grid(), c.inp.weights[:L], c.inp.w_out, c.inp.b_out, c.inp.target)
    print(f"[cfg1 step L={L}] oracle {time.time() - t:.1f}s", flush=True)
    out = run_step(c, l=L)
    for key in ("yhat", "XL", "X0rec", "dW", "dwout", "dX0"):
        bad, worst = violations(out[key], ref[key])
        rows = bad.reshape(bad.shape[0], -1).any(axis=1) if bad.ndim > 1 else bad
        print(f"[cfg1 step L={L}] {key}: rel {rel_norm(out[key], ref[key]):.2e}, bad {rows.mean():.2e}, worst {worst:.1f}",
              flush=True)
    assert np.isclose(out["loss"], ref["loss"], rtol=1e-4)
    for key, rel, frac in (("yhat", 1e-3, 2e-2), ("XL", 1e-3, 2e-2), ("X0rec", 3e-2, 1e-1), ("dX0", 5e-2, 2e-1)):
        bad, _ = violations(out[key], ref[key])
        rows = bad.reshape(bad.shape[0], -1).any(axis=1)
        assert rel_norm(out[key], ref[key]) < rel, key
        assert rows.mean() < frac, key
    assert rel_norm(out["dW"], ref["dW"]) < 2e-2
    assert rel_norm(out["dwout"], ref["dwout"]) < 1e-3


def test_cfg2_bf16_full_size_layer():
    c = case("cfg2-bf16")
    w = c.w
    X = c.x0_on_grid()
    W = c.inp.weights[0]
    Y_ref = oracle.layer_forward(c.og, c.ocfg, W, X)
    y = c.to_dev(X)
    gsr.gsr_layer_forward(c.gg, c.gcfg, torch.from_numpy(W).to(c.dev), y)
    Y = c.to_host(y)
    print(f"[cfg2 bf16] layer forward rel {rel_norm(Y, Y_ref):.2e}", flush=True)
    assert rel_norm(Y, Y_ref) <= BF16_REL
    # rows no bf16 rounding tie can reach agree to one bf16 ulp
    err = np.abs(Y - Y_ref) / np.maximum(np.abs(Y_ref), 1e-3)
    print(f"[cfg2 bf16] elements beyond 2^-7 relative: {(err > 2.0 ** -7).mean():.2e}", flush=True)
    assert (err > 2.0 ** -7).mean() < 5e-2


def test_cfg1_full_depth_step_in_the_three_index_modes():
    """cfg1 at its full depth (L = 28) against plain back-propagation from stored activations (the oracle's variant
    1, the definition of the gradients), in the three modes of the inverse sweep:
    all column sets of the forward sweep kept (Section 4.2), kept for near-tie rows only, nothing kept.
    With kept sets the inverse is continuous in its input: the input comes back to float32 rounding on every row and
    every layer's weight gradient agrees with the kept-all run to rounding; selecting again everywhere loses rows
    of the input at this depth and its gradients drift, by the figures printed and bounded here.  Against the
    oracle the comparison is in norm: the two forward sweeps differ where a near-tie was decided differently."""
    c = case("cfg1")
    w = c.w
    x0 = c.x0_on_grid()
    t = time.time()
    ref = oracle.step(c.og, c.ocfg, w.l, x0, c.inp.weights, c.inp.w_out, c.inp.b_out, c.inp.target, variant=1)
    print(f"[cfg1 L={w.l}] oracle, stored activations: {time.time() - t:.1f}s", flush=True)
    keep = {}
    saved, again = run_step(c, save_indices=1), run_step(c)
    listed = run_step(c, save_indices=2, tie_tol=2.0 ** -12, keep=keep)
    st = gsr.gsr_step_tie_stats(c.gg, keep["cfg"], keep["ws"])
    scale = np.abs(saved["XL"]).max()
    err = {name: np.abs(r["X0rec"] - x0).max(axis=1) for name, r in (("all", saved), ("near-ties", listed), ("none", again))}
    for name, e in err.items():
        print(f"[cfg1 L={w.l}] kept {name}: max|X0 rebuilt - X0| {e.max():.3g}, rows above 1e-3: {np.mean(e > 1e-3):.4f}", flush=True)
    print(f"[cfg1 L={w.l}] near-tie rows kept: {st['listed']} of {w.n * w.c * w.l} ({st['listed'] / (w.n * w.c * w.l):.4%}), "
          f"most in one block {st['max_per_block']}, dropped {st['dropped']}; scale {scale:.3g}", flush=True)
    assert st["dropped"] == 0 and st["listed"] < 0.02 * w.n * w.c * w.l
    assert err["all"].max() <= 1e-4 * max(1.0, scale) and err["near-ties"].max() <= 1e-4 * max(1.0, scale)
    assert np.abs(ref["X0rec"] - x0).max() == 0.0
    # the near-tie list against all sets kept, layer by layer: same forward sweep, so rounding only
    per_layer = [rel_norm(listed["dW"][l], saved["dW"][l]) for l in range(w.l)]
    print(f"[cfg1 L={w.l}] near-ties vs all kept: dW per layer max {max(per_layer):.2e}, dX0 {rel_norm(listed['dX0'], saved['dX0']):.2e}",
          flush=True)
    assert max(per_layer) <= 1e-5 and rel_norm(listed["dX0"], saved["dX0"]) <= 1e-5
    assert np.array_equal(listed["XL"], saved["XL"]) and listed["loss"] == saved["loss"]
    # nothing kept: measured drift of the gradients (the reason the near-tie list exists)
    per_layer0 = [rel_norm(again["dW"][l], saved["dW"][l]) for l in range(w.l)]
    print(f"[cfg1 L={w.l}] nothing kept vs all kept: dW per layer max {max(per_layer0):.2e} (layer 0 {per_layer0[0]:.2e}), "
          f"dX0 {rel_norm(again['dX0'], saved['dX0']):.2e}", flush=True)
    assert max(per_layer0) <= 2e-2 and rel_norm(again["dX0"], saved["dX0"]) <= 0.3
    # against the definition (oracle, stored activations)
    for name, r in (("all", saved), ("near-ties", listed)):
        for key in ("yhat", "XL", "dW", "dwout", "dX0"):
            print(f"[cfg1 L={w.l}] kept {name} vs oracle stored: {key} rel {rel_norm(r[key], ref[key]):.2e}", flush=True)
        assert np.isclose(r["loss"], ref["loss"], rtol=1e-3)
        for key, bound in (("yhat", 1e-2), ("XL", 1e-2), ("dW", 5e-2), ("dwout", 1e-2), ("dX0", 1e-1)):
            assert rel_norm(r[key], ref[key]) <= bound, (name, key)


def test_cfg4_full_size_sampled_rows_and_properties():
    """cfg4 (8M nodes, D 256, C 8, k 8, bf16 storage, int64 row pointers) in the launch
    configuration the benchmark uses.  The oracle cannot run a layer on 8M x 256 doubles inside
    the test budget, so block 1 of the first layer is checked on sampled rows, each computed by
    the oracle's operators from its own neighbourhood (GS of the neighbours' Y_0 rows, aggregation
    over the row's stored edges, weight product in float64); reruns must be bit-identical and
    inverse(forward(X)) must return X to bf16 rounding."""
    w = synth.workload(4)
    t = time.time()
    inp = synth.make_inputs(w, 0)
    assert inp.rowptr.dtype == np.int64
    gg = gsr.gsr_graph_create(inp.rowptr, inp.colidx)
    og = oracle.graph_build(inp.rowptr, inp.colidx)
    print(f"[cfg4] n={w.n} nnz={og.nnz} built in {time.time() - t:.1f}s", flush=True)
    dev = torch.device("cuda:0")
    dg, C, k = w.dg, w.c, w.k
    cfg = gsr.Config(n=w.n, d=w.d, c=C, k=k, l=1, dtype=gsr.GSR_BF16, norm=gsr.GSR_NORM_RMS, eps=1e-5, layout=PLANAR)
    x = torch.from_numpy(inp.x0).to(dev).to(torch.bfloat16).view(w.n, C, dg).permute(1, 0, 2).contiguous()
    W = inp.weights[0]
    Wd = torch.from_numpy(W).to(dev)
    y = x.clone()
    gsr.gsr_layer_forward(gg, cfg, Wd, y)
    y2 = x.clone()
    gsr.gsr_layer_forward(gg, cfg, Wd, y2)
    assert torch.equal(y, y2)
    gsr.gsr_layer_inverse(gg, cfg, Wd, y2)
    diff = (y2.float() - x.float()).abs().amax(dim=(0, 2))           # per row
    frac = float((diff > 0.05).float().mean().item())
    print(f"[cfg4] inverse(forward(X)): rows off by more than 0.05: {frac:.2e}", flush=True)
    assert frac < 4e-2          # bf16 near-ties re-selected differently; everything else to rounding

    # sampled rows of block 1: the two first tiles (they hold the split rows) and 3,000 random rows
    rng = np.random.default_rng(11)
    S = np.unique(np.concatenate([np.arange(32), rng.integers(0, w.n, 3000)]))
    deg = og.rp[S + 1] - og.rp[S]
    cols = np.concatenate([og.ci[og.rp[i]:og.rp[i + 1]] for i in S])
    vals = np.concatenate([og.av[og.rp[i]:og.rp[i + 1]] for i in S])
    nodes, inv = np.unique(cols, return_inverse=True)                # neighbourhood of the sample (holds S: self-loops)
    xs = synth.to_bf16_grid(inp.x0[nodes]).astype(np.float64)
    y0 = oracle.round_store(xs[:, dg:].reshape(len(nodes), C - 1, dg).sum(axis=1), oracle.STORE_BF16)
    V, I, _ = oracle.gs(y0, k, oracle.NORM_RMS, 1e-5, oracle.STORE_BF16)
    # a CSR over the neighbourhood's local numbering with the sampled rows' edges only
    pos = np.searchsorted(nodes, S)
    rp = np.zeros(len(nodes) + 1, dtype=np.int64)
    rp[pos + 1] = deg
    rp = np.cumsum(rp)
    order = np.argsort(pos, kind="stable")                           # S is sorted, so pos is: identity
    assert np.array_equal(order, np.arange(len(S)))
    sub = oracle.graph_from_csr(rp, inv.astype(np.int32), vals)
    H = oracle.aggregate(sub, V, I, dg)[pos]
    ref = oracle.round_store(xs[pos, :dg] + H @ W[0].astype(np.float64), oracle.STORE_BF16)
    got = y[0].index_select(0, torch.from_numpy(S).to(dev)).float().cpu().numpy().astype(np.float64)
    rel = rel_norm(got, ref)
    ulp_off = np.abs(got - ref) > 2.0 ** -7 * np.maximum(np.abs(ref), 2.0 ** -6)
    print(f"[cfg4] block 1 on {len(S)} sampled rows (max degree {int(deg.max())}): rel {rel:.2e}, "
          f"elements off by more than one bf16 ulp {ulp_off.mean():.2e}", flush=True)
    assert rel <= BF16_REL
    assert ulp_off.mean() < 2e-2
    del x, y, y2
    torch.cuda.empty_cache()


def test_cfg2_full_size_walkthrough_layers():
    """Algorithms 1 and 2 as the walk-throughs print them, on two planes of the 1M-node workload.  Rows whose
    second selection could differ between float32 and float64 sums (and the rows that aggregate them) are
    counted; everything else is compared element by element."""
    from oracle import literal
    c = case("cfg2")
    w = c.w
    X = c.x0_on_grid()
    dg, k = w.dg, w.k
    X1, X2 = np.ascontiguousarray(X[:, :dg]), np.ascontiguousarray(X[:, dg:2 * dg])
    x1 = torch.from_numpy(X1.astype(np.float32)).to(c.dev)
    x2 = torch.from_numpy(X2.astype(np.float32)).to(c.dev)
    gsr.gsr_alg1_layer_forward(c.gg, x1, x2, k)
    t = time.time()
    w1, w2, _ = literal.alg1_layer_forward(c.og, X1, X2, k)
    print(f"[walkthrough] oracle Alg. 1 layer {time.time() - t:.1f}s", flush=True)
    for name, got, want, frac in (("x2", x2.cpu().numpy(), w2, 1e-5), ("x1", x1.cpu().numpy(), w1, 2e-3)):
        bad, worst = violations(got, want)
        print(f"[walkthrough alg1] {name}: rows outside tolerance {int(bad.any(axis=1).sum())} of {w.n}, "
              f"rel {rel_norm(got, want):.2e}", flush=True)
        assert bad.any(axis=1).mean() <= frac and rel_norm(got, want) < 1e-3
    assert (np.count_nonzero(x1.cpu().numpy(), axis=1) <= 2 * k).all()
    rng = np.random.default_rng(9)
    G1 = (rng.standard_normal((w.n, dg)) * 1e-3).astype(np.float32)
    G2 = (rng.standard_normal((w.n, dg)) * 1e-3).astype(np.float32)
    g1, g2 = torch.from_numpy(G1).to(c.dev), torch.from_numpy(G2).to(c.dev)
    gsr.gsr_alg2_layer_backward(c.gg, g1, g2, k)
    v1, v2, _ = literal.alg2_layer_backward(c.og, G1, G2, k)
    for name, got, want in (("g1", g1.cpu().numpy(), v1), ("g2", g2.cpu().numpy(), v2)):
        bad, worst = violations(got, want)
        print(f"[walkthrough alg2] {name}: rows outside tolerance {int(bad.any(axis=1).sum())} of {w.n}, "
              f"rel {rel_norm(got, want):.2e}", flush=True)
        assert bad.any(axis=1).mean() < 2e-3 and rel_norm(got, want) < 1e-2
        assert (np.count_nonzero(got, axis=1) <= k).all()
