"""Groups wider than one 64-column tile: D/C = 128, 192, 256, the widths of the paper's own models (Section 5: hidden
256 or 384 in two groups; Algorithm 1 splits into two).  They run as D/C / 64 column blocks through the 64-column
kernels with GS over the whole row, and are compared with the oracle like every other width."""
import numpy as np
import pytest

import oracle
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth
from gpu_util import Case, assert_close, rel_norm, BF16_REL
from test_gpu_layer import run_step, ROW, PLANAR

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def wide_case(n, d, c, k, l, norm="rms", layout=ROW, dtype="f32", base=2, seed=0):
    w = synth.scaled(synth.workload(base), n, l=l, d=d, c=c, k=k, norm=norm, dtype=dtype)
    return Case(w, seed, layout)


@pytest.mark.parametrize("n,d,c,k,norm,layout", [
    (3001, 256, 2, 16, "rms", ROW),          # D/C 128
    (2049, 384, 2, 32, "rms", PLANAR),       # D/C 192: 100 layers x 384 hidden in two groups is the paper's Table 2 model
    (1500, 384, 2, 4, "none", ROW),
    (1000, 512, 2, 64, "rms", PLANAR),       # D/C 256
    (2500, 384, 3, 16, "rms", PLANAR),       # D/C 128, three groups (a Y_0 plane is formed)
    (13, 256, 2, 128, "rms", ROW),           # fewer rows than a tile, k = D/C keeps everything
])
def test_wide_layer_forward_inverse_backward(n, d, c, k, norm, layout):
    cs = wide_case(n, d, c, k, 2, norm, layout)
    w = cs.w
    W = cs.inp.weights[0]
    assert W.shape == (c, d // c, d // c)
    Wd = torch.from_numpy(W).to(cs.dev)
    X = oracle.layer_forward(cs.og, cs.ocfg, cs.inp.weights[1], cs.x0_on_grid())      # a realistic layer input
    Y_ref = oracle.layer_forward(cs.og, cs.ocfg, W, X)
    y = cs.to_dev(X)
    gsr.gsr_layer_forward(cs.gg, cs.gcfg, Wd, y)
    assert_close("Y", cs.to_host(y), Y_ref)
    X_ref = oracle.layer_inverse(cs.og, cs.ocfg, W, Y_ref)
    x = cs.to_dev(Y_ref)
    gsr.gsr_layer_inverse(cs.gg, cs.gcfg, Wd, x)
    assert_close("X rebuilt", cs.to_host(x), X_ref)
    assert_close("inverse(forward(X)) vs X", cs.to_host(x), X, rtol=1e-4, atol=1e-4)
    rng = np.random.default_rng(17)
    dY = (rng.standard_normal((w.n, w.d)) * 1e-3).astype(np.float32).astype(np.float64)
    Xb_ref, dX_ref, dW_ref = oracle.layer_backward(cs.og, cs.ocfg, W, Y_ref, dY)
    yb, dyb = cs.to_dev(Y_ref), cs.to_dev(dY)
    dW = torch.empty((w.c, w.dg, w.dg), dtype=torch.float32, device=cs.dev)
    gsr.gsr_layer_backward(cs.gg, cs.gcfg, Wd, yb, dyb, dW)
    assert_close("X rebuilt (backward)", cs.to_host(yb), Xb_ref)
    assert_close("dX", cs.to_host(dyb), dX_ref)
    assert_close("dW", dW.cpu().numpy(), dW_ref)
    assert torch.equal(yb, x)


@pytest.mark.parametrize("n,d,c,k,l,layout,save", [(3001, 384, 2, 16, 3, PLANAR, 0), (2049, 256, 2, 8, 3, ROW, 1),
                                                   (2500, 384, 3, 16, 2, ROW, 1), (4001, 384, 2, 64, 2, PLANAR, 0)])
def test_wide_step_against_oracle(n, d, c, k, l, layout, save):
    # (with nothing kept the inverse selects again on rebuilt rows: seeds where neither side meets a near-tie that the
    # other decides differently; at full size that case is handled by the audits of test_gpu_fullsize.py)
    cs = wide_case(n, d, c, k, l, "rms", layout, seed=0 if save else 1)
    w = cs.w
    ref = oracle.step(cs.og, cs.ocfg, w.l, cs.x0_on_grid(), cs.inp.weights, cs.inp.w_out, cs.inp.b_out, cs.inp.target,
                      variant=2 if save else 0)
    out = run_step(cs, save_indices=save)
    assert np.isclose(out["loss"], ref["loss"], rtol=1e-4)
    for key in ("yhat", "XL", "X0rec", "dW", "dwout", "dX0"):
        assert_close(key, out[key], ref[key])
    assert_close("X0 rebuilt vs X0", out["X0rec"], cs.x0_on_grid(), rtol=1e-4, atol=1e-4)
    a, b = run_step(cs, raw=True, save_indices=save), run_step(cs, raw=True, save_indices=save)
    for key in a:
        assert torch.equal(a[key], b[key]), key


def test_wide_step_with_the_weight_gradient_in_a_pass_of_its_own():
    """float32 graphs with at least as many tiles as resident waves run a block's backward as two kernels (inverse, then
    dW = H^T dY from H kept in memory); a small persistent grid brings a 3,001-node graph into that regime."""
    gsr.gsr_set_option("max_workgroups", 8)
    try:
        cs = wide_case(3001, 384, 2, 16, 2, "rms", PLANAR)
        w = cs.w
        ref = oracle.step(cs.og, cs.ocfg, w.l, cs.x0_on_grid(), cs.inp.weights, cs.inp.w_out, cs.inp.b_out, cs.inp.target, variant=2)
        out = run_step(cs, save_indices=1)
        for key in ("yhat", "XL", "X0rec", "dW", "dwout", "dX0"):
            assert_close(key, out[key], ref[key])
        # and the layer call: the rebuilt input equals the plain inverse's bit for bit
        W = cs.inp.weights[0]
        Wd = torch.from_numpy(W).to(cs.dev)
        Y = oracle.layer_forward(cs.og, cs.ocfg, W, cs.x0_on_grid())
        rng = np.random.default_rng(2)
        dY = (rng.standard_normal((w.n, w.d)) * 1e-3).astype(np.float32).astype(np.float64)
        Xb_ref, dX_ref, dW_ref = oracle.layer_backward(cs.og, cs.ocfg, W, Y, dY)
        yb, dyb, x = cs.to_dev(Y), cs.to_dev(dY), cs.to_dev(Y)
        dW = torch.empty((w.c, w.dg, w.dg), dtype=torch.float32, device=cs.dev)
        gsr.gsr_layer_backward(cs.gg, cs.gcfg, Wd, yb, dyb, dW)
        gsr.gsr_layer_inverse(cs.gg, cs.gcfg, Wd, x)
        assert torch.equal(yb, x)
        assert_close("dW", dW.cpu().numpy(), dW_ref)
        assert_close("dX", cs.to_host(dyb), dX_ref)
    finally:
        gsr.gsr_set_option("max_workgroups", 0)


@pytest.mark.parametrize("c,k,save", [(2, 16, 0), (2, 16, 1), (3, 8, 1), (2, 40, 0)])
def test_wide_groups_on_long_rows(c, k, save):
    """The Table-1-shaped graph (every row through the first pass) scaled down, with the paper's model split: 384
    channels in two groups of 192 (also three of 128).  The first pass over the records of such a group runs once for
    all its column blocks, value by value: the step with nothing kept and with all column sets kept, then the layer
    calls on the same graph."""
    w = synth.scaled(synth.workload(5), 1200, levels=6, l=2, c=c, k=k)
    cs = Case(w, 0, PLANAR)
    assert w.dg == 384 // c and gsr.gsr_graph_info(cs.gg)["n_hub_rows"] > 1000
    ref = oracle.step(cs.og, cs.ocfg, w.l, cs.x0_on_grid(), cs.inp.weights, cs.inp.w_out, cs.inp.b_out, cs.inp.target,
                      variant=2 if save else 0)
    out = run_step(cs, save_indices=save)
    assert np.isclose(out["loss"], ref["loss"], rtol=1e-4)
    for key in ("yhat", "XL", "X0rec", "dW", "dwout", "dX0"):
        assert_close(key, out[key], ref[key])
    W = cs.inp.weights[0]
    Wd = torch.from_numpy(W).to(cs.dev)
    X = cs.x0_on_grid()
    Y_ref = oracle.layer_forward(cs.og, cs.ocfg, W, X)
    y = cs.to_dev(X)
    gsr.gsr_layer_forward(cs.gg, cs.gcfg, Wd, y)
    assert_close("Y", cs.to_host(y), Y_ref)
    dY = (np.random.default_rng(5).standard_normal((w.n, w.d)) * 1e-3).astype(np.float32).astype(np.float64)
    Xb_ref, dX_ref, dW_ref = oracle.layer_backward(cs.og, cs.ocfg, W, Y_ref, dY)
    yb, dyb = cs.to_dev(Y_ref), cs.to_dev(dY)
    dW = torch.empty((w.c, w.dg, w.dg), dtype=torch.float32, device=cs.dev)
    gsr.gsr_layer_backward(cs.gg, cs.gcfg, Wd, yb, dyb, dW)
    assert_close("X rebuilt (backward)", cs.to_host(yb), Xb_ref)
    assert_close("dX", cs.to_host(dyb), dX_ref)
    assert_close("dW", dW.cpu().numpy(), dW_ref)


def test_wide_groups_with_bf16_storage():
    """bf16 storage, D/C = 192: a layer forward and backward under the audits of the full-size tests (bf16 near-ties
    make the two sides select differently on some rows; every row outside the bf16 bar must be explained by one, and
    in the backward the oracle is handed the GPU's selection for those rows)."""
    from gpu_util import audit_layer_forward, audit_layer_backward, bf16_bar
    cs = wide_case(3001, 384, 2, 16, 2, "rms", PLANAR, dtype="bf16")
    w = cs.w
    W = cs.inp.weights[0]
    X = cs.x0_on_grid()
    Y_ref = oracle.layer_forward(cs.og, cs.ocfg, W, X)
    y = cs.to_dev(X)
    gsr.gsr_layer_forward(cs.gg, cs.gcfg, torch.from_numpy(W).to(cs.dev), y)
    Y = cs.to_host(y)
    # group 1 follows from identical inputs and must agree on every row; with 192 bf16 columns nearly every row of its
    # output has a near-tie within one rounding step, so for group 2 the audit explains much and the norm bounds the rest
    audit_layer_forward(cs, X, Y, Y_ref, "wide bf16 fwd", bar=bf16_bar, max_reachable=1.01)
    assert not bf16_bar(Y[:, :w.dg], Y_ref[:, :w.dg]).any()
    print(f"[wide bf16 fwd] rel {rel_norm(Y, Y_ref):.2e}", flush=True)
    assert rel_norm(Y, Y_ref) <= 2 * BF16_REL
    rng = np.random.default_rng(3)
    dY = synth.to_bf16_grid((rng.standard_normal((w.n, w.d)) * 1e-3).astype(np.float32)).astype(np.float64)
    # three times the columns of a 64-wide group enter every sum, and 200 rows are handed over with values that differ
    # by a bf16 step between the sides: twice the bar of the 64-column case
    import functools
    audit_layer_backward(cs, W, Y, dY, "wide bf16 bwd", bar=functools.partial(bf16_bar, steps=2.0), dw_rtol=2e-2, max_flips=0.2)


def test_wide_groups_refuse_the_near_tie_list():
    cs = wide_case(500, 256, 2, 16, 2)
    with pytest.raises(gsr.GsrError) as e:
        run_step(cs, save_indices=2)
    assert e.value.status == gsr.GSR_ERR_UNSUPPORTED


@pytest.mark.parametrize("long_rows", [False, True])
def test_wide_step_replays_from_a_graph(long_rows):
    """Groups of 192 columns: a launch's second grid dimension is the column block written, and each column block draws
    its tiles from a counter set of its own, all of which a launch leaves clear.  A captured step must replay bit for
    bit, on a sparse graph (weight gradient in a pass of its own on a small persistent grid) and on a graph of long
    rows (one first pass for the three column blocks, fused inverse + dW)."""
    if long_rows:
        w = synth.scaled(synth.workload(5), 1200, levels=6, l=2, c=2, k=16)
        cs = Case(w, 0, PLANAR)
    else:
        gsr.gsr_set_option("max_workgroups", 8)
        try:
            cs = wide_case(3001, 384, 2, 16, 2, "rms", PLANAR)
        finally:
            gsr.gsr_set_option("max_workgroups", 0)
    cs.gcfg = gsr.Config(**{**cs.gcfg.__dict__, "save_indices": 1})
    w, dv = cs.w, cs.dev
    f32 = dict(dtype=torch.float32, device=dv)
    x0 = cs.to_dev(cs.inp.x0)
    W = torch.from_numpy(np.ascontiguousarray(cs.inp.weights[:w.l])).to(dv)
    w_out = torch.from_numpy(cs.inp.w_out).to(dv)
    b_out, target = torch.zeros(1, **f32), torch.from_numpy(cs.inp.target).to(dv)
    ws = torch.empty(gsr.gsr_workspace_size(cs.gg, cs.gcfg)[1], dtype=torch.uint8, device=dv)

    def buffers():
        return dict(loss=torch.zeros(1, **f32), dW=torch.empty_like(W), dw=torch.empty(w.d, **f32), db=torch.zeros(1, **f32),
                    dx0=torch.empty_like(x0), x0r=torch.empty_like(x0))

    def step(b):
        gsr.gsr_step(cs.gg, cs.gcfg, x0, W, w_out, b_out, target, b["loss"], b["dW"], b["dw"], b["db"], dx0_out=b["dx0"],
                     x0_rebuilt_out=b["x0r"], workspace=ws)

    eager = buffers()
    step(eager)
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in eager.items()}
    ref = oracle.step(cs.og, cs.ocfg, w.l, cs.x0_on_grid(), cs.inp.weights, cs.inp.w_out, cs.inp.b_out, cs.inp.target, variant=2)
    assert_close("dW", want["dW"].cpu().numpy(), ref["dW"])
    captured = buffers()
    stream = torch.cuda.Stream()
    stream.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            step(captured)
    for rep in range(3):
        for v in captured.values():
            v.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for k in want:
            assert torch.equal(captured[k], want[k]), (rep, k)
        step(eager)                                   # eager work between the replays
        torch.cuda.synchronize()
        for k in want:
            assert torch.equal(eager[k], want[k]), (rep, k)
