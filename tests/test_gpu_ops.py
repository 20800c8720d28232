"""GPU parity of the operators exposed by the C ABI: graph build + normalisation, GS, dense and
compressed aggregation.  Integer results (CSR structure, GS indices) must be bit-exact."""
import numpy as np
import pytest

import oracle
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth
from conftest import read_golden, dense_to_csr
from gpu_util import assert_close

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def dev():
    return torch.device("cuda:0")


@pytest.mark.parametrize("wl,n", [(0, None), (1, 20_000), (2, 30_000), (4, 40_000)])
def test_graph_build_bit_exact(wl, n):
    w = synth.workload(wl) if n is None else synth.scaled(synth.workload(wl), n)
    rng = np.random.Generator(np.random.PCG64(0))
    rp, ci = synth.circuit_dag(w, rng)
    if not w.rowptr64:
        rp = rp.astype(np.int32)
    og = oracle.graph_build(rp, ci)
    gg = gsr.gsr_graph_create(rp, ci)
    grp, gci, gav = gsr.gsr_graph_export(gg)
    assert np.array_equal(grp, og.rp)
    assert np.array_equal(gci, og.ci)
    assert np.array_equal(gav.view(np.uint32), og.av.view(np.uint32))      # values bit for bit
    info = gsr.gsr_graph_info(gg)
    assert info["n"] == w.n and info["nnz"] == og.nnz and info["max_degree"] == int(np.diff(og.rp).max())
    # unit values and back
    gsr.gsr_graph_normalize(gg, gsr.GSR_ADJ_UNIT)
    assert np.all(gsr.gsr_graph_export(gg)[2] == 1.0)
    gsr.gsr_graph_normalize(gg, gsr.GSR_ADJ_GCN_SYM)
    assert np.array_equal(gsr.gsr_graph_export(gg)[2].view(np.uint32), og.av.view(np.uint32))


def test_graph_create_empty_rows_and_duplicates():
    rp = np.array([0, 3, 3, 4, 6], dtype=np.int32)
    ci = np.array([1, 1, 0, 3, 0, 0], dtype=np.int32)
    og = oracle.graph_build(rp, ci)
    gg = gsr.gsr_graph_create(rp, ci)
    grp, gci, gav = gsr.gsr_graph_export(gg)
    assert np.array_equal(grp, og.rp) and np.array_equal(gci, og.ci)
    assert np.array_equal(gav.view(np.uint32), og.av.view(np.uint32))


def gs_inputs(n, dg, seed):
    rng = np.random.default_rng(seed)
    Z = rng.standard_normal((n, dg)).astype(np.float32)
    Z[1] = 0.0
    Z[2, ::2] = 1.5
    Z[3] = -np.abs(Z[3])
    Z[4, :] = 0.0
    Z[4, 3 % dg] = -0.0
    Z[5:40] = np.round(Z[5:40] * 2) / 2          # coarse grid: many exact ties
    Z[40:60] *= 1e-30                            # tiny magnitudes, all exponents alike
    Z[60:80] *= 1e15                             # squares still inside float32 range
    return Z


@pytest.mark.parametrize("dg,k", [(64, 16), (32, 8), (64, 1), (64, 64), (32, 32), (64, 63), (20, 5), (7, 3), (1, 1),
                                  (128, 16), (192, 64), (192, 1), (256, 255), (256, 256), (100, 33), (65, 4)])
@pytest.mark.parametrize("norm", ["none", "rms"])
def test_group_sparse_f32(dg, k, norm):
    n = 1003
    Z = gs_inputs(n, dg, dg * 131 + k)
    onorm = oracle.NORM_RMS if norm == "rms" else oracle.NORM_NONE
    gnorm = gsr.GSR_NORM_RMS if norm == "rms" else gsr.GSR_NORM_NONE
    V, I, _ = oracle.gs(Z.astype(np.float64), k, onorm, 1e-5, oracle.STORE_F32)
    v, i = gsr.gsr_group_sparse(torch.from_numpy(Z).to(dev()), k, gnorm, 1e-5)
    assert np.array_equal(i.cpu().numpy(), I)                           # indices: bit-exact
    if norm == "none":
        assert np.array_equal(v.cpu().numpy().astype(np.float64), V)    # values are copies
    else:
        assert np.allclose(v.cpu().numpy(), V, rtol=1e-5, atol=0)


@pytest.mark.parametrize("dg,k", [(64, 16), (32, 8)])
def test_group_sparse_bf16_and_strided(dg, k):
    n = 517
    Z = synth.to_bf16_grid(gs_inputs(n, dg, 5))                         # bf16 grid: ties are common
    V, I, _ = oracle.gs(Z.astype(np.float64), k, oracle.NORM_NONE, 1e-5, oracle.STORE_BF16)
    zt = torch.from_numpy(Z).to(dev()).to(torch.bfloat16)
    v, i = gsr.gsr_group_sparse(zt, k)
    assert np.array_equal(i.cpu().numpy(), I)
    assert np.array_equal(v.float().cpu().numpy().astype(np.float64), V)
    # a group is a column slice of an N x D row-major plane: row stride > dg
    wide = torch.zeros((n, 3 * dg), dtype=torch.float32, device=dev())
    wide[:, dg:2 * dg] = torch.from_numpy(Z).to(dev())
    v2, i2 = gsr.gsr_group_sparse(wide[:, dg:2 * dg], k)
    assert np.array_equal(i2.cpu().numpy(), I)


def test_group_sparse_worked_examples_of_the_paper():
    for name, mk in (("sec43_gs_first.txt", lambda b: b["Z"]), ("sec43_gs_second.txt", lambda b: b["X"] + b["M"]),
                     ("sec44_gs_signed.txt", lambda b: b["Z"]), ("sec44_gs_negative.txt", lambda b: b["G"] - b["B"])):
        b = read_golden(name)
        z = torch.from_numpy(mk(b).astype(np.float32)).to(dev())
        v, i = gsr.gsr_group_sparse(z, 1)
        assert np.array_equal(i.cpu().numpy(), b["IDX"].astype(np.int32))
        assert np.allclose(v.cpu().numpy(), b["VAL"], atol=5e-3)


def test_spmm_dense_and_transpose():
    rng = np.random.default_rng(3)
    n = 300
    A = (rng.random((n, n)) < 0.03) * rng.uniform(0.2, 1.0, (n, n))
    rp, ci, av = dense_to_csr(A)
    og = oracle.graph_from_csr(rp, ci, av)
    gg = gsr.gsr_graph_create(rp, ci, vals=av, flags=0)
    for width in (5, 64, 130):
        X = rng.standard_normal((n, width)).astype(np.float32)
        xt = torch.from_numpy(X).to(dev())
        assert_close("A X", gsr.gsr_spmm(gg, xt).cpu().numpy(), oracle.spmm(og, X))
        assert_close("A^T X", gsr.gsr_spmm(gg, xt, transpose=True).cpu().numpy(), oracle.spmm(og, X, transpose=True))
    # the paper's 4x4 example with unnormalised values (Section 4.1)
    b = read_golden("sec41_conventional_block.txt")
    g4 = gsr.gsr_graph_create(*dense_to_csr(b["A"])[:2], vals=dense_to_csr(b["A"])[2], flags=0)
    out = gsr.gsr_spmm(g4, torch.from_numpy(b["X"].astype(np.float32)).to(dev())).cpu().numpy()
    assert np.allclose(out, b["OUT"], atol=5e-3)


@pytest.mark.parametrize("width,hub_threshold", [(64, 512), (32, 512), (16, 512), (64, 6), (32, 5), (16, 5), (48, 6)])
def test_spmm_dense_on_a_circuit_graph_with_split_rows(width, hub_threshold):
    """The tiled path of gsr_spmm (widths 16, 32 and 64) with rows above the threshold reduced in two
    passes, a ragged last tile, and the row-per-wave path (width 48) on the same graph."""
    gsr.gsr_set_option("hub_threshold", hub_threshold)
    gsr.gsr_set_option("hub_chunk", 4 if hub_threshold < 100 else 64)
    try:
        w = synth.scaled(synth.workload(2), 6001)
        rng = np.random.Generator(np.random.PCG64(2))
        rp, ci = synth.circuit_dag(w, rng)
        og = oracle.graph_build(rp, ci)
        gg = gsr.gsr_graph_create(rp, ci)
        X = rng.standard_normal((w.n, width)).astype(np.float32)
        want = oracle.spmm(og, X)
        xt = torch.from_numpy(X).to(dev())
        assert_close("A X", gsr.gsr_spmm(gg, xt).cpu().numpy(), want)
        assert_close("A^T X", gsr.gsr_spmm(gg, xt, transpose=True).cpu().numpy(), want)     # the matrix is symmetric
        wide = torch.zeros((w.n, 2 * width + 16), dtype=torch.float32, device=dev())       # a column slice: row stride > width
        wide[:, 16:16 + width] = xt
        assert_close("A X (strided)", gsr.gsr_spmm(gg, wide[:, 16:16 + width]).cpu().numpy(), want)
    finally:
        gsr.gsr_set_option("hub_threshold", 0)
        gsr.gsr_set_option("hub_chunk", 0)


@pytest.mark.parametrize("dg,k,hub_threshold", [(64, 16, 512), (32, 8, 512), (64, 16, 6), (32, 8, 5)])
def test_spmm_compressed(dg, k, hub_threshold):
    gsr.gsr_set_option("hub_threshold", hub_threshold)
    gsr.gsr_set_option("hub_chunk", 4 if hub_threshold < 100 else 64)
    try:
        w = synth.scaled(synth.workload(2), 6001)
        rng = np.random.Generator(np.random.PCG64(1))
        rp, ci = synth.circuit_dag(w, rng)
        og = oracle.graph_build(rp, ci)
        gg = gsr.gsr_graph_create(rp, ci)
        if hub_threshold < 100:
            assert gsr.gsr_graph_info(gg)["n_hub_rows"] > 100
        Z = rng.standard_normal((w.n, dg)).astype(np.float32)
        V, I, _ = oracle.gs(Z.astype(np.float64), k)
        want = oracle.aggregate(og, V, I, dg)
        perm = np.argsort(rng.random((w.n, k)), axis=1)                  # any slot order is accepted
        Vp = np.take_along_axis(V, perm, axis=1).astype(np.float32)
        Ip = np.take_along_axis(I, perm, axis=1).astype(np.int32)
        got = gsr.gsr_spmm_compressed(gg, torch.from_numpy(Vp).to(dev()), torch.from_numpy(Ip).to(dev()), dg)
        assert_close("A scatter(V,I)", got.cpu().numpy(), want)
        bad = Ip.copy()
        bad[17, 0] = dg
        with pytest.raises(gsr.GsrError):
            gsr.gsr_spmm_compressed(gg, torch.from_numpy(Vp).to(dev()), torch.from_numpy(bad).to(dev()), dg)
        twice = Ip.copy()
        twice[w.n - 1, 1] = twice[w.n - 1, 0]                            # a column named twice
        with pytest.raises(gsr.GsrError):
            gsr.gsr_spmm_compressed(gg, torch.from_numpy(Vp).to(dev()), torch.from_numpy(twice).to(dev()), dg)
    finally:
        gsr.gsr_set_option("hub_threshold", 0)
        gsr.gsr_set_option("hub_chunk", 0)


def test_forward_block_example_of_the_paper():
    b = read_golden("sec41_gsr_forward_block.txt")
    rp, ci, av = dense_to_csr(b["A"])
    gg = gsr.gsr_graph_create(rp, ci, vals=av, flags=0)
    # the example has 4 columns; embed it in the first 4 of 32
    v = torch.from_numpy(b["VAL"].astype(np.float32)).to(dev())
    i = torch.from_numpy(b["IDX"].astype(np.int32)).to(dev())
    out = gsr.gsr_spmm_compressed(gg, v, i, 32).cpu().numpy()
    assert np.allclose(out[:, :4], b["OUT"], atol=5e-3) and np.all(out[:, 4:] == 0)


@pytest.mark.parametrize("workgroups,heavy_share", [(8, 0.3), (8, 1.0), (0, 1.0), (16, 0.05)])
def test_tile_operators_with_heavy_tiles_dealt_first(workgroups, heavy_share):
    """gsr_spmm (both directions, widths 16, 32 and 64) and gsr_spmm_compressed on directed graphs whose long tiles
    (more than 512 stored entries) are dealt to the waves before the sweep: a few among short tiles, all tiles
    long, more long tiles than waves, and a transpose with a different set of long tiles."""
    import scipy.sparse as sp
    gsr.gsr_set_option("max_workgroups", workgroups)
    try:
        rng = np.random.default_rng(12)
        n = 4001                                                     # ragged last tile
        nh = int(n * heavy_share) // 16 * 16
        rows, cols = [], []
        for lo, hi, deg in ((0, nh, 48), (nh, n, 3)):
            if hi > lo:
                r = np.repeat(np.arange(lo, hi), deg)
                rows.append(r)
                cols.append(rng.integers(0, n, size=len(r)))
        A = sp.csr_matrix((np.ones(sum(len(r) for r in rows)), (np.concatenate(rows), np.concatenate(cols))), shape=(n, n))
        A = (A > 0).astype(np.float64).tocsr()
        A.sort_indices()
        av = rng.uniform(0.2, 1.0, A.nnz).astype(np.float32)
        rp, ci = A.indptr.astype(np.int64), A.indices.astype(np.int32)
        og = oracle.graph_from_csr(rp, ci, av)
        gg = gsr.gsr_graph_create(rp, ci, vals=av, flags=0)
        for width in (64, 32, 16):
            X = rng.standard_normal((n, width)).astype(np.float32)
            xt = torch.from_numpy(X).to(dev())
            assert_close("A X", gsr.gsr_spmm(gg, xt).cpu().numpy(), oracle.spmm(og, X))
            assert_close("A^T X", gsr.gsr_spmm(gg, xt, transpose=True).cpu().numpy(), oracle.spmm(og, X, transpose=True))
            first = gsr.gsr_spmm(gg, xt)
            assert torch.equal(first, gsr.gsr_spmm(gg, xt))              # the counters are left clear
        for dg, k in ((64, 16), (32, 8)):
            Z = rng.standard_normal((n, dg)).astype(np.float32)
            V, I, _ = oracle.gs(Z.astype(np.float64), k)
            got = gsr.gsr_spmm_compressed(gg, torch.from_numpy(V.astype(np.float32)).to(dev()),
                                          torch.from_numpy(I.astype(np.int32)).to(dev()), dg)
            assert_close("A scatter(V,I)", got.cpu().numpy(), oracle.aggregate(og, V, I, dg))
    finally:
        gsr.gsr_set_option("max_workgroups", 0)
