"""GPU parity of the two-group pipeline that the walk-throughs of Sections 4.3 / 4.4 print (its block places a
row's sums in the row's own recorded columns), against oracle/literal.py and the paper's printed numbers."""
import numpy as np
import pytest

import oracle
from oracle import literal
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth
from conftest import read_golden, dense_to_csr
from gpu_util import assert_close, violations, rel_norm

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def dev():
    return torch.device("cuda:0")


def to_dev(a, dtype=np.float32):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=dtype)).to(dev())


def paper_graph(b):
    rp, ci, av = dense_to_csr(b["A"])
    return gsr.gsr_graph_create(rp, ci, vals=av, flags=0)


def test_walkthrough_blocks_of_the_paper():
    b = read_golden("sec43_block_first.txt")
    c = read_golden("sec44_blocks.txt")
    gg = paper_graph(b)
    for v, i, want in ((b["VAL"], b["IDX"], b["OUT"]), (c["VALA"], c["IDXA"], c["OUTA"]), (c["VALB"], c["IDXB"], c["OUTB"])):
        out = gsr.gsr_slot_block(gg, to_dev(v), to_dev(i, np.int32), 2).cpu().numpy()
        assert np.allclose(out, want, atol=5e-3)


def test_algorithm_1_layer_of_the_paper():
    b = read_golden("sec43_layer_forward.txt")
    gg = paper_graph(b)
    x1, x2 = to_dev(b["G1"]), to_dev(b["G2"])
    gsr.gsr_alg1_layer_forward(gg, x1, x2, 1)
    assert np.allclose(x2.cpu().numpy(), b["X2NEW"], atol=5e-3)
    x1 = x1.cpu().numpy()
    assert np.allclose(x1[[1, 3]], b["X1NEW"][[1, 3]], atol=5e-3)      # rows 0 and 2: see the fixture
    assert np.allclose(x1, b["X1NEW"], atol=0.07) and np.array_equal(x1 == 0, b["X1NEW"] == 0)


def test_algorithm_2_steps_of_the_paper():
    c = read_golden("sec44_blocks.txt")
    s = read_golden("sec44_gs_signed.txt")
    og = oracle.graph_from_csr(*dense_to_csr(c["A"]))
    gg = paper_graph(c)
    g1, g2 = to_dev(c["G1"]), to_dev(s["Z"])
    gsr.gsr_alg2_layer_backward(gg, g1, g2, 1)
    w1, w2, _ = literal.alg2_layer_backward(og, c["G1"], s["Z"], 1)
    assert np.allclose(g1.cpu().numpy(), w1, atol=1e-5) and np.allclose(g2.cpu().numpy(), w2, atol=1e-5)


@pytest.mark.parametrize("dg,k,hub_threshold", [(64, 16, 512), (32, 8, 512), (64, 16, 6), (20, 5, 512), (64, 40, 7)])
def test_slot_block_against_oracle(dg, k, hub_threshold):
    gsr.gsr_set_option("hub_threshold", hub_threshold)
    gsr.gsr_set_option("hub_chunk", 4 if hub_threshold < 100 else 64)
    try:
        w = synth.scaled(synth.workload(2), 6001)
        rng = np.random.Generator(np.random.PCG64(5))
        rp, ci = synth.circuit_dag(w, rng)
        og = oracle.graph_build(rp, ci)
        gg = gsr.gsr_graph_create(rp, ci)
        V = rng.standard_normal((w.n, k)).astype(np.float32)
        I = np.sort(np.argsort(rng.random((w.n, dg)), axis=1)[:, :k], axis=1).astype(np.int32)
        out = gsr.gsr_slot_block(gg, to_dev(V), to_dev(I, np.int32), dg).cpu().numpy()
        assert_close("block", out, literal.slot_block(og, V, I, dg))
        assert np.count_nonzero(out) <= w.n * k
    finally:
        gsr.gsr_set_option("hub_threshold", 0)
        gsr.gsr_set_option("hub_chunk", 0)


def test_slot_block_over_the_transpose_of_a_directed_graph():
    rng = np.random.default_rng(3)
    n, dg, k = 300, 32, 6
    A = (rng.random((n, n)) < 0.03) * rng.uniform(0.2, 1.0, (n, n))
    rp, ci, av = dense_to_csr(A)
    og = oracle.graph_from_csr(rp, ci, av)
    gg = gsr.gsr_graph_create(rp, ci, vals=av, flags=0)
    V = rng.standard_normal((n, k)).astype(np.float32)
    I = np.sort(np.argsort(rng.random((n, dg)), axis=1)[:, :k], axis=1).astype(np.int32)
    for tr in (False, True):
        out = gsr.gsr_slot_block(gg, to_dev(V), to_dev(I, np.int32), dg, transpose=tr).cpu().numpy()
        assert_close("block", out, literal.slot_block(og, V, I, dg, transpose=tr))


def test_slot_block_ignores_columns_outside_the_group_and_rejects_bad_arguments():
    b = read_golden("sec43_block_first.txt")
    gg = paper_graph(b)
    idx = b["IDX"].astype(np.int32).copy()
    idx[0, 0] = 9
    out = gsr.gsr_slot_block(gg, to_dev(b["VAL"]), to_dev(idx, np.int32), 2).cpu().numpy()
    assert np.all(out[0] == 0) and np.allclose(out[1:], b["OUT"][1:], atol=5e-3)
    with pytest.raises(gsr.GsrError):
        gsr.gsr_slot_block(gg, to_dev(np.zeros((4, 3))), to_dev(np.zeros((4, 3)), np.int32), 2)      # k > dg
    with pytest.raises(gsr.GsrError):
        gsr.gsr_slot_block(gg, to_dev(b["VAL"]), to_dev(idx, np.int32), 65)                           # dg > 64


@pytest.mark.parametrize("n,dg,k", [(6001, 64, 16), (2000, 32, 8), (777, 20, 5)])
def test_layers_of_algorithms_1_and_2_against_oracle(n, dg, k):
    """Both layers on a circuit graph; rows where the two sides' top-k selections could differ (a near-tie
    between float32 and float64 sums) are counted and bounded, all others compared element by element."""
    w = synth.scaled(synth.workload(2), n)
    rng = np.random.Generator(np.random.PCG64(6))
    rp, ci = synth.circuit_dag(w, rng)
    og = oracle.graph_build(rp, ci)
    gg = gsr.gsr_graph_create(rp, ci)
    X1 = rng.standard_normal((n, dg)).astype(np.float32)
    X2 = rng.standard_normal((n, dg)).astype(np.float32)
    x1, x2 = to_dev(X1), to_dev(X2)
    gsr.gsr_alg1_layer_forward(gg, x1, x2, k)
    w1, w2, _ = literal.alg1_layer_forward(og, X1, X2, k)
    for name, got, want in (("x2", x2.cpu().numpy(), w2), ("x1", x1.cpu().numpy(), w1)):
        bad, worst = violations(got, want)
        print(f"[alg1 n={n}] {name}: rows outside tolerance {int(bad.any(axis=1).sum())}, rel {rel_norm(got, want):.2e}", flush=True)
        assert bad.any(axis=1).mean() < 2e-3 and rel_norm(got, want) < 1e-3
    G1 = (rng.standard_normal((n, dg)) * 1e-2).astype(np.float32)
    G2 = (rng.standard_normal((n, dg)) * 1e-2).astype(np.float32)
    g1, g2 = to_dev(G1), to_dev(G2)
    gsr.gsr_alg2_layer_backward(gg, g1, g2, k)
    v1, v2, _ = literal.alg2_layer_backward(og, G1, G2, k)
    for name, got, want in (("g1", g1.cpu().numpy(), v1), ("g2", g2.cpu().numpy(), v2)):
        bad, worst = violations(got, want)
        print(f"[alg2 n={n}] {name}: rows outside tolerance {int(bad.any(axis=1).sum())}, rel {rel_norm(got, want):.2e}", flush=True)
        assert bad.any(axis=1).mean() < 2e-3 and rel_norm(got, want) < 1e-3
        assert (np.count_nonzero(got, axis=1) <= k).all()


def test_layers_on_strided_planes_and_empty_graph():
    """Planes that are column slices of one [n, 2 dg] array (Split / Concat of Algorithm 1 as plain views)."""
    n, dg, k = 1500, 32, 8
    w = synth.scaled(synth.workload(2), n)
    rng = np.random.Generator(np.random.PCG64(7))
    rp, ci = synth.circuit_dag(w, rng)
    og = oracle.graph_build(rp, ci)
    gg = gsr.gsr_graph_create(rp, ci)
    X = rng.standard_normal((n, 2 * dg)).astype(np.float32)
    x = to_dev(X)
    gsr.gsr_alg1_layer_forward(gg, x[:, :dg], x[:, dg:], k)
    w1, w2, _ = literal.alg1_layer_forward(og, X[:, :dg], X[:, dg:], k)
    got = x.cpu().numpy()
    assert rel_norm(got[:, :dg], w1) < 1e-3 and rel_norm(got[:, dg:], w2) < 1e-3
    g0 = gsr.gsr_graph_create(np.zeros(1, dtype=np.int32), np.zeros(0, dtype=np.int32))
    e = torch.empty((0, dg), dtype=torch.float32, device=dev())
    gsr.gsr_alg1_layer_forward(g0, e, e.clone(), k)
