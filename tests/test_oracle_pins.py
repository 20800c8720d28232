"""Pins of the CPU oracle against things other than itself: numbers the paper prints,
dense brute force, closed forms, invariants and finite differences.  CPU only."""
import numpy as np
import pytest

import oracle
from oracle import NORM_NONE, NORM_RMS, STORE_F64, STORE_F32, STORE_BF16
from paper_2603_27156_amd import synth
from conftest import read_golden, dense_to_csr, csr_to_dense


def small_graph(n=60, seed=1, levels=6):
    w = synth.scaled(synth.workload(0), n, levels=levels)
    rng = np.random.Generator(np.random.PCG64(seed))
    rp, ci = synth.circuit_dag(w, rng)
    return oracle.graph_build(rp, ci)


def directed_weighted_graph(n=25, seed=3):
    """Non-symmetric adjacency with arbitrary values: A != A^T, so any mix-up of G and G^T shows."""
    rng = np.random.default_rng(seed)
    A = (rng.random((n, n)) < 0.15) * rng.uniform(0.2, 1.0, (n, n))
    A[np.arange(n), np.arange(n)] = rng.uniform(0.2, 1.0, n)
    rp, ci, av = dense_to_csr(A)
    return oracle.graph_from_csr(rp, ci, av), A.astype(np.float32).astype(np.float64)


# ------------------------------------------------------------------ paper's printed numbers

def test_sec41_conventional_block_product():
    b = read_golden("sec41_conventional_block.txt")
    g = oracle.graph_from_csr(*dense_to_csr(b["A"]))
    out = oracle.spmm(g, b["X"])
    assert np.allclose(out, b["OUT"], atol=5e-3)  # printed to two decimals


def test_sec41_forward_block_on_compressed_embedding():
    b = read_golden("sec41_gsr_forward_block.txt")
    g = oracle.graph_from_csr(*dense_to_csr(b["A"]))
    out = oracle.aggregate(g, b["VAL"], b["IDX"].astype(np.int32), 4)
    assert np.allclose(out, b["OUT"], atol=5e-3)


@pytest.mark.parametrize("name,mk", [
    ("sec43_gs_first.txt", lambda b: b["Z"]),
    ("sec43_gs_second.txt", lambda b: b["X"] + b["M"]),
    ("sec44_gs_signed.txt", lambda b: b["Z"]),
    ("sec44_gs_negative.txt", lambda b: b["G"] - b["B"]),
])
def test_gs_worked_examples(name, mk):
    b = read_golden(name)
    V, I, _ = oracle.gs(mk(b), 1)
    assert np.array_equal(I, b["IDX"].astype(np.int32))
    assert np.allclose(V, b["VAL"], atol=5e-3)


# ------------------------------------------------------------------ the walk-throughs' own pipeline

def test_walkthrough_blocks_place_sums_in_the_rows_own_column():
    from oracle import literal
    b = read_golden("sec43_block_first.txt")
    g = oracle.graph_from_csr(*dense_to_csr(b["A"]))
    assert np.allclose(literal.slot_block(g, b["VAL"], b["IDX"].astype(np.int32), 2), b["OUT"], atol=5e-3)
    c = read_golden("sec44_blocks.txt")
    assert np.allclose(literal.slot_block(g, c["VALA"], c["IDXA"].astype(np.int32), 2), c["OUTA"], atol=5e-3)
    assert np.allclose(literal.slot_block(g, c["VALB"], c["IDXB"].astype(np.int32), 2), c["OUTB"], atol=5e-3)
    # the other placement (every neighbour at its own column) does not give these matrices
    assert not np.allclose(oracle.aggregate(g, b["VAL"], b["IDX"].astype(np.int32), 2), b["OUT"], atol=5e-2)


def test_sec41_backward_block_values():
    from oracle import literal
    b = read_golden("sec41_gsr_backward_block.txt")
    g = oracle.graph_from_csr(*dense_to_csr(b["A"]))
    I = b["IDX"].astype(np.int32)
    M = literal.scatter(b["VALG"], I, 4)
    M[M == 0] = 7.0                       # entries outside the recorded positions must not be read
    out = literal.block_backward(g, M, I)
    assert np.allclose(out[np.arange(4)[:, None], I], b["OUT"].sum(axis=1, keepdims=True), atol=5e-3)
    assert np.allclose(out[1:], b["OUT"][1:], atol=5e-3)       # row 0 is printed one column off
    assert np.count_nonzero(out) == 4


def test_sec43_layer_of_algorithm_1():
    from oracle import literal
    b = read_golden("sec43_layer_forward.txt")
    g = oracle.graph_from_csr(*dense_to_csr(b["A"]))
    X1n, X2n, (V1, I1, V2, I2) = literal.alg1_layer_forward(g, b["G1"], b["G2"], 1)
    assert np.allclose(X2n, b["X2NEW"], atol=5e-3)
    assert np.array_equal(I2[:, 0], [0, 1, 0, 1]) and np.allclose(V2[:, 0], [1.55, 1.2, 1.86, 1.15], atol=5e-3)
    # Algorithm 1, line 10, on the second block as printed
    assert np.allclose(literal.scatter(V1, I1, 2) + b["M2"], b["X1NEW"], atol=5e-3)
    # the whole layer: rows 1 and 3 exact, rows 0 and 2 carry the printed block's 0.06 / 0.05 slip
    assert np.allclose(X1n[[1, 3]], b["X1NEW"][[1, 3]], atol=5e-3)
    assert np.allclose(X1n, b["X1NEW"], atol=0.07)
    assert np.array_equal(X1n == 0, b["X1NEW"] == 0)


def test_sec44_steps_of_algorithm_2():
    from oracle import literal
    c = read_golden("sec44_blocks.txt")
    s = read_golden("sec44_gs_signed.txt")
    g = oracle.graph_from_csr(*dense_to_csr(c["A"]))
    _, _, im = literal.alg2_layer_backward(g, c["G1"], s["Z"], 1)
    assert np.array_equal(im["I2"], c["IDXA"].astype(np.int32)) and np.allclose(im["V2"], c["VALA"], atol=5e-3)
    assert np.allclose(im["B2"], c["OUTA"], atol=5e-3)
    assert (im["M1"] < 0).all() and np.allclose(-im["M1"], c["M1ABS"], atol=5e-3)
    assert np.array_equal(im["I1"], c["IDXB"].astype(np.int32)) and np.allclose(im["V1"], c["VALB"], atol=5e-3)
    assert np.allclose(im["Z1"], c["OUTB"], atol=5e-3)
    assert np.allclose(im["M2"], literal.scatter(c["VALA"], c["IDXA"].astype(np.int32), 2) - c["OUTB"], atol=1e-2)


def test_algorithm_2_returns_the_backward_blocks_of_its_pinned_steps():
    """What alg2_layer_backward returns (Algorithm 2, last step of the loop body): the printed final matrices of
    Section 4.4 follow no rule, so the composition is pinned by what the mathematics fixes instead.  On a directed
    weighted graph each returned plane must be the Section 4.1 backward block of the (pinned) intermediate it
    belongs to, written out with dense loops over A^T, and must satisfy the adjoint identity of that block."""
    from oracle import literal
    g, A = directed_weighted_graph(30, seed=17)
    rng = np.random.default_rng(18)
    n, dg, k = A.shape[0], 12, 4
    G1, G2 = rng.standard_normal((n, dg)), rng.standard_normal((n, dg))
    g1, g2, im = literal.alg2_layer_backward(g, G1, G2, k)
    for got, M, I in ((g1, im["M1"], im["I1"]), (g2, im["M2"], im["I2"])):
        want = np.zeros((n, dg))
        for i in range(n):
            for t in range(k):
                want[i, I[i, t]] = sum(A[j, i] * M[j, I[j, t]] for j in range(n))      # sum over G^T, slot by slot
        assert np.allclose(got, want, atol=1e-12)
        assert np.count_nonzero(got) <= n * k
        V = rng.standard_normal((n, k))
        lhs = np.sum(literal.slot_block(g, V, I, dg) * literal.scatter(M[np.arange(n)[:, None], I], I, dg))
        rhs = np.sum(V * got[np.arange(n)[:, None], I])
        assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))
    # the intermediates it was fed are the ones the printed steps pin (M1 = G1 - block(GS(G2)), ...)
    assert np.allclose(im["M1"], G1 - literal.slot_block(g, im["V2"], im["I2"], dg))
    assert np.allclose(im["M2"], literal.scatter(im["V2"], im["I2"], dg) - literal.slot_block(g, im["V1"], im["I1"], dg))


def test_slot_block_against_dense_algebra_and_its_adjoint():
    """out[i, I[i,t]] = (A V)[i,t] written with dense matrices; block_backward is the adjoint of the map
    V -> slot_block(V, I) followed by the same placement (non-symmetric A: G and G^T differ)."""
    from oracle import literal
    g, A = directed_weighted_graph()
    rng = np.random.default_rng(4)
    n, dg, k = A.shape[0], 16, 5
    I = np.sort(np.argsort(rng.random((n, dg)), axis=1)[:, :k], axis=1).astype(np.int32)
    V = rng.standard_normal((n, k))
    out = literal.slot_block(g, V, I, dg)
    S = A @ V
    ref = np.zeros((n, dg))
    for i in range(n):
        for t in range(k):
            ref[i, I[i, t]] = S[i, t]
    assert np.allclose(out, ref, atol=1e-12)
    M = rng.standard_normal((n, dg))
    lhs = np.sum(out * M)                                              # <block(V), M>
    back = literal.block_backward(g, M, I)
    rhs = np.sum(V * back[np.arange(n)[:, None], I])                   # <V, slots of block_backward(M)>
    assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))


# ------------------------------------------------------------------ GS against a full sort

@pytest.mark.parametrize("dg,k", [(32, 8), (64, 16), (64, 1), (64, 64), (8, 3)])
def test_gs_brute_force_and_invariants(dg, k):
    rng = np.random.default_rng(dg * 100 + k)
    Z = rng.standard_normal((200, dg))
    Z[5] = 0.0                      # all ties
    Z[6, ::2] = 1.5                 # many ties at the top
    Z[7] = -np.abs(Z[7])            # all negative
    Z[8, 3] = -0.0                  # -0 == +0
    Z[8, 1] = 0.0
    Z = np.round(Z * 4) / 4 if dg == 8 else Z     # coarse grid -> plenty of ties
    V, I, r = oracle.gs(Z, k)
    for row in range(Z.shape[0]):
        order = sorted(range(dg), key=lambda c: (-Z[row, c], c))[:k]
        assert list(I[row]) == sorted(order)
        assert np.array_equal(V[row], Z[row, I[row]])
        assert len(set(I[row])) == k and I[row].min() >= 0 and I[row].max() < dg
        rejected = np.setdiff1d(np.arange(dg), I[row])
        if len(rejected):
            assert Z[row, I[row]].min() >= Z[row, rejected].max()
    assert np.all(r == 1.0)


def test_gs_rms_scale_closed_form():
    rng = np.random.default_rng(0)
    Z = rng.standard_normal((50, 64)) * 3.0
    V0, I0, _ = oracle.gs(Z, 16, NORM_NONE)
    V1, I1, r = oracle.gs(Z, 16, NORM_RMS, 1e-5)
    assert np.array_equal(I0, I1)               # the scale never changes what is selected
    rms = np.sqrt((Z ** 2).mean(axis=1) + 1e-5)
    assert np.allclose(r, rms, rtol=1e-14)
    assert np.allclose(V1, V0 / rms[:, None], rtol=1e-14)


def test_storage_rounding_matches_library_conversions():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    x = np.concatenate([rng.standard_normal(2000) * 10.0 ** rng.integers(-6, 6, 2000),
                        [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -1.0 - 2.0 ** -8, 0.0, 65280.0]])
    want_bf = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    got_bf = oracle.round_store(x, STORE_BF16)
    assert np.array_equal(got_bf, want_bf)
    assert oracle.round_store(np.array([1.0 + 2.0 ** -8]), STORE_BF16)[0] == 1.0          # tie -> even
    assert oracle.round_store(np.array([1.0 + 3 * 2.0 ** -8]), STORE_BF16)[0] == 1.0 + 2.0 ** -6
    assert np.array_equal(oracle.round_store(x, STORE_F32), x.astype(np.float32).astype(np.float64))
    # the bf16 grid helper of the input generators lands on the same grid
    assert np.array_equal(synth.to_bf16_grid(x.astype(np.float32)).astype(np.float64),
                          oracle.round_store(x.astype(np.float32), STORE_BF16))


# ------------------------------------------------------------------ graph normalisation

def test_graph_build_structure_and_normalisation():
    w = synth.workload(0)
    rng = np.random.Generator(np.random.PCG64(0))
    rp_in, ci_in = synth.circuit_dag(w, rng)
    g = oracle.graph_build(rp_in, ci_in)
    n = w.n
    A = csr_to_dense(g.rp, g.ci, g.av, n)
    # structure: brute-force symmetrisation with numpy
    B = np.zeros((n, n), dtype=bool)
    for i in range(n):
        B[i, ci_in[rp_in[i]:rp_in[i + 1]]] = True
    B = B | B.T | np.eye(n, dtype=bool)
    assert np.array_equal(A != 0, B)
    for i in range(n):
        cols = g.ci[g.rp[i]:g.rp[i + 1]]
        assert np.all(np.diff(cols) > 0)                       # ascending, no duplicates
        assert (cols == i).sum() == 1                          # exactly one self-loop
    deg = B.sum(axis=1).astype(np.float64)
    want = B / np.sqrt(deg)[:, None] / np.sqrt(deg)[None, :]
    assert np.allclose(A, want, rtol=3e-7)                     # float32 recipe
    assert np.array_equal(A, A.T)                              # exactly symmetric
    assert np.allclose(A @ np.sqrt(deg), np.sqrt(deg), rtol=1e-6)   # eigenvector of eigenvalue 1
    # the fixed float32 recipe, bit for bit
    dinv = (np.float32(1.0) / np.sqrt(deg.astype(np.float32))).astype(np.float32)
    rows = np.repeat(np.arange(n), np.diff(g.rp))
    assert np.array_equal(g.av, (dinv[rows] * dinv[g.ci]).astype(np.float32))
    # transpose arrays describe the same matrix transposed
    assert np.array_equal(csr_to_dense(g.trp, g.tci, g.tav, n), A.T)


def test_graph_build_merges_duplicates_and_existing_self_loops():
    rp = np.array([0, 3, 4, 6], dtype=np.int64)
    ci = np.array([1, 1, 0, 2, 0, 0], dtype=np.int32)   # row0: 1,1,0(self)  row1: 2  row2: 0,0
    g = oracle.graph_build(rp, ci)
    assert list(g.rp) == [0, 3, 6, 9]
    assert list(g.ci) == [0, 1, 2, 0, 1, 2, 0, 1, 2]
    assert np.allclose(g.av, 1.0 / 3.0)


def test_graph_build_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.graph_build(np.array([0, 1], dtype=np.int64), np.array([5], dtype=np.int32))


# ------------------------------------------------------------------ aggregation = dense brute force

@pytest.mark.parametrize("dg,k", [(32, 8), (64, 16)])
def test_aggregate_equals_dense_product(dg, k):
    w = synth.workload(0)
    rng = np.random.Generator(np.random.PCG64(0))
    g = oracle.graph_build(*synth.circuit_dag(w, rng))
    n = w.n
    Z = rng.standard_normal((n, dg))
    V, I, _ = oracle.gs(Z, k)
    S = np.zeros((n, dg))
    np.put_along_axis(S, I.astype(np.int64), V, axis=1)
    A = csr_to_dense(g.rp, g.ci, g.av, n)
    assert np.allclose(oracle.aggregate(g, V, I, dg), A @ S, rtol=1e-12, atol=1e-14)
    X = rng.standard_normal((n, 7))
    assert np.allclose(oracle.spmm(g, X), A @ X, rtol=1e-12, atol=1e-14)


def test_spmm_transpose_on_directed_graph():
    g, A = directed_weighted_graph()
    X = np.random.default_rng(0).standard_normal((g.n, 5))
    assert np.allclose(oracle.spmm(g, X), A @ X, rtol=1e-12)
    assert np.allclose(oracle.spmm(g, X, transpose=True), A.T @ X, rtol=1e-12)


# ------------------------------------------------------------------ k = Dg: a linear GCN, closed form

def dense_linear_step(A, X0, W, w_out, b, t, C):
    """Textbook dense algebra for the k = Dg, no-normalisation case: every block is Z -> A Z W.
    Returns loss and all gradients by hand-written dense back-propagation."""
    n, D = X0.shape
    dg = D // C
    L = W.shape[0]
    X = X0.copy()
    tape = []
    for l in range(L):
        Xs = [X[:, i * dg:(i + 1) * dg] for i in range(C)]
        Ys = [sum(Xs[1:])]
        for i in range(C):
            Ys.append(A @ Ys[i] @ W[l, i] + Xs[i])
        tape.append(Ys)
        X = np.concatenate(Ys[1:], axis=1)
    yhat = X @ w_out + b
    e = yhat - t
    loss = (e ** 2).mean()
    dy = 2 * e / n
    dwout = X.T @ dy
    db = dy.sum()
    G = np.outer(dy, w_out)
    dW = np.zeros_like(W)
    for l in reversed(range(L)):
        Ys = tape[l]
        dYs = [np.zeros((n, dg))] + [G[:, i * dg:(i + 1) * dg].copy() for i in range(C)]
        for i in reversed(range(C)):
            dW[l, i] = (A @ Ys[i]).T @ dYs[i + 1]
            dYs[i] += A.T @ dYs[i + 1] @ W[l, i].T
        dXs = [dYs[1]] + [dYs[i + 1] + dYs[0] for i in range(1, C)]
        G = np.concatenate(dXs, axis=1)
    return dict(loss=loss, yhat=yhat, XL=X, dW=dW, dwout=dwout, dbout=db, dX0=G)


@pytest.mark.parametrize("C", [2, 4])
@pytest.mark.parametrize("directed", [False, True])
def test_full_k_step_is_the_linear_gcn(C, directed):
    rng = np.random.default_rng(7 + C)
    if directed:
        g, A = directed_weighted_graph(30, seed=11)
    else:
        g = small_graph(40, seed=2)
        A = csr_to_dense(g.rp, g.ci, g.av, g.n)
    n, dg, L = g.n, 6, 3
    D = dg * C
    X0 = rng.standard_normal((n, D))
    W = rng.uniform(-0.4, 0.4, (L, C, dg, dg))
    w_out = rng.uniform(-0.5, 0.5, D)
    t = rng.standard_normal(n)
    cfg = oracle.Cfg(D, C, dg, NORM_NONE)
    want = dense_linear_step(A, X0, W, w_out, 0.3, t, C)
    for variant in (0, 1, 2):
        got = oracle.step(g, cfg, L, X0, W, w_out, 0.3, t, variant=variant)
        assert np.isclose(got["loss"], want["loss"], rtol=1e-12)
        for key in ("yhat", "XL", "dW", "dwout", "dX0"):
            assert np.allclose(got[key], want[key], rtol=1e-9, atol=1e-12), key
        assert np.isclose(got["dbout"], want["dbout"], rtol=1e-10)
        assert np.allclose(got["X0rec"], X0, rtol=1e-9, atol=1e-11)


# ------------------------------------------------------------------ reversibility, variants, invariants

@pytest.mark.parametrize("C,norm", [(2, NORM_NONE), (4, NORM_RMS), (8, NORM_RMS)])
def test_inverse_undoes_forward(C, norm):
    g = small_graph(80, seed=4)
    rng = np.random.default_rng(5)
    dg, k = 8, 3
    D = dg * C
    cfg = oracle.Cfg(D, C, k, norm)
    X = rng.standard_normal((g.n, D))
    W = rng.uniform(-0.5, 0.5, (C, dg, dg))
    Y = oracle.layer_forward(g, cfg, W, X)
    assert not np.allclose(Y, X)
    Xr = oracle.layer_inverse(g, cfg, W, Y)
    assert np.max(np.abs(Xr - X)) <= 1e-12 * max(1.0, np.abs(Y).max())


def test_layer_forward_against_direct_formula():
    """eq. (6) written out with numpy on top of the pinned GS and dense products."""
    g, A = directed_weighted_graph(20, seed=5)
    rng = np.random.default_rng(6)
    C, dg, k = 3, 8, 3
    D = C * dg
    for norm in (NORM_NONE, NORM_RMS):
        cfg = oracle.Cfg(D, C, k, norm)
        X = rng.standard_normal((g.n, D))
        W = rng.uniform(-0.5, 0.5, (C, dg, dg))
        Xs = [X[:, i * dg:(i + 1) * dg] for i in range(C)]
        prev = sum(Xs[1:])
        outs = []
        for i in range(C):
            order = np.argsort(-prev, axis=1, kind="stable")[:, :k]
            S = np.zeros_like(prev)
            scale = 1.0 / np.sqrt((prev ** 2).mean(axis=1, keepdims=True) + cfg.eps) if norm == NORM_RMS else 1.0
            np.put_along_axis(S, order, np.take_along_axis(prev, order, axis=1), axis=1)
            prev = A @ (S * scale) @ W[i] + Xs[i]
            outs.append(prev)
        assert np.allclose(oracle.layer_forward(g, cfg, W, X), np.concatenate(outs, axis=1), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("C,norm", [(2, NORM_NONE), (2, NORM_RMS), (4, NORM_RMS)])
def test_interleaved_backward_equals_stored_activation_backward(C, norm):
    g, _ = directed_weighted_graph(40, seed=8)
    rng = np.random.default_rng(9)
    dg, k, L = 8, 3, 5
    D = dg * C
    cfg = oracle.Cfg(D, C, k, norm)
    X0 = rng.standard_normal((g.n, D))
    W = rng.uniform(-0.3, 0.3, (L, C, dg, dg))
    w_out = rng.uniform(-0.5, 0.5, D)
    t = rng.standard_normal(g.n)
    a = oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=0)
    b = oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=1)
    c = oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=2)
    for key in ("yhat", "XL", "dW", "dwout", "dX0", "X0rec"):
        assert np.allclose(a[key], b[key], rtol=1e-9, atol=1e-11), key
        assert np.allclose(c[key], b[key], rtol=1e-9, atol=1e-11), key
    assert a["loss"] == b["loss"] == c["loss"]


def test_saved_indices_keep_the_inverse_exact_where_reselection_flips():
    """Section 4.2 keeps the indices of the forward pass.  With coarse (bf16) stores the rebuilt
    activations differ from the forward's by rounding; selecting again then often picks another
    column at a near-tie and the rebuilt input drifts, while with the kept indices the inverse is
    continuous in its input: the input comes back to storage rounding and the gradients stay
    close to those of plain back-propagation from stored activations."""
    g = small_graph(300, seed=21)
    rng = np.random.default_rng(22)
    C, dg, k, L = 2, 16, 4, 12
    D = C * dg
    cfg = oracle.Cfg(D, C, k, NORM_RMS, 1e-5, oracle.STORE_BF16)
    X0 = oracle.round_store(rng.standard_normal((g.n, D)), oracle.STORE_BF16)
    W = rng.uniform(-0.3, 0.3, (L, C, dg, dg))
    w_out = rng.uniform(-0.5, 0.5, D)
    t = rng.standard_normal(g.n)
    stored = oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=1)
    saved = oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=2)
    again = oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=0)
    # the forward sweep is the same in all variants
    assert np.array_equal(saved["XL"], stored["XL"]) and np.array_equal(again["XL"], stored["XL"])
    scale = np.abs(saved["XL"]).max()
    err_saved, err_again = np.abs(saved["X0rec"] - X0).max(), np.abs(again["X0rec"] - X0).max()
    assert err_saved <= 2e-2 * scale                     # a few bf16 roundings (2^-9 relative each)
    assert err_again > 10 * err_saved                    # the case does exercise the difference

    def rel(x, ref):
        return np.linalg.norm(x - ref) / np.linalg.norm(ref)

    assert rel(saved["dW"], stored["dW"]) <= 5e-3 and rel(saved["dX0"], stored["dX0"]) <= 2e-2
    assert rel(again["dX0"], stored["dX0"]) > 5 * rel(saved["dX0"], stored["dX0"])


# ------------------------------------------------------------------ indices kept for near-tie rows only

def test_near_tie_rows_against_a_full_sort():
    """orc_gs_near_tie: gap between the k-th and (k+1)-th largest value against tol * max|row|, in float32.
    Brute force by a full sort; exact ties (incl. -0 against +0) are always listed, k = Dg never."""
    rng = np.random.default_rng(31)
    dg, k, n = 16, 5, 4000
    Z = rng.standard_normal((n, dg)).astype(np.float32)
    Z[::7, 3] = Z[::7, 9]                               # exact ties somewhere in the row
    Z[5] = 0.0
    Z[5, :8] = -0.0
    for tol in (0.0, 2.0 ** -12, 2.0 ** -6, 0.3):
        s = -np.sort(-Z, axis=1)
        gap = (s[:, k - 1] - s[:, k]).astype(np.float32)
        bar = (np.float32(tol) * np.abs(Z).max(axis=1)).astype(np.float32)
        assert np.array_equal(oracle.gs_near_tie(Z, k, tol), gap <= bar)
    tied = np.array([np.sort(z)[::-1][k - 1] == np.sort(z)[::-1][k] for z in Z])
    assert tied.sum() > 20 and oracle.gs_near_tie(Z, k, 0.0)[tied].all()
    assert np.array_equal(np.flatnonzero(oracle.gs_near_tie(Z, k, -1.0)), [5])      # only the all-zero row: 0 <= -1 * 0
    assert not oracle.gs_near_tie(Z, dg, 1e30).any()
    # a bf16-like case: many equal values per row
    Zb = np.round(rng.standard_normal((500, dg)) * 2) / 2
    s = -np.sort(-Zb, axis=1)
    assert np.array_equal(oracle.gs_near_tie(Zb, k, 0.0), s[:, k - 1] == s[:, k])


def test_listed_rows_take_the_kept_indices_and_the_others_select_again():
    """orc_layer_backward with (I_saved, listed): a listed row uses its kept indices, any other row the indices a
    fresh selection gives.  Pinned through the all-rows form (I_saved alone, itself pinned against stored
    activations): C = 2, rows of block 1 listed with indices that differ from the fresh selection."""
    g, _ = directed_weighted_graph(40, seed=13)
    rng = np.random.default_rng(14)
    C, dg, k = 2, 8, 3
    D = C * dg
    cfg = oracle.Cfg(D, C, k, NORM_RMS)
    Y = rng.standard_normal((g.n, D))
    dY = rng.standard_normal((g.n, D))
    W = rng.uniform(-0.4, 0.4, (C, dg, dg))
    X, _, _ = oracle.layer_backward(g, cfg, W, Y, dY)
    fresh2 = oracle.gs(Y[:, :dg], k)[1]                 # block 2 selects on Y_1
    fresh1 = oracle.gs(X[:, dg:], k)[1]                 # block 1 selects on Y_0 = X_2 (C = 2), rebuilt by block 2
    rows = np.array([1, 7, 8, 22, 39])
    alt = fresh1.copy()
    alt[rows] = np.sort((fresh1[rows] + 1 + np.arange(k)) % dg, axis=1)
    alt[rows[0]] = [0, 1, 2]
    assert all(len(set(r)) == k for r in alt[rows]) and (alt[rows] != fresh1[rows]).any()
    junk = np.zeros_like(fresh2)                        # rows that are not listed never read their kept indices
    saved = np.stack([np.where(np.isin(np.arange(g.n), rows)[:, None], alt, junk), junk])
    listed = np.zeros((C, g.n), dtype=bool)
    listed[0, rows] = True
    got = oracle.layer_backward(g, cfg, W, Y, dY, I_saved=saved, listed=listed)
    want = oracle.layer_backward(g, cfg, W, Y, dY, I_saved=np.stack([alt, fresh2]))
    plain = oracle.layer_backward(g, cfg, W, Y, dY)
    for a, b, c in zip(got, want, plain):
        assert np.array_equal(a, b) and not np.array_equal(a, c)
    # nothing listed: the plain call; everything listed: the all-rows form
    none = oracle.layer_backward(g, cfg, W, Y, dY, I_saved=saved, listed=np.zeros((C, g.n), dtype=bool))
    every = oracle.layer_backward(g, cfg, W, Y, dY, I_saved=np.stack([alt, fresh2]), listed=np.ones((C, g.n), dtype=bool))
    for a, b, c, d in zip(none, plain, every, want):
        assert np.array_equal(a, b) and np.array_equal(c, d)


def test_step_with_near_tie_list_between_nothing_kept_and_everything_kept():
    """variant 3 of the step: tol < 0 lists nothing (= variant 0, bit for bit), a huge tol lists every row
    (= variant 2, bit for bit); with coarse stores, where selecting again flips rows, a moderate tol brings the
    rebuilt input and the gradients back to those of the kept-indices run while listing a fraction of the rows."""
    g = small_graph(300, seed=21)
    rng = np.random.default_rng(22)
    C, dg, k, L = 2, 16, 4, 12
    D = C * dg
    cfg = oracle.Cfg(D, C, k, NORM_RMS, 1e-5, oracle.STORE_BF16)
    X0 = oracle.round_store(rng.standard_normal((g.n, D)), oracle.STORE_BF16)
    W = rng.uniform(-0.3, 0.3, (L, C, dg, dg))
    w_out = rng.uniform(-0.5, 0.5, D)
    t = rng.standard_normal(g.n)
    run = lambda variant, tol=0.0: oracle.step(g, cfg, L, X0, W, w_out, 0.0, t, variant=variant, tie_tol=tol)
    again, saved = run(0), run(2)
    lo, hi, mid = run(3, -1.0), run(3, 1e30), run(3, 2.0 ** -5)
    keys = ("yhat", "XL", "dW", "dwout", "dX0", "X0rec")
    assert lo["n_listed"] == 0 and hi["n_listed"] == g.n * C * L
    for key in keys:
        assert np.array_equal(lo[key], again[key]), key
        assert np.array_equal(hi[key], saved[key]), key
    assert 0 < mid["n_listed"] < 0.5 * g.n * C * L
    err = lambda r: np.abs(r["X0rec"] - X0).max()
    assert err(again) > 10 * err(saved) and err(mid) <= 2 * err(saved)


def test_zero_weights_make_layers_the_identity():
    g = small_graph(50, seed=10)
    rng = np.random.default_rng(11)
    C, dg, k, L = 2, 8, 4, 3
    D = C * dg
    cfg = oracle.Cfg(D, C, k, NORM_RMS)
    X0 = rng.standard_normal((g.n, D))
    w_out = rng.uniform(-0.5, 0.5, D)
    t = rng.standard_normal(g.n)
    out = oracle.step(g, cfg, L, X0, np.zeros((L, C, dg, dg)), w_out, 0.1, t)
    yhat = X0 @ w_out + 0.1
    assert np.allclose(out["XL"], X0) and np.allclose(out["yhat"], yhat)
    assert np.isclose(out["loss"], ((yhat - t) ** 2).mean())
    assert np.allclose(out["dX0"], np.outer(2 * (yhat - t) / g.n, w_out))


def test_node_relabelling_permutes_outputs():
    w = synth.scaled(synth.workload(0), 70, levels=7)
    rng = np.random.Generator(np.random.PCG64(12))
    rp, ci = synth.circuit_dag(w, rng)
    n = w.n
    perm = rng.permutation(n)                    # new id of old node i is perm[i]
    rows = np.repeat(np.arange(n), np.diff(rp))
    new_rows, new_cols = perm[rows], perm[ci]
    order = np.lexsort((new_cols, new_rows))
    rp2 = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rp2, new_rows + 1, 1)
    rp2 = np.cumsum(rp2)
    g1, g2 = oracle.graph_build(rp, ci), oracle.graph_build(rp2, new_cols[order].astype(np.int32))
    C, dg, k = 2, 8, 3
    cfg = oracle.Cfg(C * dg, C, k, NORM_RMS)
    X = rng.standard_normal((n, C * dg))
    W = rng.uniform(-0.5, 0.5, (C, dg, dg))
    X2 = np.zeros_like(X)
    X2[perm] = X
    Y1 = oracle.layer_forward(g1, cfg, W, X)
    Y2 = oracle.layer_forward(g2, cfg, W, X2)
    assert np.allclose(Y2[perm], Y1, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ finite differences

def _fd_check(g, cfg, L, X0, W, w_out, b, t, rng, nprobe=14):
    base = oracle.step(g, cfg, L, X0, W, w_out, b, t)

    def loss_at(Xp, Wp, wp):
        return oracle.step(g, cfg, L, Xp, Wp, wp, b, t, want=())["loss"]

    checked = 0
    for which, arr, grad in (("W", W, base["dW"]), ("w_out", w_out, base["dwout"]), ("X0", X0, base["dX0"])):
        flat_idx = rng.choice(arr.size, size=min(nprobe, arr.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            est = []
            for h in (1e-5, 5e-6):
                vals = []
                for s in (+1, -1):
                    a2 = arr.copy()
                    a2[idx] += s * h
                    args = dict(Xp=X0, Wp=W, wp=w_out)
                    args[{"W": "Wp", "w_out": "wp", "X0": "Xp"}[which]] = a2
                    vals.append(loss_at(**args))
                est.append((vals[0] - vals[1]) / (2 * h))
            # a top-k mask that flips inside the probe interval makes the two estimates disagree
            if abs(est[0] - est[1]) > 1e-5 * max(abs(est[0]), abs(est[1]), 1e-8):
                continue
            checked += 1
            assert np.isclose(grad[idx], est[1], rtol=2e-5, atol=1e-9), (which, idx, grad[idx], est)
    return checked


@pytest.mark.parametrize("C,norm,directed", [(2, NORM_NONE, False), (2, NORM_RMS, True), (4, NORM_RMS, False)])
def test_gradients_against_central_finite_differences(C, norm, directed):
    rng = np.random.default_rng(20 + C + norm)
    if directed:
        g, _ = directed_weighted_graph(30, seed=21)
    else:
        g = small_graph(40, seed=22)
    dg, k, L = 8, 3, 3
    D = dg * C
    cfg = oracle.Cfg(D, C, k, norm)
    X0 = rng.standard_normal((g.n, D))
    W = rng.uniform(-0.5, 0.5, (L, C, dg, dg))
    w_out = rng.uniform(-0.5, 0.5, D)
    t = rng.standard_normal(g.n)
    checked = _fd_check(g, cfg, L, X0, W, w_out, 0.2, t, rng)
    assert checked >= 30      # nearly all of the 42 probes are away from a mask flip


def test_head_closed_form():
    rng = np.random.default_rng(30)
    X = rng.standard_normal((33, 10))
    w = rng.standard_normal(10)
    t = rng.standard_normal(33)
    h = oracle.head(X, w, -0.4, t)
    y = X @ w - 0.4
    assert np.allclose(h["yhat"], y) and np.isclose(h["loss"], ((y - t) ** 2).mean())
    dy = 2 * (y - t) / 33
    assert np.allclose(h["dX"], np.outer(dy, w)) and np.allclose(h["dw"], X.T @ dy) and np.isclose(h["db"], dy.sum())


def test_storage_rounding_keeps_planes_on_the_grid():
    g = small_graph(60, seed=31)
    rng = np.random.default_rng(32)
    C, dg, k = 2, 8, 3
    X = rng.standard_normal((g.n, C * dg)).astype(np.float32).astype(np.float64)
    W = rng.uniform(-0.5, 0.5, (C, dg, dg))
    for sm, snap in ((STORE_F32, lambda a: a.astype(np.float32).astype(np.float64)),
                     (STORE_BF16, lambda a: oracle.round_store(a, STORE_BF16))):
        cfg = oracle.Cfg(C * dg, C, k, NORM_RMS, 1e-5, sm)
        Y = oracle.layer_forward(g, cfg, W, X)
        assert np.array_equal(Y, snap(Y))
        ref = oracle.layer_forward(g, oracle.Cfg(C * dg, C, k, NORM_RMS), W, X)
        tol = 1e-6 if sm == STORE_F32 else 2e-2
        assert np.allclose(Y, ref, rtol=tol, atol=tol)


# ------------------------------------------------------------------ parameter updates

def test_optimiser_closed_forms():
    from oracle import optim
    # gradient descent on L = w^2 / 2 (dw = w): w_t = (1 - lr)^t w_0; with weight decay the factor is 1 - lr (1 + wd)
    w = np.array([2.0, -3.0])
    for _ in range(10):
        w = optim.sgd(w, w, 0.1)
    assert np.allclose(w, 0.9 ** 10 * np.array([2.0, -3.0]), rtol=1e-12)
    assert np.allclose(optim.sgd(np.array([1.0]), np.array([1.0]), 0.1, wd=0.5), 1 - 0.1 * 1.5)
    # Adam: the first step moves every parameter by lr against the sign of its gradient, whatever its scale
    g = np.array([1e-6, -5.0, 300.0])
    w1, m, v = optim.adam(np.zeros(3), g, np.zeros(3), np.zeros(3), 1, 1e-2, eps=1e-30)
    assert np.allclose(w1, -1e-2 * np.sign(g), rtol=1e-9)
    assert np.allclose(m, 0.1 * g) and np.allclose(v, 1e-3 * g * g)
    # a constant gradient keeps the bias-corrected moments at g and g^2: every step has size lr
    w = np.zeros(3)
    for t in range(1, 8):
        w, m, v = optim.adam(w, g, m if t > 1 else np.zeros(3), v if t > 1 else np.zeros(3), t, 1e-2, eps=1e-30)
    assert np.allclose(w, -7e-2 * np.sign(g), rtol=1e-9)
