"""The pipeline of Algorithms 1 and 2 as the walk-throughs of Sections 4.3 / 4.4 print it (two groups).
TEST INFRASTRUCTURE ONLY, plain numpy, float64; the sparse product is oracle.spmm.

Here the block places a row's sums in the row's OWN recorded columns,
    block(V, I)[i, I[i,t]] = sum_j a_ij V[j,t],
which is what the printed block results of Sections 4.3 and 4.4 follow (the Section 4.1 example and eq. (10)
follow the other placement, every neighbour at its own column: oracle.aggregate).  There are no weights
in this pipeline: Algorithm 1 writes GSR-Forward(V, I, G).

Pinned by the printed numbers of Sections 4.1, 4.3 and 4.4 (tests/golden/).  The two matrices that end the
Section 4.4 walk-through follow no consistent rule, so no printed number pins what alg2_layer_backward RETURNS;
its intermediate steps are pinned by the printed ones, and the returned planes by dense algebra over A^T and
the adjoint identity of the backward block on a directed graph.
"""
from __future__ import annotations

import numpy as np

import oracle


def scatter(V, I, dg: int):
    """Dense [n, dg] with V[i,t] at column I[i,t], zero elsewhere."""
    V = np.asarray(V, dtype=np.float64)
    n = V.shape[0]
    out = np.zeros((n, dg), dtype=np.float64)
    out[np.arange(n)[:, None], np.asarray(I)] = V
    return out


def slot_block(g: oracle.Graph, V, I, dg: int, transpose: bool = False):
    """Forward block of the walk-throughs: slot-wise sums over the neighbours, placed at the row's own columns."""
    return scatter(oracle.spmm(g, np.asarray(V, dtype=np.float64), transpose=transpose), I, dg)


def block_backward(g: oracle.Graph, M, I):
    """Backward block (Section 4.1 example, eq. (11)): only the entries of M at the recorded positions are read;
    they are summed over G^T and stand at the row's own recorded positions."""
    M = np.asarray(M, dtype=np.float64)
    n, dg = M.shape
    Vg = M[np.arange(n)[:, None], np.asarray(I)]
    return slot_block(g, Vg, I, dg, transpose=True)


def alg1_layer_forward(g: oracle.Graph, X1, X2, k: int):
    """One pass of the loop body of Algorithm 1.  Returns (X1_new, X2_new, (V1, I1, V2, I2))."""
    X1 = np.asarray(X1, dtype=np.float64)
    X2 = np.asarray(X2, dtype=np.float64)
    dg = X1.shape[1]
    V1, I1, _ = oracle.gs(X1, k)
    M1 = slot_block(g, V1, I1, dg)
    X2n = X2 + M1
    V2, I2, _ = oracle.gs(X2n, k)
    M2 = slot_block(g, V2, I2, dg)
    X1n = scatter(V1, I1, dg) + M2
    return X1n, X2n, (V1, I1, V2, I2)


def alg2_layer_backward(g: oracle.Graph, G1, G2, k: int):
    """One pass of the loop body of Algorithm 2, step by step as printed.
    Returns (g1, g2, dict of the intermediate results)."""
    G1 = np.asarray(G1, dtype=np.float64)
    G2 = np.asarray(G2, dtype=np.float64)
    dg = G1.shape[1]
    V2, I2, _ = oracle.gs(G2, k)
    B2 = slot_block(g, V2, I2, dg)
    M1 = G1 - B2
    V1, I1, _ = oracle.gs(M1, k)
    Z1 = slot_block(g, V1, I1, dg)
    M2 = scatter(V2, I2, dg) - Z1
    g1 = block_backward(g, M1, I1)
    g2 = block_backward(g, M2, I2)
    return g1, g2, dict(V2=V2, I2=I2, B2=B2, M1=M1, V1=V1, I1=I1, Z1=Z1, M2=M2)
