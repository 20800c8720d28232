"""gsr_step with cfg.save_indices == 2: the column sets of the forward sweep are kept only for the rows that
selected at a near-tie (a selective form of the save of Section 4.2); every other row selects again on its
rebuilt values during the inverse sweep.  Checked against the oracle's variant 3, which follows the same rule."""
import numpy as np
import pytest

import oracle
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth
from gpu_util import Case, assert_close, rel_norm, BF16_REL
from test_gpu_layer import case, run_step, ROW, PLANAR

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def masks_of(I, dg):
    """Column sets [n, k] -> bit masks [n] (uint64)."""
    return (np.uint64(1) << I.astype(np.uint64)).sum(axis=1, dtype=np.uint64)


@pytest.mark.parametrize("name,layout,tol", [("cfg0", ROW, 2.0 ** -5), ("cfg1s", PLANAR, 2.0 ** -6), ("cfg2s", ROW, 2.0 ** -6),
                                             ("tiny", ROW, 2.0 ** -3), ("cfg2s", PLANAR, 0.0)])
def test_step_with_near_tie_list_against_oracle(name, layout, tol):
    c = case(name, layout)
    w = c.w
    ref = oracle.step(c.og, c.ocfg, w.l, c.x0_on_grid(), c.inp.weights, c.inp.w_out, c.inp.b_out, c.inp.target, variant=3,
                      tie_tol=tol, want=("yhat", "XL", "X0rec", "dW", "dwout", "dX0", "ties", "I"))
    keep = {}
    out = run_step(c, save_indices=2, tie_tol=tol, tie_capacity=16 * w.n, keep=keep)
    assert np.isclose(out["loss"], ref["loss"], rtol=1e-4)
    for key in ("yhat", "XL", "X0rec", "dW", "dwout", "dX0"):
        assert_close(key, out[key], ref[key])
    assert_close("X0 rebuilt vs X0", out["X0rec"], c.x0_on_grid(), rtol=1e-4, atol=1e-4)
    # the list itself.  The input of block 1 of layer 0 is the same bits on both sides when C = 2 (it is X_2): there
    # the rows and their column sets must agree exactly.  Further on the two forward sweeps differ by float32
    # rounding, so a row whose gap sits within that rounding of the bar may be listed on one side only.
    stats = gsr.gsr_step_tie_stats(c.gg, keep["cfg"], keep["ws"])
    assert stats["dropped"] == 0
    total, differ = 0, 0
    for l in range(w.l):
        for b in range(1, w.c + 1):
            rows, masks = gsr.gsr_step_tie_export(c.gg, keep["cfg"], keep["ws"], l, b)
            assert len(np.unique(rows)) == len(rows)
            want_rows = np.flatnonzero(ref["ties"][l, b - 1])
            want_masks = masks_of(ref["I"][l, b - 1], w.dg)
            order = np.argsort(rows)
            rows, masks = rows[order], masks[order]
            total += len(rows)
            if l == 0 and b == 1 and w.c == 2:
                assert np.array_equal(rows, want_rows)
            differ += len(np.setxor1d(rows, want_rows))
            both = np.isin(rows, want_rows)
            assert np.array_equal(masks[both], want_masks[rows[both]]), (l, b)
            assert (np.bitwise_count(masks) == w.k).all()
    assert total == stats["listed"]
    print(f"[ties {name}] listed {total} of {w.n * w.c * w.l} (oracle {ref['n_listed']}), on one side only {differ}", flush=True)
    assert differ <= max(2, total // 100)
    if tol > 0:
        assert total > 0
    # reruns are bit-identical, and the forward sweep does not depend on the mode
    a, b2, plain = (run_step(c, raw=True, save_indices=2, tie_tol=tol, tie_capacity=16 * w.n),
                    run_step(c, raw=True, save_indices=2, tie_tol=tol, tie_capacity=16 * w.n), run_step(c, raw=True))
    for key in a:
        assert torch.equal(a[key], b2[key]), key
    assert torch.equal(a["XL"], plain["XL"]) and torch.equal(a["yhat"], plain["yhat"])


def test_list_of_every_row_equals_all_indices_saved_and_an_empty_list_equals_none():
    """A bar no gap exceeds lists every row (k < Dg): the step must then equal the one that keeps all indices, bit
    for bit; a list without room for a single row must equal the step that keeps nothing."""
    c = case("cfg2s", PLANAR)
    w = c.w
    keep = {}
    every = run_step(c, raw=True, save_indices=2, tie_tol=1e30, tie_capacity=16 * w.n, keep=keep)
    saved = run_step(c, raw=True, save_indices=1)
    for key in every:                                    # (room for every row in every one of a block's sixteen sub-lists)
        assert torch.equal(every[key], saved[key]), key
    st = gsr.gsr_step_tie_stats(c.gg, keep["cfg"], keep["ws"])
    assert st["dropped"] == 0 and st["max_per_block"] == w.n and st["listed"] >= w.n * w.c * w.l
    # capacity 1: one place in each of a block's sixteen sub-lists
    keep = {}
    few = run_step(c, raw=True, save_indices=2, tie_tol=1e30, tie_capacity=1, keep=keep)
    st = gsr.gsr_step_tie_stats(c.gg, keep["cfg"], keep["ws"])
    assert st["listed"] <= 16 * w.l * w.c and st["dropped"] > 0
    assert torch.equal(few["XL"], saved["XL"])


def test_near_tie_list_with_bf16_storage():
    """bf16 storage: near-ties are common and selecting again loses the input within a few layers.  With a bar of a
    few bf16 steps the list brings the rebuilt input back to what keeping all indices gives."""
    w = synth.scaled(synth.workload(4), 4001, l=10)            # bf16 storage, dg 32, C 8
    c = Case(w, 0, PLANAR)
    x0 = c.x0_on_grid()
    keep = {}
    listed = run_step(c, save_indices=2, tie_tol=2.0 ** -4, tie_capacity=16 * w.n, keep=keep)
    saved, again = run_step(c, save_indices=1), run_step(c)
    e = lambda r: np.abs(r["X0rec"] - x0).max()
    st = gsr.gsr_step_tie_stats(c.gg, keep["cfg"], keep["ws"])
    print(f"[ties bf16] max|X0 rebuilt - X0|: all kept {e(saved):.3g}, near-ties kept {e(listed):.3g}, none {e(again):.3g}; "
          f"listed {st['listed'] / (w.n * w.c * w.l):.3f} of the rows", flush=True)
    assert e(again) > 5 * e(saved)
    assert e(listed) <= 2 * e(saved)
    for key in ("dW", "dX0", "X0rec"):
        assert rel_norm(listed[key], saved[key]) <= BF16_REL, key


def test_workspace_with_near_tie_list():
    c = case("cfg2s", PLANAR)
    w = c.w
    for L in (8, 56):
        plain = gsr.gsr_workspace_size(c.gg, gsr.Config(**{**c.gcfg.__dict__, "l": L}))[1]
        full = gsr.gsr_workspace_size(c.gg, gsr.Config(**{**c.gcfg.__dict__, "l": L, "save_indices": 1}))[1]
        ties = gsr.gsr_workspace_size(c.gg, gsr.Config(**{**c.gcfg.__dict__, "l": L, "save_indices": 2}))[1]
        cap = (w.n // 32 + 1024 + 15) // 16 * 16           # sixteen sub-lists, each with a counter on its own cache line
        want = (L + 1) * w.c * (16 * 128 + cap * (4 + w.dg // 8))
        assert want <= ties - plain < want + 3 * 256
    with pytest.raises(gsr.GsrError):
        gsr.gsr_workspace_size(c.gg, gsr.Config(**{**c.gcfg.__dict__, "save_indices": 2, "tie_tol": -1.0}))
    with pytest.raises(gsr.GsrError):
        gsr.gsr_workspace_size(c.gg, gsr.Config(**{**c.gcfg.__dict__, "save_indices": 3}))
