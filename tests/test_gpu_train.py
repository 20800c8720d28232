"""GPU parity of the parameter updates, and gsr_step + update as a training loop against the oracle's."""
import numpy as np
import pytest

import oracle
from oracle import optim
import paper_2603_27156_amd as gsr
from paper_2603_27156_amd import synth
from gpu_util import Case, assert_close, rel_norm

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")

PLANAR = gsr.GSR_LAYOUT_GROUP_PLANAR


def test_sgd_and_adam_updates_against_the_definitions():
    rng = np.random.default_rng(2)
    n = 100_003
    dv = torch.device("cuda:0")
    w0 = rng.standard_normal(n).astype(np.float32)
    w = torch.from_numpy(w0.copy()).to(dv)
    ref = w0.astype(np.float64)
    for _ in range(3):
        g = rng.standard_normal(n).astype(np.float32)
        gsr.gsr_sgd_update(w, torch.from_numpy(g).to(dv), 0.05, 0.01)
        ref = optim.sgd(ref, g, 0.05, 0.01)
    assert_close("sgd", w.cpu().numpy(), ref)
    w = torch.from_numpy(w0.copy()).to(dv)
    m, v = torch.zeros_like(w), torch.zeros_like(w)
    rw, rm, rv = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in range(1, 6):
        g = (rng.standard_normal(n) * 10.0 ** rng.integers(-4, 3, n)).astype(np.float32)
        gsr.gsr_adam_update(w, torch.from_numpy(g).to(dv), m, v, t, 1e-2, weight_decay=1e-3)
        rw, rm, rv = optim.adam(rw, g, rm, rv, t, 1e-2, wd=1e-3)
    assert_close("adam w", w.cpu().numpy(), rw)
    assert_close("adam m", m.cpu().numpy(), rm)
    assert_close("adam v", v.cpu().numpy(), rv)
    with pytest.raises(gsr.GsrError):
        gsr.gsr_adam_update(w, w, m, v, 0, 1e-2)


def test_training_loop_follows_the_oracle_and_lowers_the_loss():
    """Three steps of forward + inverse + backward + Adam on both sides (the trajectories stay within the
    float32 bar), then 40 more steps on the GPU: the loss goes down."""
    w = synth.scaled(synth.workload(1), 1501, l=3)
    c = Case(w, 0, PLANAR)
    dv = c.dev
    f32 = dict(dtype=torch.float32, device=dv)
    x0 = c.to_dev(c.inp.x0)
    W = torch.from_numpy(np.ascontiguousarray(c.inp.weights[:w.l])).to(dv)
    w_out = torch.from_numpy(c.inp.w_out.copy()).to(dv)
    b_out = torch.zeros(1, **f32)
    target = torch.from_numpy(c.inp.target).to(dv)
    params = [W, w_out, b_out]
    grads = [torch.empty_like(W), torch.empty(w.d, **f32), torch.zeros(1, **f32)]
    state = [(torch.zeros_like(p), torch.zeros_like(p)) for p in params]
    loss = torch.zeros(1, **f32)
    oW, ow, ob = c.inp.weights[:w.l].astype(np.float64), c.inp.w_out.astype(np.float64), 0.0
    ostate = [(np.zeros_like(oW), np.zeros_like(oW)), (np.zeros_like(ow), np.zeros_like(ow)), (np.zeros(1), np.zeros(1))]
    lr = 2e-3
    losses = []
    for t in range(1, 44):
        gsr.gsr_step(c.gg, c.gcfg, x0, W, w_out, b_out, target, loss, grads[0], grads[1], grads[2])
        for p, g, (m, v) in zip(params, grads, state):
            gsr.gsr_adam_update(p, g, m, v, t, lr)
        losses.append(float(loss.item()))
        if t <= 3:
            ref = oracle.step(c.og, c.ocfg, w.l, c.x0_on_grid(), oW.astype(np.float32), ow.astype(np.float32), float(np.float32(ob)),
                              c.inp.target)
            assert np.isclose(losses[-1], ref["loss"], rtol=2e-4), (t, losses[-1], ref["loss"])
            oW, m0, v0 = optim.adam(oW, ref["dW"], *ostate[0], t, lr); ostate[0] = (m0, v0)
            ow, m1, v1 = optim.adam(ow, ref["dwout"], *ostate[1], t, lr); ostate[1] = (m1, v1)
            nb, m2, v2 = optim.adam(np.array([ob]), np.array([ref["dbout"]]), *ostate[2], t, lr); ostate[2] = (m2, v2)
            ob = float(nb[0])
            # parameters after the update: Adam divides by sqrt(v), which amplifies relative differences of tiny
            # gradients, so the comparison is in norm
            assert rel_norm(W.cpu().numpy(), oW) < 1e-4 and rel_norm(w_out.cpu().numpy(), ow) < 1e-4
    print("[train] loss", " ".join(f"{x:.4f}" for x in losses[::6]), flush=True)
    assert losses[-1] < 0.9 * losses[0]
    assert all(np.isfinite(losses))
