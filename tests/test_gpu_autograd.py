"""The LF-MMI objective as a PyTorch autograd function (the step around the hot path: network output in,
objective out, Eq. 17 as its derivative), checked against the fp64 oracle.  GPU only."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

TOL_LOGZ_REL = 1e-4
TOL_POST_ABS = 1e-5


@pytest.fixture(scope="module")
def fb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2112_00709_amd as lib
    lib.lib()
    lib.POISON_NEW_BUFFERS = True   # outputs and workspaces start out as NaN
    return lib


def test_objective_and_its_derivative_match_the_oracle(fb):
    import torch
    from paper_2112_00709_amd.autograd import lfmmi_loss
    w = wl.config5(K=800, B=5, Lmin=3, Lmax=9, D=120)
    print("autograd: config5 K=800 B=5, oracle LF-MMI", flush=True)
    ref = oracle.lfmmi(w.den, w.num, w.emis, w.lengths)
    den, num = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    emis = torch.from_numpy(w.emis).cuda().requires_grad_(True)
    lengths = torch.from_numpy(w.lengths).cuda()
    loss, zn, zd = lfmmi_loss(emis, lengths, den, num)
    assert abs(float(loss.detach()) - ref.loss) <= TOL_LOGZ_REL * float(np.sum(np.abs(ref.logz_num) + np.abs(ref.logz_den)))
    assert not zn.requires_grad and not zd.requires_grad
    (loss * -0.5).sum().backward()                      # an upstream factor, as a recipe that minimises -objective / 2 has
    got = emis.grad.cpu().numpy()
    assert np.abs(got - (-0.5) * ref.grad).max() <= TOL_POST_ABS
    den.destroy(); num.destroy()


def test_sub_batches_accumulate_the_gradient_of_the_whole_batch(fb):
    """B utterances as one batch, and as F = 2 sub-batches with one backward() each: the same parameter gradient
    (the objective is a sum over utterances), for a one-layer "network" emis = X W."""
    import torch
    from paper_2112_00709_amd.autograd import lfmmi_loss
    w = wl.config5(K=600, B=6, Lmin=3, Lmax=8, D=90)
    rng = np.random.default_rng(7)
    F_in = 17
    X = torch.from_numpy(rng.normal(size=(w.B, w.N, F_in)).astype(np.float32)).cuda()
    W0 = torch.from_numpy((rng.normal(size=(F_in, w.D)) * 0.7).astype(np.float32)).cuda()
    lengths = torch.from_numpy(w.lengths).cuda()
    den = fb.graph_from(w.den, w.D)

    def run(groups):
        W = W0.clone().requires_grad_(True)
        total = 0.0
        for sel in groups:
            num = fb.graph_from(wl.packed_subset(w.num, sel), w.D)
            idx = torch.as_tensor(sel, device="cuda")
            emis = X[idx] @ W
            loss, _, _ = lfmmi_loss(emis, lengths[idx].contiguous(), den, num)
            (-loss.sum() / w.B).backward()
            total += float(loss.detach())
            torch.cuda.synchronize()
            num.destroy()
        return total, W.grad.detach().cpu().numpy().astype(np.float64)

    print("autograd: whole batch", flush=True)
    l1, g1 = run([list(range(w.B))])
    print("autograd: two sub-batches", flush=True)
    l2, g2 = run([[0, 1, 2], [3, 4, 5]])
    assert abs(l1 - l2) <= 1e-6 * max(1.0, abs(l1))
    assert np.abs(g1 - g2).max() <= 1e-4 * max(1.0, np.abs(g1).max())
    # and the whole-batch gradient is the oracle's Eq. 17 pushed through the layer: dL/dW = X^T grad
    emis_np = (X.cpu().numpy().astype(np.float64) @ W0.cpu().numpy().astype(np.float64)).astype(np.float32)
    ref = oracle.lfmmi(w.den, w.num, emis_np, w.lengths)
    want = -np.einsum("bnf,bnd->fd", X.cpu().numpy().astype(np.float64), ref.grad.astype(np.float64)) / w.B
    assert np.abs(g1 - want).max() <= 2e-4 * max(1.0, np.abs(want).max())
    den.destroy()
