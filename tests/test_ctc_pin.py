"""An independent pin of the oracle on a third graph family: on the CTC topology with log-softmax emissions,
log Z is minus the CTC loss and the pdf posteriors are the derivative of log Z with respect to the emissions.
The library routine (PyTorch's CPU ctc_loss in double precision, and its autograd) shares nothing with the oracle."""
from __future__ import annotations

import numpy as np
import torch

import oracle
import workloads as wl


def _torch_ctc_loss(emis64, w):
    lp = torch.tensor(emis64.transpose(1, 0, 2).copy(), requires_grad=True)     # [N, B, D]
    targets = torch.tensor(np.concatenate([np.asarray(l, np.int64) for l in w.labels]))
    tl = torch.tensor([len(l) for l in w.labels], dtype=torch.long)
    il = torch.tensor(w.lengths.astype(np.int64))
    return lp, torch.nn.functional.ctc_loss(lp, targets, il, tl, blank=0, reduction="none", zero_infinity=False)


def test_oracle_logz_and_pdf_posteriors_equal_the_ctc_library_routine():
    w = wl.ctc_workload()
    ref = oracle.forward_backward(w.num, w.emis, w.lengths)
    e64 = w.emis.astype(np.float64)
    lp, loss = _torch_ctc_loss(e64, w)
    np.testing.assert_allclose(ref.logz, -loss.detach().numpy(), rtol=1e-10, atol=1e-9)
    # The library's backward pass returns the derivative with respect to the scores in front of a log-softmax,
    # softmax - occupancy; the occupancies (what the derivative of log Z with respect to free emissions is) follow.
    loss.sum().backward()
    occ = (np.exp(e64) - lp.grad.numpy().transpose(1, 0, 2))
    for b in range(w.B):
        T = int(w.lengths[b])
        np.testing.assert_allclose(ref.rho[b][:T], occ[b, :T], rtol=0, atol=1e-9)
    # that reading of the library's gradient, checked by central differences of its loss at sampled entries
    rng = np.random.default_rng(0)
    h = 1e-6
    for _ in range(12):
        b = int(rng.integers(0, w.B)); n = int(rng.integers(0, w.lengths[b])); d = int(np.argmax(ref.rho[b][n]) if rng.random() < 0.7 else rng.integers(0, w.D))
        ep, em = e64.copy(), e64.copy()
        ep[b, n, d] += h; em[b, n, d] -= h
        fd = -(_torch_ctc_loss(ep, w)[1][b].item() - _torch_ctc_loss(em, w)[1][b].item()) / (2 * h)
        assert abs(fd - ref.rho[b][n, d]) <= 1e-6, (b, n, d, fd, ref.rho[b][n, d])


def test_ctc_topology_shape():
    g = wl.ctc_graphs([[3, 3, 5], [7]])
    assert g.K == 7 + 3 and list(g.state_off) == [0, 7, 10]
    # label 3 -> label 3 has no skip arc, label 3 -> label 5 has one
    arcs = set(zip(g.src.tolist(), g.dst.tolist()))
    assert (1, 3) not in arcs and (3, 5) in arcs and (0, 2) not in arcs
    assert list(g.pdf[:7]) == [0, 3, 0, 3, 0, 5, 0]
    assert np.isfinite(g.init[:2]).all() and np.isneginf(g.init[2:7]).all()
    assert np.isfinite(g.final[5:7]).all() and np.isneginf(g.final[:5]).all()
