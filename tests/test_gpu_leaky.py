"""GPU parity of the leaky-HMM comparison mode (fb_leaky_posteriors) against oracle/leaky.py, through the C-ABI."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import leaky as oleaky

pytestmark = pytest.mark.gpu

TOL_LOGZ_REL = 1e-4      # as for the exact path
TOL_POST_ABS = 1e-5


@pytest.fixture(scope="module")
def fb():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2112_00709_amd as lib
    lib.lib()
    lib.POISON_NEW_BUFFERS = True
    return lib


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(fb, g, D, emis, lengths, leak):
    import torch
    G = fb.graph_from(g, D)
    logz, post = fb.fb_leaky_posteriors(G, dev(emis), dev(lengths.astype(np.int32)), leak)
    torch.cuda.synchronize()
    out = logz.cpu().numpy(), post.cpu().numpy()
    G.destroy()
    return out


def compare(fb, g, D, emis, lengths, leak, sel=None, name=""):
    B = emis.shape[0]
    sel = list(range(B)) if sel is None else list(sel)
    print(f"[gpu-case] {name}: fb_leaky_posteriors B={B} N={emis.shape[1]} D={D} K={g.K} E={g.E} leak={leak}", flush=True)
    ref = oleaky.forward_backward(g, emis, lengths, leak, sel=sel)
    logz, post = run(fb, g, D, emis, lengths, leak)
    for i, b in enumerate(sel):
        T = int(lengths[b])
        if np.isneginf(ref.logz[i]):
            assert np.isneginf(logz[b]) and np.all(post[b] == 0), f"{name} b={b}"
            continue
        assert abs(logz[b] - ref.logz[i]) <= TOL_LOGZ_REL * max(1.0, abs(ref.logz[i])), f"{name} b={b}: {logz[b]} vs {ref.logz[i]}"
        err = np.abs(post[b] - ref.rho[i]).max()
        assert err <= TOL_POST_ABS, f"{name} b={b}: pdf posterior err {err}"
    for b in range(B):
        T = int(lengths[b])
        assert np.all(post[b, T:] == 0)
        assert not np.isnan(post[b]).any()
    return logz, post


@pytest.mark.parametrize("leak", [0.0, 1e-5, 0.1])
def test_small_graphs_every_sequence(fb, leak):
    rng = np.random.default_rng(31)
    g = wl.random_graph(rng, 90, 11, mean_extra_deg=3.0)
    emis = (rng.standard_normal((5, 14, 11)) * 2).astype(np.float32)
    compare(fb, g, 11, emis, np.array([14, 1, 9, 14, 3], np.int32), leak, name="random graph K=90")
    g2 = wl.tiny_graph(9, 6, 4)                                       # -inf init/final entries, sourceless states
    e2 = rng.normal(size=(2, 7, 4)).astype(np.float32)
    e2[0, 3, 1] = -np.inf
    compare(fb, g2, 4, e2, np.array([7, 5], np.int32), leak, name="tiny graph with -inf entries")


def test_hub_rows_and_several_blocks(fb):
    """A Zipf graph: rows of more than 64 arcs (walked by a wave each) and more than 1024 short rows (several blocks),
    ragged lengths, an odd state count."""
    w = wl.config4(K=2501, B=6, Nmin=5, Nmax=30, D=120)
    deg = np.bincount(w.den.dst, minlength=w.den.K)
    assert deg.max() > 64
    compare(fb, w.den, w.D, w.emis, w.lengths, 0.01, name="config4-like, K=2501")
    w3 = wl.config3(K=2000, B=4, N=20, D=84)
    compare(fb, w3.den, w3.D, w3.emis, w3.lengths, 1e-3, name="config3")


def test_no_leak_is_the_exact_path(fb):
    import torch
    w = wl.config4(K=1500, B=4, Nmin=8, Nmax=25, D=100)
    logz, post = run(fb, w.den, w.D, w.emis, w.lengths, 0.0)
    G = fb.graph_from(w.den, w.D)
    e, l = dev(w.emis), dev(w.lengths.astype(np.int32))
    a, _, za = fb.fb_alpha(G, e, l)
    b, _, _ = fb.fb_beta(G, e, l)
    _, rho = fb.fb_posteriors(G, a, b, l, w.B, w.N, want_state=False)
    torch.cuda.synchronize()
    za, rho = za.cpu().numpy(), rho.cpu().numpy()
    G.destroy()
    assert np.all(np.abs(logz - za) <= TOL_LOGZ_REL * np.maximum(1.0, np.abs(za)))
    assert np.abs(post - rho).max() <= 2 * TOL_POST_ABS


def test_a_frame_nobody_can_emit(fb):
    rng = np.random.default_rng(4)
    g = wl.random_graph(rng, 40, 5, mean_extra_deg=2.0)
    emis = rng.normal(size=(3, 8, 5)).astype(np.float32)
    emis[1, 4, :] = -np.inf
    emis = np.concatenate([emis, np.full((3, 2, 5), np.nan, np.float32)], axis=1)   # padding is never read
    logz, post = compare(fb, g, 5, emis, np.array([8, 8, 6], np.int32), 0.05, name="a frame of zero-bar")
    assert np.isneginf(logz[1]) and np.isfinite(logz[0]) and np.isfinite(logz[2])


def test_a_pdf_no_state_is_tied_to_far_above_the_others(fb):
    """The per-frame scale of the emissions is the largest emission a state has, not the largest of the row: an
    unused pdf 130 binary orders above the rest must not flush the frame's factors to zero."""
    rng = np.random.default_rng(8)
    g = wl.random_graph(rng, 300, 40, mean_extra_deg=3.0)
    g.pdf[:] = g.pdf % 20
    emis = (rng.standard_normal((3, 10, 40)) * 2).astype(np.float32)
    emis[:, ::2, 39] = 90.0
    emis[1, 3, 30] = 200.0
    compare(fb, g, 40, emis, np.array([10, 7, 10], np.int32), 1e-3, name="unused pdf far above the others")


def test_config4_full_size_sampled(fb):
    w = wl.config4()
    order = np.argsort(w.lengths)
    sel = [int(order[0]), int(order[len(order) // 2]), int(order[-1])]
    compare(fb, w.den, w.D, w.emis, w.lengths, 1e-5, sel=sel, name="config4 full size")


def test_argument_errors(fb):
    rng = np.random.default_rng(2)
    g = wl.random_graph(rng, 20, 4)
    G = fb.graph_from(g, 4)
    emis, lengths = dev(np.zeros((2, 3, 4), np.float32)), dev(np.array([3, 2], np.int32))
    with pytest.raises(fb.FBError):
        fb.fb_leaky_posteriors(G, emis, lengths, -0.1)
    with pytest.raises(fb.FBError):
        fb.fb_leaky_posteriors(G, emis, lengths, float("nan"))
    import torch
    with pytest.raises(fb.FBError):
        fb.fb_leaky_posteriors(G, emis, lengths, 0.1, ws=torch.empty((16,), dtype=torch.uint8, device="cuda"))
    w = wl.config2(B=2, Lmin=2, Lmax=3, D=4)
    Gp = fb.graph_from(w.num, 4)
    with pytest.raises(fb.FBError):
        fb.fb_leaky_posteriors(Gp, dev(w.emis), dev(w.lengths.astype(np.int32)), 0.1)
    G.destroy(); Gp.destroy()
