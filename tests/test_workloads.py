"""The synthetic configurations have the stated shapes and are reproducible."""
import numpy as np

import workloads as wl


def test_config1_shape():
    w = wl.config1()
    g = w.den
    assert (g.K, g.E, w.B, w.N, w.D) == (16, 48, 1, 50, 16)
    assert np.array_equal(g.dst[0::3], np.arange(16)) and np.array_equal(g.pdf, np.arange(16))
    p = np.exp(g.logw.astype(np.float64)).reshape(16, 3).sum(axis=1)
    np.testing.assert_allclose(p, 1.0, atol=1e-6)
    assert g.init[0] == 0 and np.all(np.isneginf(g.init[1:])) and np.all(g.final == 0)


def test_config2_shape_and_reproducible():
    w = wl.config2()
    g = w.num
    Kb = np.diff(g.state_off)
    assert w.B == 32 and np.all(Kb % 3 == 0) and Kb.min() >= 30 and Kb.max() <= 120
    assert g.E == int(np.sum(2 * Kb - 1)) and np.all(g.logw == np.float32(np.log(0.5)))
    assert np.all(w.lengths >= Kb) and np.all(w.lengths <= 4 * Kb // 3) and w.N == w.lengths.max()
    assert np.array_equal(g.arcs_per_seq(32), 2 * Kb - 1)
    w2 = wl.config2()
    assert np.array_equal(w.emis, w2.emis) and np.array_equal(g.pdf, w2.num.pdf)


def test_config3_small_statistics():
    w = wl.config3(B=2, N=4)
    g = w.den
    assert g.K == 2000 and abs(g.E - 20000) < 1000 and w.D == 84
    deg = np.bincount(g.src, minlength=g.K)
    assert deg.min() >= 1 and abs(deg.mean() - 10) < 0.5
    np.testing.assert_allclose(g.init, -np.log(2000), rtol=1e-6)


def test_config4_graph_has_hubs_and_sourceless_states():
    w = wl.config4(B=2, Nmin=3, Nmax=4)
    g = w.den
    indeg = np.bincount(g.dst, minlength=g.K)
    assert g.K == 6000 and abs(g.E - 60000) < 2000
    assert indeg.max() > 0.1 * g.E                 # top hub takes a large share of all arcs
    assert 0.15 < np.mean(indeg == 0) < 0.35       # many states have no in-arc at all
    g5 = wl.config5(B=2, Lmin=2, Lmax=3).den
    assert np.array_equal(g.dst, g5.dst) and np.array_equal(g.logw, g5.logw)   # config 5 reuses it


def test_config5_lengths():
    w = wl.config5(B=6, Lmin=2, Lmax=5, D=40, K=50)
    Kb = np.diff(w.num.state_off)
    assert np.array_equal(w.lengths, np.rint(1.2 * Kb).astype(np.int32))
    assert w.arc_updates(w.den) == 2 * int(w.lengths.sum()) * w.den.E
    assert w.arc_updates(w.num) == 2 * int(np.sum(w.lengths.astype(np.int64) * (2 * Kb - 1)))
