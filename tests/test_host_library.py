"""Host-side logic of libfb_amd, no GPU: the library loads and exports every
symbol of include/fb.h, argument errors are reported as codes, the graph layout
(integer work) is bit-exact against the oracle's stable sorts, and the static
work plan the kernels walk computes the same sparse products as a direct
evaluation."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2112_00709_amd as fb
import workloads as wl
from oracle import layout as olayout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(fb.LIB_PATH):
        from paper_2112_00709_amd import build
        build.build_library()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "fb.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\(", header)) - {"defined", "__cplusplus"}
    declared = {d for d in declared if d.startswith(("fb_", "lfmmi_"))}
    assert declared == set(fb.SYMBOLS)
    L = fb.lib()
    for name in declared:
        assert getattr(L, name) is not None


def _host_graph(g, D):
    return fb.graph_from(g, D, host_only=True)


@pytest.mark.parametrize("case", ["config1", "chains", "zipf"])
def test_graph_layout_bit_exact(case):
    if case == "config1":
        w = wl.config1(); g = w.den
    elif case == "chains":
        w = wl.config2(B=5); g = w.num
    else:
        w = wl.config4(K=1500, B=2, Nmin=3, Nmax=4, D=200); g = w.den
    h = _host_graph(g, w.D)
    ref = olayout.graph_layout(g.K, w.D, g.src, g.dst, g.logw, g.pdf)
    for name, want in ref.items():
        got = fb.fb_graph_layout(h, name)
        assert got.dtype == want.dtype and got.shape == want.shape, name
        assert np.array_equal(got.view(np.int32), want.view(np.int32)), name     # bit-exact, weights included
    h.destroy()


def _direct_product(K, rows, cols, w2, x):
    """y[r] = log2-sum-exp2 over entries (r, c) of w2 + x[c], in double."""
    y = np.full(K, -np.inf)
    t = w2 + x[cols]
    for r in range(K):
        sel = t[rows == r]
        if sel.size and np.max(sel) > -np.inf:
            m = np.max(sel)
            y[r] = m + np.log2(np.sum(np.exp2(sel - m)))
    return y


def _pack(graphs):
    src, dst, lw, pdf, init, fin, off = [], [], [], [], [], [], [0]
    for g in graphs:
        src.append(g.src + off[-1]); dst.append(g.dst + off[-1]); lw.append(g.logw)
        pdf.append(g.pdf); init.append(g.init); fin.append(g.final); off.append(off[-1] + g.K)
    return wl.Graph(K=off[-1], src=np.concatenate(src).astype(np.int32), dst=np.concatenate(dst).astype(np.int32),
                    logw=np.concatenate(lw).astype(np.float32), pdf=np.concatenate(pdf).astype(np.int32),
                    init=np.concatenate(init).astype(np.float32), final=np.concatenate(fin).astype(np.float32),
                    state_off=np.array(off, dtype=np.int32))


@pytest.mark.parametrize("case", ["zipf_hubs", "zipf_clones", "packed_clones", "uniform", "chains"])
def test_kernel_schedule_computes_the_sparse_products(case):
    rng = np.random.default_rng(5)
    if case == "zipf_hubs":          # hub rows are spread over 2 ... 64 lanes
        w = wl.config4(K=900, B=2, Nmin=3, Nmax=4, D=64); g = w.den
    elif case == "zipf_clones":      # the largest hubs are too long for one slice and get clones
        w = wl.config4(K=3500, B=2, Nmin=3, Nmax=4, D=64); g = w.den
    elif case == "packed_clones":    # packed graphs of different sizes, the smaller one with cloned hubs
        w = wl.config4(K=3500, B=2, Nmin=3, Nmax=4, D=64)
        g = _pack([wl.config4(K=3800, B=1, Nmin=3, Nmax=4, D=64).den, w.den])
    elif case == "uniform":
        w = wl.config3(K=300, B=2, N=3, D=20); g = w.den
    else:
        w = wl.config2(B=4); g = w.num
    h = _host_graph(g, w.D)
    off = g.state_off if g.packed else np.array([0, g.K])
    w2 = (g.logw.astype(np.float64) * np.log2(np.e)).astype(np.float32).astype(np.float64)
    for sub in range(len(off) - 1):
        k0, k1 = int(off[sub]), int(off[sub + 1])
        Ks = k1 - k0
        x = rng.normal(size=Ks) * 5
        x[rng.integers(0, Ks)] = -np.inf
        inside = (g.src >= k0) & (g.src < k1)
        src, dst, ww = g.src[inside] - k0, g.dst[inside] - k0, w2[inside]
        parallel = np.unique(src.astype(np.int64) * Ks + dst).size < src.size
        for which, rows, cols in ((0, dst, src), (1, src, dst)):
            y = fb.fb_graph_schedule_apply_host(h, which, sub, x, np.full(Ks, 123.0))
            want = _direct_product(Ks, rows, cols, ww, x)
            fin = np.isfinite(want)
            assert np.array_equal(np.isneginf(y), np.isneginf(want))
            # the plans hold the (+)-sum of parallel arcs rounded to float once more: 1e-6 where a graph has any
            np.testing.assert_allclose(y[fin], want[fin], rtol=0, atol=1e-6 if parallel else 1e-9)
        gam = rng.random(Ks)
        y = fb.fb_graph_schedule_apply_host(h, 2, sub, gam, np.zeros(w.D))
        want = np.bincount(g.pdf[k0:k1], weights=gam, minlength=w.D)
        np.testing.assert_allclose(y, want, atol=1e-12)
    h.destroy()


@pytest.mark.parametrize("seed", range(8))
def test_kernel_schedule_on_random_graph_shapes(seed):
    """The plans of randomly shaped graphs (hubs, parallel arcs, -inf weights, packed graphs of unequal size, sourceless
    and sinkless states), interpreted on the host, against the direct sparse products."""
    rng = np.random.default_rng(100 + seed)
    kind = seed % 4
    if kind == 0:
        g = wl.random_graph(rng, int(rng.integers(5, 3000)), 9, zipf_s=float(rng.uniform(1.0, 1.6)),
                            mean_extra_deg=float(rng.uniform(0.5, 14)))
    elif kind == 1:
        g = _pack([wl.random_graph(rng, int(rng.integers(2, 1800)), 9, zipf_s=1.3) for _ in range(int(rng.integers(2, 5)))])
    elif kind == 2:
        g = _pack([wl.tiny_graph(int(rng.integers(0, 99)), int(rng.integers(1, 9)), 9) for _ in range(3)])
    else:
        g0 = wl.random_graph(rng, 5200, 9, mean_extra_deg=1.0)          # one giant hub and parallel arcs into it
        every = np.concatenate([np.arange(g0.K), np.arange(0, g0.K, 3)]).astype(np.int32)
        g = wl.Graph(g0.K, np.concatenate([g0.src, every]), np.concatenate([g0.dst, np.full(every.size, 7, np.int32)]),
                     np.concatenate([g0.logw, rng.normal(size=every.size).astype(np.float32)]), g0.pdf, g0.init, g0.final)
    h = _host_graph(g, 9)
    off = g.state_off if g.packed else np.array([0, g.K])
    w2 = (g.logw.astype(np.float64) * np.log2(np.e)).astype(np.float32).astype(np.float64)
    for sub in range(len(off) - 1):
        k0, k1 = int(off[sub]), int(off[sub + 1])
        Ks = k1 - k0
        x = rng.normal(size=Ks) * 5
        x[rng.integers(0, Ks, size=max(1, Ks // 10))] = -np.inf
        inside = (g.src >= k0) & (g.src < k1)
        src, dst, ww = g.src[inside] - k0, g.dst[inside] - k0, w2[inside]
        for which, rows, cols in ((0, dst, src), (1, src, dst)):
            y = fb.fb_graph_schedule_apply_host(h, which, sub, x, np.full(Ks, 123.0))
            want = _direct_product(Ks, rows, cols, ww, x)
            fin = np.isfinite(want)
            assert np.array_equal(np.isneginf(y), np.isneginf(want))
            np.testing.assert_allclose(y[fin], want[fin], rtol=0, atol=1e-6)
    h.destroy()


@pytest.mark.parametrize("seed", range(6))
def test_plans_with_weights_as_powers_of_two(seed):
    """The form of the plans the multiplying kernel instantiation walks (weights as 2^w; zero-bar arcs and padding
    gather the dump slot; the lanes of a row spread over several lanes all write the row's total to its state):
    interpreted on the host it gives the same products as the adding form, and the walk finds nothing the
    multiplying kernel could not rely on.  Graphs with hubs, clones, parallel arcs, zero-bar weights; packed graphs;
    a weight out of range is refused."""
    rng = np.random.default_rng(300 + seed)
    kind = seed % 3
    if kind == 0:
        g = wl.random_graph(rng, int(rng.integers(1100, 3600)), 9, zipf_s=float(rng.uniform(1.0, 1.5)),
                            mean_extra_deg=float(rng.uniform(2, 12)))
    elif kind == 1:
        g = _pack([wl.random_graph(rng, int(rng.integers(200, 1500)), 9, zipf_s=1.3) for _ in range(3)])
    else:
        g0 = wl.random_graph(rng, 5200, 9, mean_extra_deg=1.0)          # one giant hub and parallel arcs into it
        every = np.concatenate([np.arange(g0.K), np.arange(0, g0.K, 3)]).astype(np.int32)
        g = wl.Graph(g0.K, np.concatenate([g0.src, every]), np.concatenate([g0.dst, np.full(every.size, 7, np.int32)]),
                     np.concatenate([g0.logw, rng.normal(size=every.size).astype(np.float32)]), g0.pdf, g0.init, g0.final)
    logw = g.logw.copy()
    logw[rng.integers(0, logw.size, size=logw.size // 20)] = -np.inf     # zero-bar arcs
    logw[rng.integers(0, logw.size, size=5)] = -30.0                      # 2^-43: tiny, in range
    g = wl.Graph(g.K, g.src, g.dst, logw, g.pdf, g.init, g.final, state_off=g.state_off if g.packed else None)
    h = _host_graph(g, 9)
    off = g.state_off if g.packed else np.array([0, g.K])
    for sub in range(len(off) - 1):
        Ks = int(off[sub + 1] - off[sub])
        x = rng.normal(size=Ks) * 30                                      # a wide range: the maximum matters
        x[rng.integers(0, Ks, size=max(1, Ks // 10))] = -np.inf
        for which in (0, 1):
            want = fb.fb_graph_schedule_apply_host(h, which, sub, x, np.full(Ks, 123.0))
            y = fb.fb_graph_schedule_apply_host(h, which + 3, sub, x, np.full(Ks, 123.0))
            assert np.array_equal(np.isneginf(y), np.isneginf(want))
            fin = np.isfinite(want)
            np.testing.assert_allclose(y[fin], want[fin], rtol=0, atol=1e-5)
    h.destroy()
    far = g.logw.copy()
    far[g.src == g.src[np.flatnonzero(np.isfinite(far))[0]]] = -60.0      # every arc out of one state 2^-86.6: out of range
    h = _host_graph(wl.Graph(g.K, g.src, g.dst, far, g.pdf, g.init, g.final, state_off=g.state_off if g.packed else None), 9)
    with pytest.raises(fb.FBError) as err:
        fb.fb_graph_schedule_apply_host(h, 3, 0, np.zeros(int(off[1] - off[0])), np.zeros(int(off[1] - off[0])))
    assert err.value.code == fb.FB_EUNSUPPORTED
    h.destroy()


def test_hub_graphs_really_have_long_rows():
    w = wl.config4(K=900, B=2, Nmin=3, Nmax=4, D=64)
    assert np.bincount(w.den.dst, minlength=900).max() > 32 * 32     # a row spread over all 64 lanes
    w = wl.config4(K=3500, B=2, Nmin=3, Nmax=4, D=64)
    assert np.bincount(w.den.dst, minlength=3500).max() > 64 * 64       # a row that needs a clone


def _raises(code, fn, *a, **k):
    with pytest.raises(fb.FBError) as e:
        fn(*a, **k)
    assert e.value.code == code, str(e.value)
    assert str(e.value)


def test_graph_create_argument_errors():
    g = wl.config1().den
    ok = dict(K=g.K, src=g.src, dst=g.dst, logw=g.logw, pdf=g.pdf, init=g.init, final=g.final, D=16, host_only=True)

    def make(**kw):
        a = dict(ok); a.update(kw)
        fb.fb_graph_create(**a).destroy()

    make()
    _raises(fb.FB_EINVAL, make, K=0)
    _raises(fb.FB_EINVAL, make, D=0)
    bad = g.dst.copy(); bad[3] = 16
    _raises(fb.FB_EINVAL, make, dst=bad)
    bad = g.src.copy(); bad[0] = -1
    _raises(fb.FB_EINVAL, make, src=bad)
    bad = g.pdf.copy(); bad[5] = 16
    _raises(fb.FB_EINVAL, make, pdf=bad)
    _raises(fb.FB_EINVAL, make, D=15)
    for val in (np.nan, np.inf):
        bad = g.logw.copy(); bad[7] = val
        _raises(fb.FB_EINVAL, make, logw=bad)
        bad = g.init.copy(); bad[2] = val
        _raises(fb.FB_EINVAL, make, init=bad)
        bad = g.final.copy(); bad[2] = val
        _raises(fb.FB_EINVAL, make, final=bad)
    ninf = g.logw.copy(); ninf[7] = -np.inf          # the semiring zero is a legal weight
    make(logw=ninf)
    # packed graphs
    c = wl.config2(B=3).num
    okp = dict(K=c.K, src=c.src, dst=c.dst, logw=c.logw, pdf=c.pdf, init=c.init, final=c.final, D=84,
               state_off=c.state_off, host_only=True)
    fb.fb_graph_create(**okp).destroy()
    so = c.state_off.copy(); so[1], so[2] = so[2], so[1]
    _raises(fb.FB_EINVAL, lambda: fb.fb_graph_create(**dict(okp, state_off=so)))
    so = c.state_off.copy(); so[-1] -= 1
    _raises(fb.FB_EINVAL, lambda: fb.fb_graph_create(**dict(okp, state_off=so)))
    so = c.state_off.copy(); so[1] += 1               # the arc into the moved state now crosses two graphs
    _raises(fb.FB_EINVAL, lambda: fb.fb_graph_create(**dict(okp, state_off=so)))
    L = fb.lib()
    assert L.fb_graph_create(None, 1, 0, None, None, None, None, None, None, 1, 0, None, 1) == fb.FB_EINVAL
    h = ctypes.c_void_p()
    assert L.fb_graph_create(ctypes.byref(h), 4, 0, None, None, None, None, None, None, 1, 0, None, 1) == fb.FB_EINVAL


def test_too_large_graph_is_unsupported_not_a_crash():
    K = fb.fb_limits_max_states(84, True) * 2
    z = np.zeros(K, np.float32)
    _raises(fb.FB_EUNSUPPORTED, fb.fb_graph_create, K, np.arange(K) % K, (np.arange(K) + 1) % K, z,
            np.zeros(K, np.int32), z, z, 84, host_only=True)
    assert fb.fb_limits_max_states(84, True) > 6000 and fb.fb_limits_max_states(3000, True) > 6000
    assert fb.fb_limits_max_states(3000, False) > 450


def test_compute_calls_reject_bad_arguments_without_a_gpu():
    g = wl.config1().den
    h = _host_graph(g, 16)
    L = fb.lib()
    one = ctypes.c_void_p(256)      # never dereferenced: the checks come first
    assert L.fb_alpha(None, one, one, 1, 50, 16, None, None, None, None) == fb.FB_EINVAL
    assert L.fb_alpha(h.handle, one, one, 1, 50, 16, None, None, None, None) == fb.FB_EINVAL     # host-only graph
    assert b"HOST_ONLY" in L.fb_last_error()
    assert L.fb_beta(h.handle, None, one, 1, 50, 16, None, None, None, None) == fb.FB_EINVAL
    assert L.fb_posteriors(h.handle, one, one, None, 1, 50, 16, one, one, None) == fb.FB_EINVAL
    assert L.lfmmi_loss_grad(h.handle, h.handle, one, one, 1, 50, 16, one, None, None, one, one, 1 << 30, None) == fb.FB_EINVAL
    assert L.fb_lfmmi_workspace_bytes(None, None, 1, 1, 1) == 0
    assert L.fb_graph_layout(h.handle, 99, one, 4) == fb.FB_EINVAL
    assert L.fb_graph_layout(h.handle, 0, one, 3) == fb.FB_EINVAL
    assert L.fb_graph_layout_size(h.handle, 99) == fb.FB_EINVAL
    assert L.fb_graph_destroy(None) == fb.FB_OK
    assert L.fb_strerror(fb.FB_EUNSUPPORTED) and L.fb_strerror(12345)
    h.destroy()


def test_check_lengths():
    fb.fb_check_lengths(np.array([1, 5, 3]), 5)
    _raises(fb.FB_EINVAL, fb.fb_check_lengths, np.array([1, 6, 3]), 5)
    _raises(fb.FB_EINVAL, fb.fb_check_lengths, np.array([0, 2]), 5)


@pytest.mark.parametrize("seed", range(6))
def test_probability_domain_plans(seed):
    """The plan the probability-domain kernel walks (two arcs per lane and unit, weights as 2^w, the lanes of a long
    row added up, clones, padding that reads the dump slot or repeats an address), interpreted on the host in
    ordinary arithmetic: y = A x for the forward (which = 5) and the backward (6) matrix, against the direct sparse
    product.  Graphs with hubs over several lanes, clones, parallel arcs, zero-bar weights, states without arcs.  The
    modelled gather cycles of a step are never below two per gather.  Graphs the kernel cannot take have no plan:
    packed ones, small ones, weights far out of range."""
    rng = np.random.default_rng(500 + seed)
    kind = seed % 3
    if kind == 0:
        g = wl.random_graph(rng, int(rng.integers(1100, 3600)), 9, zipf_s=float(rng.uniform(1.0, 1.5)),
                            mean_extra_deg=float(rng.uniform(2, 12)))
    elif kind == 1:
        g = wl.config4(K=3500, B=2, Nmin=3, Nmax=4, D=64).den               # hubs long enough for clones
    else:
        g0 = wl.random_graph(rng, 5200, 9, mean_extra_deg=1.0)              # one giant hub and parallel arcs into it
        every = np.concatenate([np.arange(g0.K), np.arange(0, g0.K, 3)]).astype(np.int32)
        g = wl.Graph(g0.K, np.concatenate([g0.src, every]), np.concatenate([g0.dst, np.full(every.size, 7, np.int32)]),
                     np.concatenate([g0.logw, rng.normal(size=every.size).astype(np.float32)]), g0.pdf, g0.init, g0.final)
    logw = g.logw.copy()
    logw[rng.integers(0, logw.size, size=logw.size // 20)] = -np.inf        # zero-bar arcs
    lonely = int(rng.integers(0, g.K))
    logw[(g.src == lonely) | (g.dst == lonely)] = -np.inf                    # a state without arcs
    g = wl.Graph(g.K, g.src, g.dst, logw, g.pdf, g.init, g.final)
    D = int(g.pdf.max()) + 1
    h = _host_graph(g, D)
    assert fb.fb_graph_linear_weights(h) == 2
    W = np.exp(g.logw.astype(np.float64))
    x = rng.random(g.K)
    x[rng.integers(0, g.K, size=g.K // 10)] = 0.0
    for which, rows, cols in ((5, g.dst, g.src), (6, g.src, g.dst)):
        want = np.zeros(g.K)
        np.add.at(want, rows, W * x[cols])
        y = fb.fb_graph_schedule_apply_host(h, which, 0, x, np.full(g.K, np.nan))
        assert np.all(y[want == 0] == 0)
        np.testing.assert_allclose(y, want, rtol=2e-6, atol=0)              # weights (parallel arcs merged) as floats, products in double
        cycles, floor = fb.fb_graph_plan_cycles(h, which == 6)
        assert floor > 0 and floor % 2 == 0 and cycles >= floor
        assert cycles <= 2.5 * floor                                        # the order keeps most gathers free of conflicts
    h.destroy()
    small = wl.random_graph(rng, 300, 9)
    h = _host_graph(small, 9)
    assert fb.fb_graph_linear_weights(h) != 2                               # the 4-wave kernels' territory
    with pytest.raises(fb.FBError):
        fb.fb_graph_schedule_apply_host(h, 5, 0, np.zeros(small.K), np.zeros(small.K))
    h.destroy()
    far = g.logw.copy()
    far[g.src == g.src[np.flatnonzero(np.isfinite(far))[0]]] = -70.0          # every arc out of one state 2^-101: beyond the weight span
    h = _host_graph(wl.Graph(g.K, g.src, g.dst, far, g.pdf, g.init, g.final), D)
    assert fb.fb_graph_linear_weights(h) != 2
    h.destroy()
