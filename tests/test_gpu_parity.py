"""Parity of the HIP path (through the C ABI) against the fp64 CPU oracle.

Tolerances (stated by the benchmark spec): log Z 1e-4 relative; posteriors and gradients
1e-5 absolute; the integer graph layout bit-exact.  Stored alpha / beta rows are
normalised, so they are compared after adding back the offsets (1e-4 relative)
and, more sharply, row by row relative to the row maximum.
"""
import sys

import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import layout as olayout

pytestmark = pytest.mark.gpu

TOL_LOGZ_REL = 1e-4
TOL_POST_ABS = 1e-5


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def fb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2112_00709_amd as lib
    lib.lib()                       # fails loudly if the HIP library is not built
    lib.POISON_NEW_BUFFERS = True   # outputs and workspaces start out as NaN: nothing passes on stale memory
    return lib


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def gpu_forward_backward(fb, g, D, emis, lengths, state="auto"):
    """alpha/beta reconstructed per sequence (float64), gamma, rho, logz from the GPU library."""
    import torch
    G = fb.graph_from(g, D, state=state)
    e, l = dev(emis), dev(lengths.astype(np.int32))
    B, N, _ = emis.shape
    a, acum, za = fb.fb_alpha(G, e, l)
    b, bcum, zb = fb.fb_beta(G, e, l)
    gam, rho = fb.fb_posteriors(G, a, b, l, B, N)
    # the pdf posteriors alone: for a shared graph of fitting size another kernel than the one above
    _, rho_only = fb.fb_posteriors(G, a, b, l, B, N, want_state=False)
    torch.cuda.synchronize()
    out = dict(alpha=host(a), beta=host(b), acum=host(acum), bcum=host(bcum),
               logz=host(za), logz_b=host(zb), gamma=host(gam), rho=host(rho), rho_only=host(rho_only))
    G.destroy()
    return out


def seq_view(g, arr, b, T):
    """Rows of sequence b from a [B,N,K] (shared) or [N,K] (packed) array."""
    if g.packed:
        return arr[:T, g.state_off[b]:g.state_off[b + 1]]
    return arr[b, :T]


def check_log_rows(got_norm, off_cum, want, what):
    """got_norm: float32 normalised rows [T,K]; off_cum: [T] the rows' shifts (float64); want: oracle rows (float64)."""
    assert off_cum.dtype == np.float64
    got = got_norm.astype(np.float64) + off_cum[:, None]
    inf_w = np.isneginf(want)
    assert np.array_equal(np.isneginf(got_norm), inf_w), f"{what}: -inf pattern differs"
    fin = ~inf_w
    err = np.abs(got[fin] - want[fin])
    # relative to the value (the shifts come in double; a stored entry carries float32 rounding of its own size)
    assert np.all(err <= TOL_LOGZ_REL * np.maximum(1.0, np.abs(want[fin]))), f"{what}: max err {err.max()}"
    # shape of each row relative to its maximum (what posteriors depend on)
    for n in range(want.shape[0]):
        if not fin[n].any():
            continue
        gw = want[n][fin[n]] - want[n][fin[n]].max()
        gg = got_norm[n][fin[n]].astype(np.float64) - got_norm[n][fin[n]].astype(np.float64).max()
        assert np.all(np.abs(gw - gg) <= 2e-5 * (1.0 + np.abs(gw))), f"{what}: frame {n} row shape"


def compare_fb(fb, g, D, emis, lengths, sel=None, name="", state="auto", post_tol=TOL_POST_ABS):
    B = emis.shape[0]
    sel = list(range(B)) if sel is None else list(sel)
    say(f"{name}: oracle on {len(sel)} of {B} sequences")
    ref = oracle.forward_backward(g, emis, lengths, sel=sel)
    say(f"{name}: fb_alpha / fb_beta / fb_posteriors B={B} N={emis.shape[1]} D={D} K={g.K} E={g.E} state={state}")
    out = gpu_forward_backward(fb, g, D, emis, lengths, state)
    for i, b in enumerate(sel):
        T = int(lengths[b])
        wz = ref.logz[i]
        for z in (out["logz"][b], out["logz_b"][b]):
            if np.isneginf(wz):
                assert np.isneginf(z)
            else:
                assert abs(z - wz) <= TOL_LOGZ_REL * max(1.0, abs(wz)), f"{name} b={b}: logZ {z} vs {wz}"
        if np.isneginf(wz):
            assert np.all(seq_view(g, out["gamma"], b, T) == 0) and np.all(out["rho"][b] == 0)
            assert np.all(out["rho_only"][b] == 0)
            continue
        check_log_rows(seq_view(g, out["alpha"], b, T), out["acum"][b, :T], ref.alpha[i], f"{name} alpha b={b}")
        check_log_rows(seq_view(g, out["beta"], b, T), out["bcum"][b, :T], ref.beta[i],
                       f"{name} beta b={b}")
        dg = np.abs(seq_view(g, out["gamma"], b, T) - ref.gamma[i]).max()
        dr = np.abs(out["rho"][b] - ref.rho[i]).max()
        assert dg <= post_tol, f"{name} b={b}: state posterior err {dg}"
        assert dr <= post_tol, f"{name} b={b}: pdf posterior err {dr}"
        dr = np.abs(out["rho_only"][b] - ref.rho[i]).max()
        assert dr <= post_tol, f"{name} b={b}: pdf posterior err {dr} (pdf posteriors alone)"
    # padded frames, every sequence
    N = emis.shape[1]
    for b in range(B):
        T = int(lengths[b])
        if T < N:
            assert np.all(out["rho"][b, T:] == 0) and np.all(out["rho_only"][b, T:] == 0)
            pad = out["gamma"][T:, g.state_off[b]:g.state_off[b + 1]] if g.packed else out["gamma"][b, T:]
            assert np.all(pad == 0)
            assert np.all(out["acum"][b, T:] == 0) and np.all(out["bcum"][b, T:] == 0)
            pa = out["alpha"][T:, g.state_off[b]:g.state_off[b + 1]] if g.packed else out["alpha"][b, T:]
            assert np.all(np.isneginf(pa))
    return out


def compare_lfmmi(fb, w, sel=None, name="", ragged=False, emis=None):
    """emis: emissions to use in place of w.emis (calls that follow one another in a test take different ones, so
    that what an earlier call left in recycled device memory is never the right answer of a later one)."""
    import torch
    B = w.B
    emis = w.emis if emis is None else emis
    sel = list(range(B)) if sel is None else list(sel)
    say(f"{name}: oracle LF-MMI on {len(sel)} of {B} sequences")
    ref = oracle.lfmmi(w.den, w.num, emis, w.lengths, sel=sel)
    say(f"{name}: lfmmi_loss_grad B={B} N={w.N} D={w.D} Kden={w.den.K} Knum={w.num.K}")
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    # workspace and gradient handed in, every byte set: NaN wherever the call does not write
    ws = torch.full((fb.fb_lfmmi_workspace_bytes(Gd, Gn, B, w.N, w.D),), 255, dtype=torch.uint8, device="cuda")
    grad = torch.full((B, w.N, w.D), float("nan"), dtype=torch.float32, device="cuda")
    loss, zn, zd, grad = fb.lfmmi_loss_grad(Gd, Gn, dev(emis), dev(w.lengths.astype(np.int32)), ws=ws, grad=grad,
                                            lengths_host=w.lengths if ragged else None)
    torch.cuda.synchronize()
    loss, zn, zd = float(host(loss)[0]), host(zn), host(zd)
    for i, b in enumerate(sel):
        assert abs(zn[b] - ref.logz_num[i]) <= TOL_LOGZ_REL * max(1.0, abs(ref.logz_num[i]))
        assert abs(zd[b] - ref.logz_den[i]) <= TOL_LOGZ_REL * max(1.0, abs(ref.logz_den[i]))
        gb = host(grad[b])
        err = np.abs(gb - ref.grad[i]).max()
        assert err <= TOL_POST_ABS, f"{name} b={b}: grad err {err}"
    assert abs(loss - float(np.sum(zn - zd))) <= 1e-9 * max(1.0, float(np.sum(np.abs(zn) + np.abs(zd))))
    if len(sel) == B:
        assert abs(loss - ref.loss) <= TOL_LOGZ_REL * float(np.sum(np.abs(ref.logz_num) + np.abs(ref.logz_den)))
    # properties that hold at any size: rows of real frames sum to 0, padded rows are 0
    rows = host(grad.sum(dim=2))
    absrows = host(grad.abs().sum(dim=2))
    for b in range(B):
        T = int(w.lengths[b])
        assert np.all(np.abs(rows[b, :T]) <= 2e-4)
        assert np.all(absrows[b, T:] == 0)
        assert np.all(absrows[b, :T] > 0)
    Gd.destroy(); Gn.destroy()
    return loss


# ------------------------------------------------------------------ layout on the device build

def test_layout_bit_exact_from_device_graph(fb):
    w = wl.config3(B=1, N=2)
    say("layout: config3 graph, device build")
    G = fb.graph_from(w.den, w.D)
    ref = olayout.graph_layout(w.den.K, w.D, w.den.src, w.den.dst, w.den.logw, w.den.pdf)
    for name, want in ref.items():
        assert np.array_equal(fb.fb_graph_layout(G, name).view(np.int32), want.view(np.int32)), name
    G.destroy()


# ------------------------------------------------------------------ the five configurations

def test_config1(fb):
    w = wl.config1()
    compare_fb(fb, w.den, w.D, w.emis, w.lengths, name="config1")


def test_config2(fb):
    w = wl.config2()
    compare_fb(fb, w.num, w.D, w.emis, w.lengths, name="config2")


def test_config3_full(fb):
    w = wl.config3()
    out = compare_fb(fb, w.den, w.D, w.emis, w.lengths, sel=range(0, 64, 4), name="config3")
    np.testing.assert_allclose(out["rho"].sum(axis=2), 1.0, atol=2e-5)      # every sequence, every frame


def test_config4_scaled(fb):
    """Full 6000-state hub graph (rows spread over up to 64 lanes, the largest hubs cloned), small ragged batch."""
    w = wl.config4(B=6, Nmin=20, Nmax=60)
    compare_fb(fb, w.den, w.D, w.emis, w.lengths, name="config4-scaled")


def test_config5_scaled(fb):
    w = wl.config5(B=6, Lmin=5, Lmax=15)
    compare_lfmmi(fb, w, name="config5-scaled")
    compare_fb(fb, w.num, w.D, w.emis, w.lengths, name="config5-scaled numerator")


def spread_by_length(lengths, n):
    """n sequences spread evenly over the batch in order of length (the shortest and the longest included)."""
    order = np.argsort(lengths, kind="stable")
    return sorted(int(order[i]) for i in np.unique(np.linspace(0, len(order) - 1, n).round().astype(int)))


def test_config4_full_size_sampled(fb):
    w = wl.config4()
    sel = spread_by_length(w.lengths, 32)
    out = compare_fb(fb, w.den, w.D, w.emis, w.lengths, sel=sel, name="config4-full")
    for b in range(w.B):
        T = int(w.lengths[b])
        np.testing.assert_allclose(out["rho"][b, :T].sum(axis=1), 1.0, atol=5e-5)
        np.testing.assert_allclose(out["gamma"][b, :T].sum(axis=1), 1.0, atol=5e-5)
    ok = np.isfinite(out["logz"]) & (np.abs(out["logz"] - out["logz_b"]) <= TOL_LOGZ_REL * np.abs(out["logz"]))
    assert ok.all()                                                  # forward and backward agree on log Z


def test_config5_full_size_every_sequence(fb):
    """Configuration 5 at full size, every one of the 128 sequences against the oracle, through both entry points;
    the second call takes other emissions than the first, and both get a workspace and a gradient buffer full of NaN."""
    w = wl.config5()
    compare_lfmmi(fb, w, name="config5-full")
    other = np.ascontiguousarray(w.emis[::-1])          # the same draws dealt to other sequences
    compare_lfmmi(fb, w, name="config5-full, as bench.py launches it", ragged=True, emis=other)


def test_lfmmi_large_denominator_ragged_every_rank(fb):
    """A denominator large enough for the 16-wave recursion kernel and the specialised gradient kernel (K = 1500,
    about 15k arcs) under a ragged batch of 64 (length groups, the counter-gated part of the longest range
    included): every sequence against the oracle, through both entry points, on different emissions."""
    w = wl.config5(K=1500, B=64, Lmin=3, Lmax=40, D=200)
    assert w.den.E >= 4096 and w.lengths.mean() < 0.85 * w.lengths.max()
    compare_lfmmi(fb, w, name="lfmmi, K=1500, B=64 ragged", ragged=True)
    compare_lfmmi(fb, w, name="lfmmi, K=1500, B=64, plain entry point", emis=np.ascontiguousarray(w.emis[::-1]))
    w = wl.config5(K=1500, B=80, Lmin=3, Lmax=40, D=200)
    compare_lfmmi(fb, w, name="lfmmi, K=1500, B=80 ragged", ragged=True, emis=np.ascontiguousarray(-w.emis))


def test_paper_shape_full_size_sampled(fb):
    """The shape of the paper's benchmark (Analysis section; Table 1): a 3022-state denominator of about 51k arcs,
    128 sequences of 700 frames, 84 outputs, numerator chains of 453 states.  16 sequences spread over the batch
    against the oracle: fb_alpha / fb_beta / fb_posteriors, and the LF-MMI call in its schedule for equal lengths."""
    w = wl.paper_shape_lfmmi()
    sel = list(range(3, w.B, 8))
    out = compare_fb(fb, w.den, w.D, w.emis, w.lengths, sel=sel, name="paper-shaped denominator")
    np.testing.assert_allclose(out["rho"].sum(axis=2), 1.0, atol=5e-5)
    del out
    compare_lfmmi(fb, w, sel=sel, name="paper-shaped LF-MMI (equal lengths)", ragged=True,
                  emis=np.ascontiguousarray(w.emis[::-1]))
    compare_lfmmi(fb, w, sel=sel, name="paper-shaped LF-MMI, plain entry point", emis=np.ascontiguousarray(-w.emis))


def test_carrier_precision_can_be_forced(fb):
    """Both carrier types on both kernel shapes: double on a large graph, single on small chains."""
    w = wl.config3(B=4, N=30)
    compare_fb(fb, w.den, w.D, w.emis, w.lengths, name="config3 wide state", state="wide")
    w = wl.config4(K=3000, B=3, Nmin=20, Nmax=30, D=500)
    compare_fb(fb, w.den, w.D, w.emis, w.lengths, name="zipf graph wide state", state="wide")
    c = wl.config2(B=6)
    # single carriers on left-to-right chains lose accuracy where alpha is far below the frame's best
    # state (that is why small graphs default to double): sane, but only to 1e-4
    compare_fb(fb, c.num, c.D, c.emis, c.lengths, name="config2 narrow state", state="narrow", post_tol=1e-4)
    compare_fb(fb, c.num, c.D, c.emis, c.lengths, name="config2 wide state", state="wide")


def test_long_chains_through_float_rows(fb):
    """fb_alpha / fb_beta hand their rows over as float32 (relative to the frame's best state, the shift in double).
    In a long left-to-right chain a state that matters can lie hundreds of units below its frame's best forward
    entry (the backward entry makes up for it), and a float that large is rounded at 2e-5: state posteriors formed
    from such rows by fb_posteriors are good to that, not to 1e-5.  (Inside lfmmi_loss_grad the numerators' rows stay
    in the carrier's type, double; the config-5 and paper-shaped gradient tests hold 1e-5.)  Sub-graphs of 511 and
    514 states also sit on both sides of the 512 states whose pdf offsets the data-moving wave keeps in registers."""
    rng = np.random.default_rng(7)
    D = 40
    phones = np.array([170, 171, 2])
    g = wl.chain_graphs(rng, phones, D)
    lengths = np.array([546, 550, 9], dtype=np.int32)
    emis = (rng.standard_normal((3, 551, D)) * 2.0).astype(np.float32)
    compare_fb(fb, g, D, emis, lengths, name="chains of 511 / 514 / 7 states over 550 frames", post_tol=5e-5)


def test_cloned_hub_rows_small(fb):
    """A 3500-state hub graph whose largest in-degree needs clones, every sequence checked in full."""
    w = wl.config4(K=3500, B=3, Nmin=10, Nmax=25, D=300)
    assert np.bincount(w.den.dst, minlength=3500).max() > 64 * 64
    compare_fb(fb, w.den, w.D, w.emis, w.lengths, name="config4 K=3500 (cloned hubs)")


def _pack(graphs):
    src, dst, lw, pdf, init, fin, off = [], [], [], [], [], [], [0]
    for g in graphs:
        src.append(g.src + off[-1]); dst.append(g.dst + off[-1]); lw.append(g.logw)
        pdf.append(g.pdf); init.append(g.init); fin.append(g.final); off.append(off[-1] + g.K)
    return wl.Graph(K=off[-1], src=np.concatenate(src).astype(np.int32), dst=np.concatenate(dst).astype(np.int32),
                    logw=np.concatenate(lw).astype(np.float32), pdf=np.concatenate(pdf).astype(np.int32),
                    init=np.concatenate(init).astype(np.float32), final=np.concatenate(fin).astype(np.float32),
                    state_off=np.array(off, dtype=np.int32))


def test_packed_graphs_with_hubs_and_clones(fb):
    """Packed graphs of different sizes on the 16-wave kernel, each with rows spread over many lanes and with cloned
    rows (the clone slots of a smaller graph sit behind the largest graph's states); and a shared graph with one
    giant hub that every state points to."""
    rng = np.random.default_rng(11)
    g = _pack([wl.random_graph(rng, K, 64, zipf_s=1.3) for K in (2200, 1700)])
    assert min(np.bincount(g.dst[g.dst >= 2200], minlength=g.K).max(), np.bincount(g.dst[g.dst < 2200]).max()) > 64 * 64
    emis = (rng.standard_normal((2, 14, 64)) * 2).astype(np.float32)
    compare_fb(fb, g, 64, emis, np.array([14, 9], np.int32), name="packed hub graphs")
    compare_fb(fb, g, 64, emis, np.array([14, 9], np.int32), name="packed hub graphs, double vectors", state="wide")
    g0 = wl.random_graph(rng, 2600, 17, mean_extra_deg=2.0)
    every = np.arange(g0.K, dtype=np.int32)
    hub = wl.Graph(g0.K, np.concatenate([g0.src, every]), np.concatenate([g0.dst, np.zeros(g0.K, np.int32)]),
                   np.concatenate([g0.logw, np.full(g0.K, -1.5, np.float32)]), g0.pdf, g0.init, g0.final)
    emis = (rng.standard_normal((2, 11, 17)) * 2).astype(np.float32)
    compare_fb(fb, hub, 17, emis, np.array([11, 6], np.int32), name="one giant hub")


def test_gradient_kernel_paths(fb):
    """lfmmi_loss_grad through the specialised gradient kernel (any state count up to its limit: rows of the
    workspace are padded to 16 bytes) and through the general posterior kernel (numerators over 512 states, more
    than 3072 pdfs), both against the oracle."""
    compare_lfmmi(fb, wl.config5(K=800, B=5, Lmin=3, Lmax=9, D=120), name="lfmmi, K=800 (specialised kernel)")
    for K in (798, 797, 799):
        compare_lfmmi(fb, wl.config5(K=K, B=5, Lmin=3, Lmax=9, D=120), name=f"lfmmi, K={K} (specialised kernel, padded rows)")
    compare_lfmmi(fb, wl.config5(K=1000, B=4, Lmin=3, Lmax=9, D=50), name="lfmmi, D=50 (fewer pdfs than threads)")
    compare_lfmmi(fb, wl.config5(K=300, B=3, Lmin=171, Lmax=180, D=40), name="lfmmi, numerators over 512 states (general kernel)")
    compare_lfmmi(fb, wl.config5(K=250, B=3, Lmin=3, Lmax=6, D=3100), name="lfmmi, D=3100 (general kernel)")


@pytest.mark.parametrize("B", [32, 37, 66])
def test_lfmmi_in_length_groups(fb, B):
    """Batches large enough for lfmmi_loss_grad to cut them into ranges of sequences by length (one denominator and
    one gradient launch per range on streams of their own): batch sizes that are and are not multiples of the
    range granularity, many equal lengths, every sequence checked against the oracle; a second call on the same
    graphs must give the same bits, the plain entry point the same objective and log Z bit for bit and the
    same gradient to rounding (the launches form the same sums in another order)."""
    import torch
    w2 = wl.config5(K=300, B=B, Lmin=2, Lmax=9, D=40)   # 8 distinct lengths: most ranks are decided by index
    assert np.unique(w2.lengths).size < B // 3
    assert w2.lengths.mean() < 0.85 * w2.lengths.max()   # unequal enough for the ragged entry point to cut
    compare_lfmmi(fb, w2, name=f"lfmmi in length groups, B={B}", ragged=True)
    Gd, Gn = fb.graph_from(w2.den, w2.D), fb.graph_from(w2.num, w2.D)
    e, l = dev(w2.emis), dev(w2.lengths.astype(np.int32))
    first = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, e, l, lengths_host=w2.lengths)]
    again = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, e, l, lengths_host=w2.lengths)]
    plain = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, e, l)]
    torch.cuda.synchronize()
    for i, (a, b, c) in enumerate(zip(first, again, plain)):
        assert np.array_equal(a, b)
        if i < 3:
            assert np.array_equal(a, c)                  # objective and log Z: the two entry points agree bit for bit
        else:
            assert np.allclose(a, c, rtol=0, atol=3e-6)  # gradient: the same sums formed in another order
    Gd.destroy(); Gn.destroy()


@pytest.mark.parametrize("phones,N,short", [(5, 24, (21, 23, 16)), (180, 560, (555, 559, 545))])
def test_lfmmi_equal_lengths_numerators_apart(fb, phones, N, short):
    """A batch of (nearly) equal lengths whose denominator workgroups take every compute unit (B = 128, a graph
    large enough for the 16-wave kernel): the ragged entry point then forms the denominator's share of the
    gradient while the numerator recursion runs and adds the numerators' share in a launch of its own: the
    one-wave kernel for numerators of up to 512 states, the general posterior kernel for larger ones (540 here).
    Every sequence against the oracle; a few shorter sequences so that padded frames occur; same results as the
    plain entry point to rounding."""
    import torch
    base = wl.paper_shape_den(K=1100, E_target=5000, B=128, N=N, D=30)
    rng = np.random.default_rng(5)
    num = wl.chain_graphs(rng, np.full(128, phones, dtype=np.int64), 30)
    lengths = base.lengths.copy()
    lengths[[3, 77, 127]] = short
    w = wl.Workload("equal lengths", 30, base.emis, lengths, den=base.den, num=num)
    assert w.lengths.mean() >= 0.85 * w.lengths.max()
    compare_lfmmi(fb, w, name=f"lfmmi, equal lengths, numerators of {3 * phones} states apart", ragged=True)
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    e, l = dev(w.emis), dev(w.lengths.astype(np.int32))
    apart = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, e, l, lengths_host=w.lengths)]
    again = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, e, l, lengths_host=w.lengths)]
    plain = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, e, l)]
    torch.cuda.synchronize()
    for a, b, c in zip(apart, again, plain):
        assert np.array_equal(a, b)
        assert np.allclose(a, c, rtol=0, atol=3e-6)      # the same sums formed in another order
    Gd.destroy(); Gn.destroy()


def test_lfmmi_with_an_infeasible_numerator(fb):
    """A numerator chain longer than its utterance: log Z_num = -inf, its pdf posteriors are 0, the gradient of that
    utterance is minus the denominator's pdf posteriors, nothing is NaN."""
    import torch
    w = wl.config5(K=400, B=4, Lmin=3, Lmax=6, D=60)
    lengths = w.lengths.copy()
    lengths[1] = 4                                   # 3 states per phone, at least 3 phones: cannot finish
    ref = oracle.lfmmi(w.den, w.num, w.emis, lengths)
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    loss, zn, zd, grad = fb.lfmmi_loss_grad(Gd, Gn, dev(w.emis), dev(lengths.astype(np.int32)))
    torch.cuda.synchronize()
    zn, zd, grad = host(zn), host(zd), host(grad)
    assert np.isneginf(zn[1]) and np.isneginf(ref.logz_num[1]) and np.isfinite(zd).all()
    assert not np.isnan(grad).any()
    for b in range(w.B):
        assert np.abs(grad[b] - ref.grad[b]).max() <= TOL_POST_ABS
    np.testing.assert_allclose(grad[1, :4].sum(axis=1), -1.0, atol=2e-5)
    assert np.isneginf(float(host(loss)[0]))
    Gd.destroy(); Gn.destroy()


def test_ctc_topology(fb):
    """A third graph family: CTC topologies (blank states tied to one pdf, two start and two end states per graph,
    unit weights), log-softmax emissions."""
    w = wl.ctc_workload()
    compare_fb(fb, w.num, w.D, w.emis, w.lengths, name="ctc topologies")
    compare_fb(fb, w.num, w.D, w.emis, w.lengths, name="ctc topologies, float vectors", state="narrow", post_tol=1e-4)


# ------------------------------------------------------------------ edge cases

def test_largest_graphs_the_kernels_take(fb):
    """State counts right at the documented limit (the state vectors fill the on-chip memory of a compute unit)."""
    rng = np.random.default_rng(21)
    K = fb.fb_limits_max_states(84, True)
    g = wl.random_graph(rng, K, 84, mean_extra_deg=2.0)
    emis = (rng.standard_normal((2, 6, 84)) * 2).astype(np.float32)
    compare_fb(fb, g, 84, emis, np.array([6, 4], np.int32), name=f"shared graph at the limit K={K}")
    Kp = fb.fb_limits_max_states(40, False)
    gp = _pack([wl.random_graph(rng, Kp, 40, mean_extra_deg=2.0), wl.random_graph(rng, 700, 40)])
    emis = (rng.standard_normal((2, 5, 40)) * 2).astype(np.float32)
    compare_fb(fb, gp, 40, emis, np.array([5, 5], np.int32), name=f"packed graphs, the larger at the limit K={Kp}")


def test_single_frame_and_single_state(fb):
    g = wl.Graph(1, np.array([0], np.int32), np.array([0], np.int32), np.array([-0.25], np.float32),
                 np.array([2], np.int32), np.array([-0.5], np.float32), np.array([-1.0], np.float32))
    emis = np.random.default_rng(1).normal(size=(3, 4, 5)).astype(np.float32)
    compare_fb(fb, g, 5, emis, np.array([1, 4, 2], np.int32), name="one-state graph, lengths 1/4/2")


def test_ragged_batch_with_fully_padded_tail(fb):
    w = wl.config3(K=500, B=5, N=12, D=30)
    lengths = np.array([12, 1, 7, 9, 3], np.int32)
    emis = np.concatenate([w.emis, np.full((5, 3, 30), np.nan, np.float32)], axis=1)     # padding must never be read into results
    compare_fb(fb, w.den, 30, emis, lengths, name="ragged + NaN padding")


@pytest.mark.parametrize("K,D", [(501, 30), (503, 3), (1022, 500), (6001, 3000)])
def test_pdf_posteriors_alone_rows_of_any_length(fb, K, D):
    """fb_posteriors asked for the pdf posteriors only reads the rows of a shared graph in 16-byte pieces whatever
    their length and alignment (the last piece of a row element by element), with one or several threads per pdf."""
    B, N = (3, 9) if K < 2000 else (2, 4)
    w = wl.config3(K=K, B=B, N=N, D=D)
    lengths = np.array([N, 1, N - 2][:B], np.int32)
    compare_fb(fb, w.den, D, w.emis, lengths, name=f"pdf posteriors alone, K={K} D={D}")


def test_infeasible_and_semiring_zero_inputs(fb):
    rng = np.random.default_rng(3)
    g = wl.chain_graphs(rng, np.array([2, 3, 2]), 11)                 # 6, 9, 6 states
    lengths = np.array([6, 8, 9], np.int32)                           # second chain cannot finish: log Z = -inf
    emis = rng.normal(size=(3, 9, 11)).astype(np.float32)
    emis[2, 4, :] = -np.inf                                           # a frame nobody can emit: log Z = -inf
    out = compare_fb(fb, g, 11, emis, lengths, name="infeasible chains")
    assert np.isneginf(out["logz"][1]) and np.isneginf(out["logz"][2]) and np.isfinite(out["logz"][0])
    assert not np.isnan(out["rho"]).any() and not np.isnan(out["gamma"]).any()
    g2 = wl.tiny_graph(9, 6, 4)                                       # -inf init/final entries, sourceless states
    e2 = rng.normal(size=(2, 7, 4)).astype(np.float32)
    e2[0, 3, 1] = -np.inf
    compare_fb(fb, g2, 4, e2, np.array([7, 5], np.int32), name="tiny graph with -inf entries")


def test_zero_length_sequence_is_skipped(fb):
    import torch
    w = wl.config5(K=200, B=4, Lmin=2, Lmax=4, D=40)
    lengths = w.lengths.copy(); lengths[1] = 0
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    say("zero-length sequence: lfmmi_loss_grad")
    loss, zn, zd, grad = fb.lfmmi_loss_grad(Gd, Gn, dev(w.emis), dev(lengths))
    torch.cuda.synchronize()
    keep = [0, 2, 3]
    ref = oracle.lfmmi(w.den, w.num, w.emis, w.lengths, sel=keep)
    assert abs(float(host(loss)[0]) - ref.loss) <= TOL_LOGZ_REL * float(np.sum(np.abs(ref.logz_num) + np.abs(ref.logz_den)))
    assert np.all(host(grad[1]) == 0) and np.isneginf(host(zn)[1]) and np.isneginf(host(zd)[1])
    np.testing.assert_allclose(host(grad)[keep], ref.grad, atol=TOL_POST_ABS)
    Gd.destroy(); Gn.destroy()


def test_shared_graph_equals_its_packed_replication(fb):
    """Block-diagonal batching: the same graph replicated as packed graphs gives the same posteriors."""
    rng = np.random.default_rng(8)
    g = wl.random_graph(rng, 70, 9, mean_extra_deg=3.0)
    B, N = 3, 10
    emis = rng.normal(size=(B, N, 9)).astype(np.float32)
    lengths = np.array([10, 4, 7], np.int32)
    rep = wl.Graph(B * g.K, np.concatenate([g.src + b * g.K for b in range(B)]).astype(np.int32),
                   np.concatenate([g.dst + b * g.K for b in range(B)]).astype(np.int32), np.tile(g.logw, B),
                   np.tile(g.pdf, B), np.tile(g.init, B), np.tile(g.final, B),
                   state_off=(np.arange(B + 1) * g.K).astype(np.int32))
    say("shared vs packed replication")
    a = gpu_forward_backward(fb, g, 9, emis, lengths)
    p = gpu_forward_backward(fb, rep, 9, emis, lengths)
    np.testing.assert_allclose(a["rho"], p["rho"], atol=2e-6)
    np.testing.assert_allclose(a["logz"], p["logz"], rtol=1e-6)
    for b in range(B):
        np.testing.assert_allclose(a["gamma"][b, :lengths[b]], p["gamma"][:lengths[b], b * g.K:(b + 1) * g.K], atol=2e-6)


def test_both_forms_of_the_arc_weights(fb):
    """Large graphs with float vectors run the kernel instantiation that takes weights as 2^w when every finite weight
    is within 64 binary orders of magnitude of 1, the adding one otherwise.  The same hub-heavy graph (rows spread
    over several lanes) with: ordinary weights; some arcs of weight zero-bar and some tiny but in-range weights,
    from sources that dominate the frame (they must not swamp the other terms of their rows); one weight out of
    range (falls back to the adding form).  All against the oracle."""
    rng = np.random.default_rng(77)
    D, B, N = 60, 6, 20
    g = wl.random_graph(rng, 1500, D, zipf_s=1.1, mean_extra_deg=6.0)
    emis = (rng.standard_normal((B, N, D)) * 2.5).astype(np.float32)
    emis[:, :, 7] += 30.0                                     # the states tied to pdf 7 dominate every frame
    lengths = np.array([20, 17, 20, 3, 11, 20], dtype=np.int32)
    strong = np.flatnonzero(g.pdf[g.src] == 7)                # arcs that leave the dominating states
    assert strong.size > 50

    G = fb.graph_from(g, D)
    assert fb.fb_graph_linear_weights(G)
    G.destroy()
    compare_fb(fb, g, D, emis, lengths, name="weights as 2^w, ordinary weights")

    w2 = g.logw.copy()
    w2[strong[0::3]] = -np.inf                                # zero-bar arcs out of the strongest sources
    w2[strong[1::3]] = -40.0                                  # 2^-57.7: tiny, in range
    g2 = wl.Graph(g.K, g.src, g.dst, w2, g.pdf, g.init, g.final)
    G = fb.graph_from(g2, D)
    assert fb.fb_graph_linear_weights(G)
    G.destroy()
    compare_fb(fb, g2, D, emis, lengths, name="weights as 2^w, zero-bar and tiny weights on dominating sources")

    w3 = g.logw.copy()
    w3[strong[0]] = -60.0                                     # 2^-86.6: out of range
    g3 = wl.Graph(g.K, g.src, g.dst, w3, g.pdf, g.init, g.final)
    G = fb.graph_from(g3, D)
    assert not fb.fb_graph_linear_weights(G)
    G.destroy()
    compare_fb(fb, g3, D, emis, lengths, name="a weight out of range: the adding form")


def test_strong_weight_on_a_weak_source(fb):
    """A row that mixes a strong weight (2^60) on an arc from a weak source with a tiny weight (2^-60) on an arc from
    the source that dominates the frame: the two terms are of comparable size although the gathered values lie more
    than a float's exponent range apart once normalised by their maximum.  Such weights are outside what the
    instantiations that take weights as 2^w accept (the probability-domain kernel's row sums, the 2^w form's
    span), so the graph runs in the adding form; every sequence against the oracle."""
    rng = np.random.default_rng(78)
    D, B, N = 60, 4, 16
    g = wl.random_graph(rng, 1500, D, zipf_s=1.1, mean_extra_deg=6.0)
    emis = (rng.standard_normal((B, N, D)) * 2.5).astype(np.float32)
    emis[:, :, 7] += 40.0                                     # the states tied to pdf 7 dominate every frame
    lengths = np.array([16, 9, 16, 2], dtype=np.int32)
    strong = np.flatnonzero(g.pdf[g.src] == 7)
    weak = np.flatnonzero(g.pdf[g.src] != 7)
    w = g.logw.copy()
    # rows (destinations) fed by both kinds of source
    both = np.intersect1d(g.dst[strong], g.dst[weak])
    assert both.size > 20
    for d in both[:40]:
        w[strong[g.dst[strong] == d][0]] = -60.0 * np.log(2.0)
        w[weak[g.dst[weak] == d][0]] = 60.0 * np.log(2.0)
    g2 = wl.Graph(g.K, g.src, g.dst, w, g.pdf, g.init, g.final)
    G = fb.graph_from(g2, D)
    assert fb.fb_graph_linear_weights(G) == 0
    G.destroy()
    compare_fb(fb, g2, D, emis, lengths, name="strong weights on weak sources: the adding form")


def test_probability_domain_gives_up_and_falls_back(fb):
    """The probability-domain recursion keeps a step's vector as floats scaled by a power of two; a run whose
    entries could fall below that range gives up (judged by the smallest row sum and the frame's smallest emission
    factor) and the sequence is redone in the log form.  Emissions that force this: a pdf far below the others in
    every frame of every sequence; in a single frame in the middle of one sequence; a pdf of probability zero.  The
    counter of given-up runs must move exactly where expected, and every sequence must match the oracle."""
    rng = np.random.default_rng(79)
    D, B, N = 60, 5, 18
    g = wl.random_graph(rng, 1500, D, zipf_s=1.1, mean_extra_deg=6.0)
    lengths = np.array([18, 7, 18, 1, 12], dtype=np.int32)
    base = (rng.standard_normal((B, N, D)) * 2.0).astype(np.float32)
    G = fb.graph_from(g, D)
    assert fb.fb_graph_linear_weights(G) == 2
    G.destroy()

    r0 = fb.fb_debug_linear_restarts()
    compare_fb(fb, g, D, base, lengths, name="probability domain, ordinary emissions")
    r1 = fb.fb_debug_linear_restarts()
    assert r1 == r0                                           # nothing gives up

    e2 = base.copy()
    e2[:, :, 11] = -400.0                                     # 2^-577 of the others: no float holds both
    compare_fb(fb, g, D, e2, lengths, name="a pdf far below the others in every frame")
    r2 = fb.fb_debug_linear_restarts()
    assert r2 - r1 == 2 * B                                   # forward and backward of every sequence (the first vector already holds such an entry)

    e3 = base.copy()
    e3[2, 9, 23] = -400.0                                     # one frame in the middle of one sequence
    compare_fb(fb, g, D, e3, lengths, name="a pdf far below the others in one frame")
    r3 = fb.fb_debug_linear_restarts()
    assert r3 - r2 == 2

    e4 = base.copy()
    e4[4, 5, :] = -np.inf
    e4[4, 5, 3] = 0.0                                         # a frame in which only one pdf has probability above zero
    e4[0, :, 40] = -np.inf
    compare_fb(fb, g, D, e4, lengths, name="pdfs of probability zero")
    r4 = fb.fb_debug_linear_restarts()
    assert r4 - r3 == 4


@pytest.mark.parametrize("case", ["odd_sizes", "clones", "one_frame", "big_emissions", "sparse_ends"])
def test_probability_domain_shapes(fb, case):
    """Shapes the probability-domain recursion has code paths of its own for, every sequence against the oracle:
    a number of pdfs and of states that are not multiples of four (rows staged and stored entry by entry, the
    emission row's last group); hub rows long enough for clones (a cloned state leaves as the sum of its clones, as
    a logarithm here); sequences of one and two frames and a batch of one; emissions far from zero (only
    differences to the frame's largest matter); few start and end states."""
    rng = np.random.default_rng(90)
    if case == "odd_sizes":
        g = wl.random_graph(rng, 1501, 85, zipf_s=1.2, mean_extra_deg=5.0)
        D, lengths = 85, np.array([9, 4, 12], dtype=np.int32)
    elif case == "clones":
        g = wl.config4(K=3500, B=2, Nmin=3, Nmax=4, D=64).den
        D, lengths = 64, np.array([7, 10], dtype=np.int32)
    elif case == "one_frame":
        g = wl.random_graph(rng, 1500, 60, zipf_s=1.1, mean_extra_deg=6.0)
        D, lengths = 60, np.array([1, 2, 1, 5], dtype=np.int32)
    elif case == "big_emissions":
        g = wl.random_graph(rng, 1500, 60, zipf_s=1.1, mean_extra_deg=6.0)
        D, lengths = 60, np.array([8], dtype=np.int32)
    else:
        g0 = wl.random_graph(rng, 1500, 60, zipf_s=1.1, mean_extra_deg=6.0)
        init = np.full(g0.K, -np.inf, dtype=np.float32); init[[3, 700]] = np.log(0.5)
        final = np.full(g0.K, -np.inf, dtype=np.float32); final[rng.integers(0, g0.K, size=40)] = 0.0
        g = wl.Graph(g0.K, g0.src, g0.dst, g0.logw, g0.pdf, init, final)
        D, lengths = 60, np.array([10, 6], dtype=np.int32)
    B, N = lengths.size, int(lengths.max()) + 1
    emis = (rng.standard_normal((B, N, D)) * 2.0).astype(np.float32)
    if case == "big_emissions":
        emis += 700.0
        emis[0, 3] -= 1500.0
    G = fb.graph_from(g, D)
    assert fb.fb_graph_linear_weights(G) == 2
    G.destroy()
    r0 = fb.fb_debug_linear_restarts()
    compare_fb(fb, g, D, emis, lengths, name=f"probability domain, {case}")
    assert fb.fb_debug_linear_restarts() == r0


def test_lfmmi_with_sequences_that_fall_back(fb):
    """Inside the LF-MMI call the denominator's rows reach the gradient kernel as the probability-domain kernel keeps
    them, except those of a sequence (and direction) that gave up and was redone in the log form: a batch that mixes
    both, every sequence against the oracle, both entry points.  Three causes of giving up are present: a pdf far
    below the others in one frame, a pdf of probability zero throughout, and (in this small graph as drawn) states
    that only feed one another, whose forward values fall below the range after some twenty frames."""
    w = wl.config5(K=1500, B=36, Lmin=3, Lmax=10, D=100)
    emis = w.emis.copy()
    long_ones = np.argsort(-w.lengths)[:3]
    emis[long_ones[0], 4, 17] = -400.0
    emis[long_ones[1], :, 55] = -np.inf
    r0 = fb.fb_debug_linear_restarts()
    compare_lfmmi(fb, w, name="lfmmi with fallbacks, plain entry point", emis=emis)
    r1 = fb.fb_debug_linear_restarts()
    assert 4 <= r1 - r0 < w.B                                 # of 2 B runs: some fall back, most do not
    compare_lfmmi(fb, w, name="lfmmi with fallbacks, ragged", ragged=True, emis=emis)
    assert fb.fb_debug_linear_restarts() - r1 == r1 - r0      # the same sequences, whatever the entry point


def test_backward_start_row_stays_in_range(fb):
    """The backward recursion's first row is the final weights, before the frame's emissions; the vector it continues
    from carries them.  When every state's emission in the last frame lies far below the frame's largest (a pdf no
    state is tied to), the scale that suits the vector would push that row beyond a float: it must stay finite, and
    the gradient of the last frame with it."""
    w = wl.config5(K=1500, B=6, Lmin=2, Lmax=6, D=100)
    w.den.pdf[:] = w.den.pdf % 50
    w.num.pdf[:] = w.num.pdf % 50
    emis = w.emis.copy()
    for b in range(w.B):
        emis[b, int(w.lengths[b]) - 1, 99] = 60.0        # 87 binary orders above everything a state emits
        emis[b, 0, 98] = 45.0
    compare_lfmmi(fb, w, name="lfmmi, an unused pdf far above the others in the last frame", emis=emis)
    compare_fb(fb, w.den, w.D, emis, w.lengths, name="the same through fb_alpha / fb_beta / fb_posteriors")


def test_lfmmi_calls_from_two_host_threads(fb):
    """Two host threads call lfmmi_loss_grad at the same time on the same graphs, each on its own inputs, workspace,
    outputs and stream (the library's side streams and events are shared by the process and guarded by a lock
    while a call enqueues): every call must give the bits a call made alone gives."""
    import threading
    import torch
    w = wl.config5(K=1500, B=40, Lmin=3, Lmax=12, D=100)
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    lengths = dev(w.lengths.astype(np.int32))
    emis = [dev(w.emis), dev(np.ascontiguousarray(-w.emis[::-1]))]
    need = fb.fb_lfmmi_workspace_bytes(Gd, Gn, w.B, w.N, w.D)
    alone = []
    for e in emis:
        out = fb.lfmmi_loss_grad(Gd, Gn, e, lengths)
        torch.cuda.synchronize()
        alone.append([host(x).copy() for x in out])
    results, errors = [None, None], []

    def worker(i):
        try:
            stream = torch.cuda.Stream()
            ws = torch.full((need,), 255, dtype=torch.uint8, device="cuda")
            grad = torch.full((w.B, w.N, w.D), float("nan"), dtype=torch.float32, device="cuda")
            with torch.cuda.stream(stream):
                for _ in range(12):
                    out = fb.lfmmi_loss_grad(Gd, Gn, emis[i], lengths, ws=ws, grad=grad)
            stream.synchronize()
            results[i] = [host(x).copy() for x in out]
        except Exception as exc:   # noqa: BLE001 (reported by the main thread)
            errors.append(exc)

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i in range(2):
        for a, b in zip(alone[i], results[i]):
            assert np.array_equal(a, b)
    Gd.destroy(); Gn.destroy()


def test_lfmmi_call_replayed_from_a_graph(fb):
    """The LF-MMI call captured into a HIP graph (through torch) on a side stream and replayed: the library's own
    streams are forked from and joined into the capturing stream with events, it allocates nothing and clears its
    counters with a kernel, so every replay - with new emissions written into the same input buffer between
    replays, and eager work in between - must give what the eager call gives on those emissions."""
    import torch
    w = wl.config5(K=300, B=40, Lmin=2, Lmax=9, D=40)
    assert w.lengths.mean() < 0.85 * w.lengths.max()
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    e = dev(w.emis).clone()
    l = dev(w.lengths.astype(np.int32))
    ws = torch.empty((fb.fb_lfmmi_workspace_bytes(Gd, Gn, w.B, w.N, w.D),), dtype=torch.uint8, device="cuda")
    grad = torch.empty((w.B, w.N, w.D), dtype=torch.float32, device="cuda")
    fb.lfmmi_loss_grad(Gd, Gn, e, l, ws=ws, grad=grad, lengths_host=w.lengths)      # warm-up outside the capture
    torch.cuda.synchronize()
    say("graph: capture of lfmmi_loss_grad_ragged")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = fb.lfmmi_loss_grad(Gd, Gn, e, l, ws=ws, grad=grad, lengths_host=w.lengths)
    rng = np.random.default_rng(3)
    for rep in range(3):
        new = (w.emis + rng.standard_normal(w.emis.shape).astype(np.float32) * (0.5 * rep)).astype(np.float32)
        e.copy_(dev(new))
        torch.cuda.synchronize()
        say(f"graph: replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        got = [host(x).copy() for x in out]
        ws2 = torch.empty_like(ws)
        want = [host(x).copy() for x in fb.lfmmi_loss_grad(Gd, Gn, dev(new), l, ws=ws2, lengths_host=w.lengths)]   # eager, other buffers
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(got, want)):
            if i < 3:
                assert np.array_equal(a, b), i
            else:
                assert np.allclose(a, b, rtol=0, atol=3e-6)
    Gd.destroy(); Gn.destroy()


def test_results_are_deterministic(fb):
    import torch
    w = wl.config5(K=800, B=5, Lmin=3, Lmax=8, D=120)
    Gd, Gn = fb.graph_from(w.den, w.D), fb.graph_from(w.num, w.D)
    e, l = dev(w.emis), dev(w.lengths)
    say("determinism: two lfmmi_loss_grad calls")
    r1 = fb.lfmmi_loss_grad(Gd, Gn, e, l)
    r2 = fb.lfmmi_loss_grad(Gd, Gn, e, l)
    torch.cuda.synchronize()
    for x, y in zip(r1, r2):
        assert torch.equal(x, y)
    Gd.destroy(); Gn.destroy()


def test_device_call_argument_errors(fb):
    w = wl.config2(B=3)
    G = fb.graph_from(w.num, w.D)
    e, l = dev(w.emis), dev(w.lengths)
    with pytest.raises(fb.FBError) as err:
        fb.fb_alpha(G, e[:2].contiguous(), l[:2].contiguous())          # B differs from the number of packed graphs
    assert err.value.code == fb.FB_EINVAL
    Gs = fb.graph_from(wl.config1().den, 16)
    with pytest.raises(fb.FBError) as err:
        fb.fb_alpha(Gs, e, l)                                           # D mismatch
    assert err.value.code == fb.FB_EINVAL
    with pytest.raises(fb.FBError) as err:
        fb.lfmmi_loss_grad(G, G, e, l)                                  # den must be shared
    assert err.value.code == fb.FB_EINVAL
    G.destroy(); Gs.destroy()
