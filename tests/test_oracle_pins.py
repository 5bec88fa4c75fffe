"""Pins for the fp64 CPU oracle: every check here compares oracle/ against
something that is not the oracle -- exhaustive path enumeration, dense
probability-domain matrix products (Eq. 4-5), a hand-computed example, closed
forms, invariants that follow from Eq. 1, finite differences (Eq. 17), the
block-diagonal batching and phony-end-state constructions of the
Dealing-with-batches section.  No GPU involved."""
import itertools
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import layout as olayout
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers

def dense_T(g):
    """Probability-domain transition matrix, row = source (parallel arcs add)."""
    T = np.zeros((g.K, g.K))
    np.add.at(T, (g.src, g.dst), np.exp(g.logw.astype(np.float64)))
    return T


def brute_force(g, emis_row, T_len):
    """Sum over all K**T state paths in the probability domain.
    Returns Z, alpha[T,K], beta[T,K], gamma[T,K] straight from their definitions:
    alpha_n(k) = p(x_0..x_n, z_n=k), beta_n(k) = p(x_{n+1}.., end | z_n=k)."""
    K = g.K
    A = dense_T(g)
    pi = np.exp(g.init.astype(np.float64))
    fin = np.exp(g.final.astype(np.float64))
    v = np.exp(emis_row.astype(np.float64))[:, g.pdf]          # [T, K]
    Z = 0.0
    gam = np.zeros((T_len, K))
    for z in itertools.product(range(K), repeat=T_len):
        p = pi[z[0]] * v[0, z[0]]
        for n in range(1, T_len):
            p *= A[z[n - 1], z[n]] * v[n, z[n]]
        p *= fin[z[-1]]
        Z += p
        for n in range(T_len):
            gam[n, z[n]] += p
    alpha = np.zeros((T_len, K))
    beta = np.zeros((T_len, K))
    for n in range(T_len):
        for z in itertools.product(range(K), repeat=n + 1):            # prefixes ending at frame n
            p = pi[z[0]] * v[0, z[0]]
            for m in range(1, n + 1):
                p *= A[z[m - 1], z[m]] * v[m, z[m]]
            alpha[n, z[-1]] += p
        for k in range(K):
            for z in itertools.product(range(K), repeat=T_len - 1 - n):  # suffixes after frame n
                p, prev = 1.0, k
                for i, s in enumerate(z):
                    p *= A[prev, s] * v[n + 1 + i, s]
                    prev = s
                beta[n, k] += p * fin[prev]
    return Z, alpha, beta, gam / Z


def lse(x, axis=None):
    x = np.asarray(x, dtype=np.float64)
    m = np.max(x, axis=axis, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        return np.squeeze(m + np.log(np.sum(np.exp(x - m), axis=axis, keepdims=True)), axis=axis)


def run1(g, emis, T=None):
    emis = np.asarray(emis, dtype=np.float32)
    if emis.ndim == 2:
        emis = emis[None]
    lengths = np.array([emis.shape[1] if T is None else T], dtype=np.int32)
    return oracle.forward_backward(g, emis, lengths)


def close_log(a, b, tol=1e-10):
    """Compare log-domain arrays; -inf must match exactly."""
    a, b = np.asarray(a), np.asarray(b)
    inf_a, inf_b = np.isneginf(a), np.isneginf(b)
    assert np.array_equal(inf_a, inf_b)
    np.testing.assert_allclose(a[~inf_a], b[~inf_b], rtol=0, atol=tol)


# ---------------------------------------------------------------- pins

def test_hand_computed_two_state_example():
    with open(os.path.join(GOLDEN, "two_state_example.json")) as f:
        ex = json.load(f)
    fr = lambda t: np.array([[float(Fraction(x)) for x in row] for row in t])
    arcs = ex["arcs"]
    g = wl.Graph(2,
                 np.array([a[0] for a in arcs], np.int32), np.array([a[1] for a in arcs], np.int32),
                 np.log([float(Fraction(a[2])) for a in arcs]).astype(np.float32),
                 np.arange(2, dtype=np.int32),
                 np.log([float(Fraction(x)) for x in ex["init"]]).astype(np.float32),
                 np.log([float(Fraction(x)) for x in ex["final"]]).astype(np.float32))
    r = run1(g, np.log(fr(ex["emis_prob"])))
    np.testing.assert_allclose(np.exp(r.alpha[0]), fr(ex["alpha"]), rtol=1e-6)
    np.testing.assert_allclose(np.exp(r.beta[0]), fr(ex["beta"]), rtol=1e-6)
    np.testing.assert_allclose(np.exp(r.logz[0]), float(Fraction(ex["Z"])), rtol=1e-6)
    np.testing.assert_allclose(r.gamma[0], fr(ex["gamma"]), rtol=1e-6)
    np.testing.assert_allclose(r.rho[0], fr(ex["gamma"]), rtol=1e-6)   # identity pdf map


@pytest.mark.parametrize("seed,K,T,D", [(1, 2, 5, 2), (2, 3, 5, 2), (3, 4, 4, 3), (4, 3, 6, 5), (5, 4, 5, 2)])
def test_brute_force_enumeration(seed, K, T, D):
    g = wl.tiny_graph(seed, K, D)
    rng = np.random.default_rng(100 + seed)
    emis = rng.normal(size=(T, D)).astype(np.float32)
    Z, alpha, beta, gam = brute_force(g, emis, T)
    assert Z > 0
    r = run1(g, emis)
    with np.errstate(divide="ignore"):
        close_log(r.alpha[0], np.log(alpha), 1e-10)
        close_log(r.beta[0], np.log(beta), 1e-10)
    assert abs(r.logz[0] - np.log(Z)) < 1e-10
    np.testing.assert_allclose(r.gamma[0], gam, atol=1e-12)
    rho = np.zeros((T, D))
    for k in range(K):
        rho[:, g.pdf[k]] += gam[:, k]
    np.testing.assert_allclose(r.rho[0], rho, atol=1e-12)


def test_dense_probability_domain_matrix_form():
    """Eq. 4-5 with numpy matmul in the probability domain on a short sequence."""
    g = wl.random_graph(np.random.default_rng(7), 40, 11, mean_extra_deg=3.0)
    T = 12
    emis = np.random.default_rng(8).normal(size=(T, 11)).astype(np.float32)
    A = dense_T(g)
    v = np.exp(emis.astype(np.float64))[:, g.pdf]
    a = np.zeros((T, g.K)); b = np.zeros((T, g.K))
    a[0] = np.exp(g.init.astype(np.float64)) * v[0]
    for n in range(1, T):
        a[n] = v[n] * (A.T @ a[n - 1])
    b[T - 1] = np.exp(g.final.astype(np.float64))
    for n in range(T - 2, -1, -1):
        b[n] = A @ (b[n + 1] * v[n + 1])
    Z = a[T - 1] @ b[T - 1]
    r = run1(g, emis)
    with np.errstate(divide="ignore"):
        close_log(r.alpha[0], np.log(a), 1e-9)
        close_log(r.beta[0], np.log(b), 1e-9)
    assert abs(r.logz[0] - np.log(Z)) < 1e-9
    np.testing.assert_allclose(r.gamma[0], a * b / Z, atol=1e-12)


def test_single_path_chain_closed_form():
    """A left-to-right chain run for exactly as many frames as it has states
    admits one path: log Z is the sum of its weights and every posterior is 0 or 1."""
    rng = np.random.default_rng(11)
    g = wl.chain_graphs(rng, np.array([4]), 9)          # 12 states
    T = g.K
    emis = rng.normal(size=(T, 9)).astype(np.float32)
    r = run1(g, emis)
    expect = sum(float(emis[n, g.pdf[n]]) for n in range(T)) + (T - 1) * float(np.float32(np.log(0.5))) \
        + float(np.float32(np.log(0.5)))
    assert abs(r.logz[0] - expect) < 1e-9
    np.testing.assert_allclose(r.gamma[0], np.eye(T), atol=1e-12)
    # one frame too few: no path reaches the final state
    r2 = oracle.forward_backward(g, emis[None], np.array([T - 1], np.int32))
    assert np.isneginf(r2.logz[0]) and np.all(r2.gamma[0] == 0) and np.all(r2.rho[0] == 0)


def test_constant_emission_markov_chain_closed_form():
    """With emis == c everywhere, a row-stochastic graph and final == 0, log Z = N*c
    and the posteriors are the n-step marginals of the Markov chain started at init."""
    g = wl.random_graph(np.random.default_rng(21), 30, 5, mean_extra_deg=2.0)
    T, c = 9, -0.75
    r = run1(g, np.full((T, 5), c, np.float32))
    assert abs(r.logz[0] - T * c) < 1e-6            # weights are float32-rounded logs
    A = dense_T(g)
    m = np.exp(g.init.astype(np.float64))
    for n in range(T):
        np.testing.assert_allclose(r.gamma[0][n], m / m.sum(), atol=1e-6)
        m = A.T @ m


@pytest.mark.parametrize("cfg", ["random", "zipf", "chain"])
def test_invariants(cfg):
    rng = np.random.default_rng(31)
    if cfg == "chain":
        g = wl.chain_graphs(rng, np.array([5]), 7)
        T, D = 22, 7
    else:
        g = wl.random_graph(rng, 60, 13, mean_extra_deg=4.0, zipf_s=1.1 if cfg == "zipf" else None)
        T, D = 25, 13
    emis = (2.0 * rng.normal(size=(T, D))).astype(np.float32)
    r = run1(g, emis)
    ab = r.alpha[0] + r.beta[0]
    z_n = lse(ab, axis=1)                                   # (+)-sum_k alpha_n (x) beta_n, every n
    np.testing.assert_allclose(z_n, r.logz[0], atol=1e-9)
    np.testing.assert_allclose(r.gamma[0].sum(axis=1), 1.0, atol=1e-12)
    np.testing.assert_allclose(r.rho[0].sum(axis=1), 1.0, atol=1e-12)
    assert np.all(r.gamma[0] >= 0)


def test_finite_difference_of_logz_is_pdf_posterior():
    """Eq. 17: d log Z / d phi[n, d] = posterior of pdf d at frame n."""
    rng = np.random.default_rng(41)
    g = wl.random_graph(rng, 25, 6, mean_extra_deg=2.0)
    T, D, h = 7, 6, 2.0 ** -9
    emis = (np.round(rng.normal(size=(T, D)) * 64) / 64).astype(np.float32)   # +-h exactly representable
    base = run1(g, emis)
    for n in range(T):
        for d in range(D):
            vals = []
            for step in (h, 2 * h):                        # Richardson: error O(h^4)
                ep, em = emis.copy(), emis.copy()
                ep[n, d] += step; em[n, d] -= step
                vals.append((run1(g, ep).logz[0] - run1(g, em).logz[0]) / (2 * step))
            fd = (4 * vals[0] - vals[1]) / 3
            assert abs(fd - base.rho[0][n, d]) < 1e-8


def _lfmmi_case(seed=51, B=3, D=9):
    rng = np.random.default_rng(seed)
    den = wl.random_graph(rng, 20, D, mean_extra_deg=2.0)
    phones = np.array([2, 3, 2][:B])
    num = wl.chain_graphs(rng, phones, D)
    lengths = np.array([8, 11, 7][:B], np.int32)
    N = int(lengths.max()) + 1                                  # a fully padded last frame
    emis = (np.round(rng.normal(size=(B, N, D)) * 32) / 32).astype(np.float32)
    return den, num, emis, lengths


def test_lfmmi_matches_separate_runs_and_sums_to_zero():
    den, num, emis, lengths = _lfmmi_case()
    r = oracle.lfmmi(den, num, emis, lengths)
    rn = oracle.forward_backward(num, emis, lengths)
    rd = oracle.forward_backward(den, emis, lengths)
    np.testing.assert_allclose(r.logz_num, rn.logz, atol=1e-12)
    np.testing.assert_allclose(r.logz_den, rd.logz, atol=1e-12)
    np.testing.assert_allclose(r.grad, rn.rho - rd.rho, atol=1e-12)
    for b, T in enumerate(lengths):
        np.testing.assert_allclose(r.grad[b, :T].sum(axis=1), 0.0, atol=1e-12)
        assert np.all(r.grad[b, T:] == 0)
    assert abs(r.loss - float(np.sum(rn.logz - rd.logz))) < 1e-12


def test_lfmmi_gradient_finite_difference():
    den, num, emis, lengths = _lfmmi_case(B=2)
    base = oracle.lfmmi(den, num, emis, lengths)
    h = 2.0 ** -9
    rng = np.random.default_rng(52)
    for _ in range(25):
        b = int(rng.integers(0, emis.shape[0])); n = int(rng.integers(0, emis.shape[1])); d = int(rng.integers(0, emis.shape[2]))
        vals = []
        for step in (h, 2 * h):
            ep, em = emis.copy(), emis.copy()
            ep[b, n, d] += step; em[b, n, d] -= step
            vals.append((oracle.lfmmi(den, num, ep, lengths).loss - oracle.lfmmi(den, num, em, lengths).loss) / (2 * step))
        fd = (4 * vals[0] - vals[1]) / 3
        assert abs(fd - base.grad[b, n, d]) < 1e-8            # also 0 on padded frames


def test_batch_equals_per_sequence_and_packed_equals_shared():
    """Block-diagonal batching: a batch is its sequences run one by one, and a shared
    graph gives the same result as the same graph replicated on the block diagonal."""
    rng = np.random.default_rng(61)
    g = wl.random_graph(rng, 15, 4, mean_extra_deg=2.0)
    B, N = 3, 9
    lengths = np.array([9, 5, 7], np.int32)
    emis = rng.normal(size=(B, N, 4)).astype(np.float32)
    batch = oracle.forward_backward(g, emis, lengths)
    for b in range(B):
        one = oracle.forward_backward(g, emis[b:b + 1, :lengths[b]], lengths[b:b + 1])
        np.testing.assert_array_equal(one.alpha[0], batch.alpha[b])
        np.testing.assert_array_equal(one.beta[0], batch.beta[b])
        assert one.logz[0] == batch.logz[b]
    rep = wl.Graph(B * g.K,
                   np.concatenate([g.src + b * g.K for b in range(B)]).astype(np.int32),
                   np.concatenate([g.dst + b * g.K for b in range(B)]).astype(np.int32),
                   np.tile(g.logw, B), np.tile(g.pdf, B), np.tile(g.init, B), np.tile(g.final, B),
                   state_off=(np.arange(B + 1) * g.K).astype(np.int32))
    packed = oracle.forward_backward(rep, emis, lengths)
    for b in range(B):
        np.testing.assert_array_equal(packed.alpha[b], batch.alpha[b])
        np.testing.assert_array_equal(packed.gamma[b], batch.gamma[b])
    np.testing.assert_array_equal(packed.rho, batch.rho)


def test_lengths_equal_phony_end_state_construction():
    """Variable length through an extra self-looping end state and semiring-zero
    padding of v, run to the padded length, equals running the real frames only."""
    rng = np.random.default_rng(71)
    g = wl.tiny_graph(72, 5, 3, density=0.5)
    D, Tb, Nmax = 3, 6, 10
    emis = rng.normal(size=(Nmax, D)).astype(np.float32)
    ref = oracle.forward_backward(g, emis[None], np.array([Tb], np.int32))
    K = g.K
    ninf = np.float32(-np.inf)
    aug = wl.Graph(K + 1,
                   np.concatenate([g.src, np.arange(K), [K]]).astype(np.int32),
                   np.concatenate([g.dst, np.full(K, K), [K]]).astype(np.int32),
                   np.concatenate([g.logw, g.final, [0.0]]).astype(np.float32),
                   np.concatenate([g.pdf, [D]]).astype(np.int32),
                   np.concatenate([g.init, [ninf]]).astype(np.float32),
                   np.concatenate([np.full(K, ninf), [0.0]]).astype(np.float32))
    keep = np.isfinite(aug.logw)                 # arcs with weight zero-bar are not stored
    aug.src, aug.dst, aug.logw = aug.src[keep], aug.dst[keep], aug.logw[keep]
    e2 = np.full((Nmax, D + 1), ninf, np.float32)
    e2[:Tb, :D] = emis[:Tb]
    e2[Tb:, D] = 0.0
    r = oracle.forward_backward(aug, e2[None], np.array([Nmax], np.int32))
    assert abs(r.alpha[0][Nmax - 1, K] - ref.logz[0]) < 1e-12
    assert abs(r.logz[0] - ref.logz[0]) < 1e-12
    close_log(r.alpha[0][:Tb, :K], ref.alpha[0], 1e-12)
    close_log(r.beta[0][:Tb, :K], ref.beta[0], 1e-12)
    np.testing.assert_allclose(r.gamma[0][:Tb, :K], ref.gamma[0], atol=1e-12)


def test_semiring_zero_handling():
    """States without in-arcs, -inf emissions and weights never give NaN."""
    g = wl.Graph(3, np.array([0, 0, 1], np.int32), np.array([0, 1, 1], np.int32),
                 np.array([-1.0, -0.5, -np.inf], np.float32), np.array([0, 1, 1], np.int32),
                 np.array([0.0, -np.inf, -np.inf], np.float32), np.zeros(3, np.float32))
    emis = np.zeros((4, 2), np.float32); emis[2, 1] = -np.inf
    r = run1(g, emis)
    for a in (r.alpha[0], r.beta[0], r.gamma[0], r.rho[0]):
        assert not np.any(np.isnan(a))
    assert np.all(np.isneginf(r.alpha[0][:, 2]))        # state 2 is unreachable
    assert np.isfinite(r.logz[0])
    np.testing.assert_allclose(r.gamma[0].sum(axis=1), 1.0, atol=1e-12)


def test_layout_oracle_invariants():
    w = wl.scaled(4, K=300, B=2, Nmin=5, Nmax=6, D=50)
    g = w.den
    L = olayout.graph_layout(g.K, w.D, g.src, g.dst, g.logw, g.pdf)
    for ptr, perm, key in ((L["in_ptr"], L["in_perm"], g.dst), (L["out_ptr"], L["out_perm"], g.src),
                           (L["pdf_ptr"], L["pdf_states"], g.pdf)):
        assert sorted(perm.tolist()) == list(range(len(key)))
        ks = key[perm]
        assert np.all(np.diff(ks) >= 0)
        same = np.diff(ks) == 0
        assert np.all(np.diff(perm)[same] > 0)            # ties keep the original order
        assert ptr[0] == 0 and ptr[-1] == len(key)
        for j in (0, 1, len(ptr) // 2, len(ptr) - 2):
            assert np.all(ks[ptr[j]:ptr[j + 1]] == j)
    assert np.array_equal(L["in_w"], g.logw[L["in_perm"]]) and np.array_equal(L["out_dst"], g.dst[L["out_perm"]])
    assert L["in_ptr"][-1] == g.E
    assert int(np.max(np.diff(L["in_ptr"]))) > 20 * g.E // g.K // 4      # the Zipf hub is there
