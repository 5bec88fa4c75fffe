"""Pins of the tropical-semiring (Viterbi) oracle: exhaustive enumeration, the zero-temperature limit of the
pinned log-semiring oracle, and the sandwich score <= log Z <= score + log(number of state sequences)."""
from __future__ import annotations

import itertools

import numpy as np

import oracle
import workloads as wl


def _enumerate_best(g, emis_b, T):
    best, arg = -np.inf, None
    for p in itertools.product(range(g.K), repeat=T):
        s = oracle.path_score(g, emis_b, np.array(p))
        if s > best:
            best, arg = s, p
    return best, arg


def test_best_path_equals_exhaustive_enumeration():
    rng = np.random.default_rng(4)
    for seed in range(6):
        g = wl.tiny_graph(seed, int(rng.integers(2, 5)), 3)
        B, N = 3, 5
        emis = rng.normal(size=(B, N, 3)).astype(np.float32)
        lengths = np.array([5, 3, 1], np.int32)
        r = oracle.viterbi(g, emis, lengths)
        for b in range(B):
            T = int(lengths[b])
            want, _ = _enumerate_best(g, emis[b], T)
            if np.isneginf(want):
                assert np.isneginf(r.score[b]) and np.all(r.path[b] == -1)
                continue
            assert abs(r.score[b] - want) <= 1e-12 * max(1.0, abs(want))
            assert np.all(r.path[b, T:] == -1)
            assert abs(oracle.path_score(g, emis[b], r.path[b, :T]) - want) <= 1e-12 * max(1.0, abs(want))


def test_score_is_the_zero_temperature_limit_of_log_z():
    """tau * log Z computed from weights / tau and emissions / tau tends to the best-path score from above, and is
    within tau * log(number of state sequences) of it: the log-semiring oracle is pinned elsewhere."""
    rng = np.random.default_rng(8)
    g = wl.random_graph(rng, 12, 5, mean_extra_deg=2.0)
    emis = rng.normal(size=(2, 7, 5)).astype(np.float32)
    lengths = np.array([7, 4], np.int32)
    r = oracle.viterbi(g, emis, lengths)
    tau = 1.0 / 64                                   # a power of two: the scaled float inputs are exact
    gs = wl.Graph(g.K, g.src, g.dst, (g.logw / tau).astype(np.float32), g.pdf, (g.init / tau).astype(np.float32),
                  (g.final / tau).astype(np.float32))
    z = oracle.forward_backward(gs, (emis / tau).astype(np.float32), lengths, want_gamma=False, want_rho=False).logz * tau
    for b in range(2):
        n_paths_log = lengths[b] * np.log(g.K)
        assert r.score[b] - 1e-6 <= z[b] <= r.score[b] + tau * n_paths_log + 1e-6


def test_score_and_log_z_sandwich_and_chain_closed_form():
    w = wl.config2(B=4)
    r = oracle.viterbi(w.num, w.emis, w.lengths)
    z = oracle.forward_backward(w.num, w.emis, w.lengths, want_gamma=False, want_rho=False).logz
    assert np.all(r.score <= z + 1e-9)
    # a left-to-right chain visited in exactly as many frames as it has states has a single path
    rng = np.random.default_rng(1)
    g = wl.chain_graphs(rng, np.array([2]), 7)      # 6 states
    emis = rng.normal(size=(1, 6, 7)).astype(np.float32)
    r1 = oracle.viterbi(g, emis, np.array([6], np.int32))
    z1 = oracle.forward_backward(g, emis, np.array([6], np.int32)).logz
    assert abs(r1.score[0] - z1[0]) <= 1e-12 * abs(z1[0]) and list(r1.path[0]) == [0, 1, 2, 3, 4, 5]
