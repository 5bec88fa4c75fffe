"""Pins of the leaky-HMM oracle (oracle/leaky.py): the rank-one route against the definition written out as a
dense graph and run through the exact oracle, the limit leak = 0, a closed form, invariants.  CPU only."""
import numpy as np
import pytest

import oracle
import workloads as wl
from oracle import leaky


def _case(seed, K, D, B=3, N=7, density=0.5):
    rng = np.random.default_rng(seed)
    g = wl.tiny_graph(seed, K, D, density=density)
    emis = (rng.standard_normal((B, N, D)) * 1.5).astype(np.float32)
    lengths = np.array([N, max(1, N - 3), 1][:B], np.int32)
    return g, emis, lengths


@pytest.mark.parametrize("seed,K,D,leak", [(1, 5, 3, 0.1), (2, 9, 4, 1e-3), (3, 14, 6, 0.5), (4, 3, 2, 1e-5)])
def test_rank_one_route_equals_the_dense_graph_through_the_exact_oracle(seed, K, D, leak):
    g, emis, lengths = _case(seed, K, D)
    got = leaky.forward_backward(g, emis, lengths, leak)
    ref = oracle.forward_backward(leaky.leaky_graph(g, leak), emis, lengths)
    for b in range(emis.shape[0]):
        if np.isneginf(ref.logz[b]):
            assert np.isneginf(got.logz[b])
            continue
        assert abs(got.logz[b] - ref.logz[b]) <= 1e-6 * max(1.0, abs(ref.logz[b]))
        np.testing.assert_allclose(got.gamma[b], ref.gamma[b], atol=1e-6)
        np.testing.assert_allclose(got.rho[b], ref.rho[b], atol=1e-6)


def test_dense_graph_is_the_stated_matrix():
    g, _, _ = _case(7, 6, 3)
    leak = 0.25
    K = g.K
    T = np.zeros((K, K))
    np.add.at(T, (g.src, g.dst), np.exp(g.logw.astype(np.float64)))
    pi = np.exp(g.init.astype(np.float64)); pi /= pi.sum()
    want = (np.eye(K) + leak * np.outer(np.ones(K), pi)) @ T
    lg = leaky.leaky_graph(g, leak)
    got = np.zeros((K, K))
    got[lg.src, lg.dst] = np.exp(lg.logw.astype(np.float64))
    np.testing.assert_allclose(got, want, rtol=1e-6, atol=0)


@pytest.mark.parametrize("seed", [11, 12])
def test_no_leak_is_the_graph_itself(seed):
    g, emis, lengths = _case(seed, 8, 4)
    got = leaky.forward_backward(g, emis, lengths, 0.0)
    ref = oracle.forward_backward(g, emis, lengths)
    for b in range(emis.shape[0]):
        if np.isneginf(ref.logz[b]):
            assert np.isneginf(got.logz[b])
            continue
        assert abs(got.logz[b] - ref.logz[b]) <= 1e-9 * max(1.0, abs(ref.logz[b]))
        np.testing.assert_allclose(got.gamma[b], ref.gamma[b], atol=1e-9)
        np.testing.assert_allclose(got.rho[b], ref.rho[b], atol=1e-9)


def test_one_state_closed_form():
    """One state with a self-loop of weight w: pi = 1, T' = (1 + leak) w, so Z = init * final * prod_n v_n *
    ((1 + leak) w)^(T - 1)."""
    w, leak = 0.7, 0.3
    g = wl.Graph(1, np.array([0], np.int32), np.array([0], np.int32), np.array([np.log(w)], np.float32),
                 np.array([1], np.int32), np.array([-0.5], np.float32), np.array([-1.25], np.float32))
    emis = np.random.default_rng(5).normal(size=(2, 6, 3)).astype(np.float32)
    lengths = np.array([6, 2], np.int32)
    got = leaky.forward_backward(g, emis, lengths, leak)
    for b in range(2):
        T = int(lengths[b])
        # (the weight as the oracle sees it: float32 of log w)
        want = -0.5 - 1.25 + float(emis[b, :T, 1].astype(np.float64).sum()) + (T - 1) * (np.log(1 + leak) + float(np.float32(np.log(w))))
        assert abs(got.logz[b] - want) <= 1e-9 * max(1.0, abs(want))
        np.testing.assert_allclose(got.gamma[b], 1.0, atol=1e-12)


def test_posteriors_sum_to_one_and_the_leak_matters():
    rng = np.random.default_rng(9)
    g = wl.random_graph(rng, 60, 7, mean_extra_deg=2.0)
    emis = (rng.standard_normal((2, 12, 7)) * 2).astype(np.float32)
    lengths = np.array([12, 5], np.int32)
    a = leaky.forward_backward(g, emis, lengths, 0.05)
    b = leaky.forward_backward(g, emis, lengths, 0.0)
    for i in range(2):
        T = int(lengths[i])
        np.testing.assert_allclose(a.gamma[i].sum(axis=1), 1.0, atol=1e-12)
        np.testing.assert_allclose(a.rho[i, :T].sum(axis=1), 1.0, atol=1e-12)
        assert np.all(a.rho[i, T:] == 0)
        assert a.logz[i] > b.logz[i]                      # every entry of T' is at least that of T
        assert np.abs(a.rho[i] - b.rho[i]).max() > 1e-6   # and the posteriors are not those of the graph itself


def test_a_state_without_a_path_gets_one_through_the_leak():
    """A state no arc enters has forward probability zero after the first frame in the graph itself; with the leak it
    is still unreachable (the leak hands probability to states, the arcs out of them are the graph's), but a state
    that only the initial distribution reaches keeps being fed: its successors stay alive."""
    # 0 -> 1 -> 1, start in 0 only; without the leak state 0 is dead from the second frame on
    g = wl.Graph(2, np.array([0, 1], np.int32), np.array([1, 1], np.int32), np.log(np.array([1.0, 1.0], np.float32)),
                 np.array([0, 1], np.int32), np.array([0.0, -np.inf], np.float32), np.array([0.0, 0.0], np.float32))
    emis = np.zeros((1, 4, 2), np.float32)
    lengths = np.array([4], np.int32)
    exact = leaky.forward_backward(g, emis, lengths, 0.0)
    np.testing.assert_allclose(exact.gamma[0][1:, 1], 1.0, atol=1e-12)
    lk = leaky.forward_backward(g, emis, lengths, 0.5)
    # T' = [[0, 1.5], [0, 1.5]]: still only 0 -> 1 and 1 -> 1 (u = pi T = (0, 1)), weights 1.5: Z = 1.5^3
    assert abs(lk.logz[0] - 3 * np.log(1.5)) <= 1e-12


# ---------------------------------------------------------------- planted mistakes: the pins above must notice them

_MUTANTS = [
    ("the leak is left out of the forward recursion", "spread = a[n - 1] + leak * a[n - 1].sum() * pi", "spread = a[n - 1]"),
    ("the leak is left out of the backward recursion", "bt = y + leak * float(pi @ y)", "bt = y"),
    ("backward: the leaked share is the plain sum, not the sum weighted by pi", "leak * float(pi @ y)", "leak * float(y.sum())"),
    ("backward: the emissions of the frame itself instead of the next one", "(v[n + 1] * bt)[dst]", "(v[n] * bt)[dst]"),
    ("the final weights are dropped from log Z", "zl = float((a[T - 1] * fin).sum())", "zl = float(a[T - 1].sum())"),
    ("the emission scales are left out of log Z", "log_scale = float(shift.sum())", "log_scale = 0.0"),
    ("forward walks the arcs the wrong way round", "np.add.at(x, dst, w * spread[src])", "np.add.at(x, src, w * spread[dst])"),
    ("dense graph: the rank-one term transposed", "Tp = T + leak * u[None, :]", "Tp = T + leak * u[:, None]"),
    ("dense graph: pi taken as uniform", "u = _pi(g.init) @ T", "u = np.full(K, 1.0 / K) @ T"),
    ("posteriors are not normalised per frame", "gam[n] = p / p.sum()", "gam[n] = p"),
]


def _pins_hold(mod) -> bool:
    try:
        for seed, K, D, leak in [(1, 5, 3, 0.1), (3, 14, 6, 0.5)]:
            g, emis, lengths = _case(seed, K, D)
            got = mod.forward_backward(g, emis, lengths, leak)
            ref = oracle.forward_backward(mod.leaky_graph(g, leak), emis, lengths)
            for b in range(emis.shape[0]):
                if np.isneginf(ref.logz[b]):
                    if not np.isneginf(got.logz[b]):
                        return False
                    continue
                if abs(got.logz[b] - ref.logz[b]) > 1e-6 * max(1.0, abs(ref.logz[b])):
                    return False
                if np.abs(got.gamma[b] - ref.gamma[b]).max() > 1e-6 or np.abs(got.rho[b] - ref.rho[b]).max() > 1e-6:
                    return False
        # the stated matrix, typed out again
        g, _, _ = _case(7, 6, 3)
        T = np.zeros((g.K, g.K))
        np.add.at(T, (g.src, g.dst), np.exp(g.logw.astype(np.float64)))
        pi = np.exp(g.init.astype(np.float64)); pi /= pi.sum()
        lg = mod.leaky_graph(g, 0.25)
        got = np.zeros((g.K, g.K))
        got[lg.src, lg.dst] = np.exp(lg.logw.astype(np.float64))
        if not np.allclose(got, (np.eye(g.K) + 0.25 * np.outer(np.ones(g.K), pi)) @ T, rtol=1e-6, atol=0):
            return False
        # two states, worked by hand: Z = 1.5^3
        g2 = wl.Graph(2, np.array([0, 1], np.int32), np.array([1, 1], np.int32), np.log(np.array([1.0, 1.0], np.float32)),
                      np.array([0, 1], np.int32), np.array([0.0, -np.inf], np.float32), np.array([0.0, 0.0], np.float32))
        lk = mod.forward_backward(g2, np.zeros((1, 4, 2), np.float32), np.array([4], np.int32), 0.5)
        if abs(lk.logz[0] - 3 * np.log(1.5)) > 1e-12 or np.abs(lk.gamma[0].sum(axis=1) - 1.0).max() > 1e-12:
            return False
        # one state, closed form with emissions
        w, leak = 0.7, 0.3
        g1 = wl.Graph(1, np.array([0], np.int32), np.array([0], np.int32), np.array([np.log(w)], np.float32),
                      np.array([1], np.int32), np.array([-0.5], np.float32), np.array([-1.25], np.float32))
        emis = np.random.default_rng(5).normal(size=(1, 6, 3)).astype(np.float32)
        got = mod.forward_backward(g1, emis, np.array([6], np.int32), leak)
        want = -0.5 - 1.25 + float(emis[0, :, 1].astype(np.float64).sum()) + 5 * (np.log(1 + leak) + float(np.float32(np.log(w))))
        if abs(got.logz[0] - want) > 1e-9 * max(1.0, abs(want)):
            return False
        return True
    except (FloatingPointError, ValueError, IndexError):
        return False


def _load_variant(old=None, new=None):
    import os
    import types
    path = os.path.join(os.path.dirname(os.path.abspath(leaky.__file__)), "leaky.py")
    src = open(path).read()
    if old is not None:
        assert src.count(old) == 1, f"mutation site not found exactly once: {old!r}"
        src = src.replace(old, new)
    mod = types.ModuleType("leaky_variant")
    mod.__dict__["__name__"] = "leaky_variant"
    import sys
    sys.modules["leaky_variant"] = mod        # dataclasses look the module up
    exec(compile(src, path, "exec"), mod.__dict__)
    return mod


def test_pins_hold_for_the_oracle_as_it_is():
    assert _pins_hold(_load_variant())


@pytest.mark.parametrize("what,old,new", _MUTANTS, ids=[m[0] for m in _MUTANTS])
def test_planted_mistake_is_noticed(what, old, new):
    assert not _pins_hold(_load_variant(old, new)), f"the pins did not notice: {what}"
