"""Seeded synthetic inputs for the forward-backward / LF-MMI hot path.

This module only *draws* inputs (graphs, emissions, lengths).  It contains none
of the method's arithmetic, so the CPU oracle and the HIP path can both be fed
from it without sharing any code of their own.

The paper benchmarks on graphs derived from the WSJ corpus (Analysis section:
a 454-state / 1036-arc alignment graph, a 3022-state / 50984-arc 3-gram
phonotactic denominator graph, 128 sequences of 700 frames, 84 network
outputs).  Those graphs are not available, so the five configurations below
stand in for them with the same structure: left-to-right chains of a few
hundred states for numerators, a random graph of a few thousand states with
about ten arcs per state for the denominator, Gaussian pseudo-log-likelihoods.

Conventions
-----------
* A graph is a ``Graph``: COO arcs ``(src, dst, logw)`` in generation order,
  ``pdf[k]`` (emission index of state k), ``init[k]`` and ``final[k]``
  log-weights (``-inf`` = the semiring zero).  ``state_off`` is ``None`` for a
  graph shared by every sequence of the batch, or an int32 array of B+1
  offsets for B graphs packed block-diagonally (Dealing-with-batches section).
* Emissions are float32 ``[B, N, D]``; ``lengths[b]`` real frames, the rest is
  padding filled with the same noise (a correct implementation ignores it).
* The random stream is ``numpy.random.default_rng(SEED0 + config)`` and every
  draw happens in the order the code below makes it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np

SEED0 = 211200709
NEG_INF = np.float32(-np.inf)


@dataclass
class Graph:
    K: int
    src: np.ndarray          # int32 [E]
    dst: np.ndarray          # int32 [E]
    logw: np.ndarray         # float32 [E]
    pdf: np.ndarray          # int32 [K]
    init: np.ndarray         # float32 [K]
    final: np.ndarray        # float32 [K]
    state_off: Optional[np.ndarray] = None   # int32 [B+1] when packed

    @property
    def E(self) -> int:
        return int(self.src.shape[0])

    @property
    def packed(self) -> bool:
        return self.state_off is not None

    def arcs_per_seq(self, B: int) -> np.ndarray:
        """Number of arcs each sequence of the batch runs over."""
        if not self.packed:
            return np.full(B, self.E, dtype=np.int64)
        seq_of_state = np.searchsorted(self.state_off, np.arange(self.K), side="right") - 1
        return np.bincount(seq_of_state[self.src], minlength=B).astype(np.int64)


def packed_subset(g: "Graph", sel) -> "Graph":
    """The packed graphs of the sequences in ``sel`` (in that order) as a packed graph of their own."""
    assert g.packed
    so = g.state_off
    src, dst, lw, pdf, init, fin, off = [], [], [], [], [], [], [0]
    for b in sel:
        k0, k1 = int(so[b]), int(so[b + 1])
        m = (g.src >= k0) & (g.src < k1)
        src.append(g.src[m] - k0 + off[-1]); dst.append(g.dst[m] - k0 + off[-1]); lw.append(g.logw[m])
        pdf.append(g.pdf[k0:k1]); init.append(g.init[k0:k1]); fin.append(g.final[k0:k1])
        off.append(off[-1] + k1 - k0)
    return Graph(K=off[-1], src=np.concatenate(src).astype(np.int32), dst=np.concatenate(dst).astype(np.int32),
                 logw=np.concatenate(lw).astype(np.float32), pdf=np.concatenate(pdf).astype(np.int32),
                 init=np.concatenate(init).astype(np.float32), final=np.concatenate(fin).astype(np.float32),
                 state_off=np.array(off, dtype=np.int32))


@dataclass
class Workload:
    name: str
    D: int
    emis: np.ndarray         # float32 [B, N, D]
    lengths: np.ndarray      # int32 [B]
    den: Optional[Graph] = None     # shared graph (or the only graph)
    num: Optional[Graph] = None     # packed graphs

    @property
    def B(self) -> int:
        return int(self.emis.shape[0])

    @property
    def N(self) -> int:
        return int(self.emis.shape[1])

    def arc_updates(self, graph: Graph) -> int:
        """2 * sum_b N_b * E_b: one forward and one backward visit of every arc
        on every real frame (the unit of the throughput metric)."""
        return int(2 * np.sum(self.lengths.astype(np.int64) * graph.arcs_per_seq(self.B)))


# --------------------------------------------------------------------------
# graph families
# --------------------------------------------------------------------------

def _log_dirichlet1_per_source(rng: np.random.Generator, deg: np.ndarray) -> np.ndarray:
    """log of a Dirichlet(1,...,1) draw for every source state, concatenated.
    A Dirichlet(1) vector is a vector of unit exponentials divided by its sum."""
    e = rng.exponential(size=int(deg.sum()))
    seg = np.repeat(np.arange(deg.shape[0]), deg)
    tot = np.bincount(seg, weights=e, minlength=deg.shape[0])
    return np.log(e / tot[seg]).astype(np.float32)


def random_graph(rng: np.random.Generator, K: int, D: int, *, mean_extra_deg: float = 9.0,
                 zipf_s: Optional[float] = None, uniform_init: bool = True) -> Graph:
    """Denominator-like graph: out-degree 1 + Poisson(mean_extra_deg); destinations
    uniform (with replacement) or, with ``zipf_s``, drawn by rank from the bounded
    Zipf pmf r**-zipf_s over 1..K through a random permutation of the states (hub
    states with a very high in-degree); weights log Dirichlet(1) per source;
    pdf ids uniform on [0, D); every state final with weight 0."""
    deg = 1 + rng.poisson(mean_extra_deg, size=K)
    E = int(deg.sum())
    src = np.repeat(np.arange(K, dtype=np.int32), deg)
    if zipf_s is None:
        dst = rng.integers(0, K, size=E, dtype=np.int64).astype(np.int32)
    else:
        perm = rng.permutation(K)
        pmf = np.arange(1, K + 1, dtype=np.float64) ** (-zipf_s)
        pmf /= pmf.sum()
        rank = rng.choice(K, size=E, p=pmf)
        dst = perm[rank].astype(np.int32)
    logw = _log_dirichlet1_per_source(rng, deg)
    pdf = rng.integers(0, D, size=K, dtype=np.int64).astype(np.int32)
    if uniform_init:
        init = np.full(K, -np.log(K), dtype=np.float32)
    else:
        init = np.full(K, NEG_INF, dtype=np.float32)
        init[0] = 0.0
    final = np.zeros(K, dtype=np.float32)
    return Graph(K, src, dst, logw, pdf, init, final)


def chain_graphs(rng: np.random.Generator, phones: np.ndarray, D: int) -> Graph:
    """Numerator-like graphs, one left-to-right chain per sequence, packed
    block-diagonally.  A chain of L phones has 3L states; every state has a
    self-loop and (except the last) an arc to the next state, all with weight
    log 0.5; the chain starts in its first state and ends in its last one with
    final weight log 0.5; pdf ids are uniform on [0, D)."""
    B = int(phones.shape[0])
    Kb = 3 * phones.astype(np.int64)
    off = np.zeros(B + 1, dtype=np.int64)
    np.cumsum(Kb, out=off[1:])
    K = int(off[-1])
    half = np.float32(np.log(0.5))
    src, dst = [], []
    for b in range(B):
        s = np.arange(off[b], off[b + 1], dtype=np.int32)
        # per state: self-loop first, then the forward arc
        a_src = np.repeat(s, 2)[:-1]
        a_dst = np.stack([s, s + 1], axis=1).reshape(-1)[:-1]
        src.append(a_src)
        dst.append(a_dst.astype(np.int32))
    src = np.concatenate(src)
    dst = np.concatenate(dst)
    logw = np.full(src.shape[0], half, dtype=np.float32)
    pdf = rng.integers(0, D, size=K, dtype=np.int64).astype(np.int32)
    init = np.full(K, NEG_INF, dtype=np.float32)
    init[off[:-1]] = 0.0
    final = np.full(K, NEG_INF, dtype=np.float32)
    final[off[1:] - 1] = half
    return Graph(K, src, dst, logw, pdf, init, final, state_off=off.astype(np.int32))


def ctc_graphs(labels: list, blank: int = 0) -> Graph:
    """Connectionist-temporal-classification topologies (the paper's introduction names CTC as one of
    the sequence criteria its forward-backward serves), one per label sequence, packed block-diagonally.
    A sequence of L labels has 2L + 1 states: blank, label 1, blank, label 2, ..., label L, blank.  Every state
    has a self-loop and an arc to the next state; a label state also has an arc to the next label state when the
    two labels differ.  All weights are 1-bar (log 1 = 0): the model has no transition probabilities.  A path
    starts in the first blank or the first label and ends in the last label or the last blank.  pdf of a blank
    state = ``blank``, of a label state = its label."""
    src, dst, pdf, init, final, off = [], [], [], [], [], [0]
    for lab in labels:
        lab = [int(x) for x in lab]
        L = len(lab)
        assert L >= 1 and all(x != blank for x in lab)
        k0, Kb = off[-1], 2 * L + 1
        for s in range(Kb):
            src.append(k0 + s); dst.append(k0 + s)                       # self-loop
            if s + 1 < Kb:
                src.append(k0 + s); dst.append(k0 + s + 1)               # to the next state
            if s % 2 == 1 and s + 2 < Kb and lab[s // 2] != lab[s // 2 + 1]:
                src.append(k0 + s); dst.append(k0 + s + 2)               # label to a different next label
            pdf.append(blank if s % 2 == 0 else lab[s // 2])
            init.append(0.0 if s <= 1 else NEG_INF)
            final.append(0.0 if s >= Kb - 2 else NEG_INF)
        off.append(k0 + Kb)
    E = len(src)
    return Graph(K=off[-1], src=np.asarray(src, np.int32), dst=np.asarray(dst, np.int32), logw=np.zeros(E, np.float32),
                 pdf=np.asarray(pdf, np.int32), init=np.asarray(init, np.float32), final=np.asarray(final, np.float32),
                 state_off=np.asarray(off, np.int32))


def ctc_workload(B: int = 12, D: int = 40, Lmin: int = 3, Lmax: int = 25, seed: int = SEED0 + 6) -> Workload:
    """Random label sequences (repeats allowed, so some skip arcs are absent), N_b uniform on [2 L_b + 1, 3 L_b + 4],
    emissions = log-softmax of N(0, 2) scores, as a network with a softmax output layer gives them."""
    rng = np.random.default_rng(seed)
    L = rng.integers(Lmin, Lmax + 1, size=B)
    labels = [rng.integers(1, D, size=int(l)).tolist() for l in L]
    lengths = np.array([int(rng.integers(2 * l + 1, 3 * l + 5)) for l in L], dtype=np.int32)
    N = int(lengths.max())
    x = rng.standard_normal((B, N, D)) * 2.0
    emis = (x - np.log(np.sum(np.exp(x), axis=2, keepdims=True))).astype(np.float32)
    w = Workload(name="ctc", D=D, emis=emis, lengths=lengths, num=ctc_graphs(labels))
    w.labels = labels
    return w


def _emissions(rng: np.random.Generator, B: int, N: int, D: int, sigma: float) -> np.ndarray:
    out = np.empty((B, N, D), dtype=np.float32)
    for b in range(B):                      # per sequence: bounded temporaries
        out[b] = rng.standard_normal((N, D), dtype=np.float32)
    out *= np.float32(sigma)
    return out


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config1() -> Workload:
    """Single sequence, 16 states, 48 arcs (self-loop + two uniform destinations
    per state), identity state->pdf map, start in state 0, all states final."""
    rng = np.random.default_rng(SEED0 + 1)
    K = 16
    src = np.repeat(np.arange(K, dtype=np.int32), 3)
    dst = np.empty(3 * K, dtype=np.int32)
    dst[0::3] = np.arange(K)
    dst[1::3] = rng.integers(0, K, size=K)
    dst[2::3] = rng.integers(0, K, size=K)
    logw = _log_dirichlet1_per_source(rng, np.full(K, 3))
    pdf = np.arange(K, dtype=np.int32)
    init = np.full(K, NEG_INF, dtype=np.float32)
    init[0] = 0.0
    final = np.zeros(K, dtype=np.float32)
    g = Graph(K, src, dst, logw, pdf, init, final)
    emis = _emissions(rng, 1, 50, K, 1.0)
    return Workload("config1", K, emis, np.array([50], dtype=np.int32), den=g)


def _chain_workload(name: str, seed: int, B: int, Lmin: int, Lmax: int, D: int, sigma: float,
                    frames: str) -> Workload:
    rng = np.random.default_rng(seed)
    phones = rng.integers(Lmin, Lmax + 1, size=B)
    g = chain_graphs(rng, phones, D)
    if frames == "3L..4L":
        lengths = rng.integers(3 * phones, 4 * phones + 1).astype(np.int32)
    else:  # "1.2x": chain length (3L states) times 1.2, rounded
        lengths = np.rint(3.6 * phones).astype(np.int32)
    emis = _emissions(rng, B, int(lengths.max()), D, sigma)
    return Workload(name, D, emis, lengths, num=g)


def config2(B: int = 32, Lmin: int = 10, Lmax: int = 40, D: int = 84) -> Workload:
    """Numerator-style batch of packed phone chains, N_b uniform on 3L..4L."""
    return _chain_workload("config2", SEED0 + 2, B, Lmin, Lmax, D, 2.0, "3L..4L")


def config3(K: int = 2000, B: int = 64, N: int = 150, D: int = 84) -> Workload:
    """Denominator graph with uniform destinations, all sequences full length."""
    rng = np.random.default_rng(SEED0 + 3)
    g = random_graph(rng, K, D)
    emis = _emissions(rng, B, N, D, 2.0)
    return Workload("config3", D, emis, np.full(B, N, dtype=np.int32), den=g)


def _den4(rng: np.random.Generator, K: int, D: int) -> Graph:
    return random_graph(rng, K, D, zipf_s=1.1)


def config4(K: int = 6000, B: int = 128, Nmin: int = 100, Nmax: int = 500, D: int = 3000) -> Workload:
    """Large denominator graph with Zipf(1.1)-skewed destinations, ragged lengths."""
    rng = np.random.default_rng(SEED0 + 4)
    g = _den4(rng, K, D)
    lengths = rng.integers(Nmin, Nmax + 1, size=B).astype(np.int32)
    emis = _emissions(rng, B, int(lengths.max()), D, 3.0)
    return Workload("config4", D, emis, lengths, den=g)


def config5(K: int = 6000, B: int = 128, Lmin: int = 30, Lmax: int = 150, D: int = 3000) -> Workload:
    """Full LF-MMI: the config-4 denominator graph (same seed, same draws) plus
    one packed numerator chain per utterance; N_b = round(3.6 L_b)."""
    g_den = _den4(np.random.default_rng(SEED0 + 4), K, D)
    w = _chain_workload("config5", SEED0 + 5, B, Lmin, Lmax, D, 3.0, "1.2x")
    w.den = g_den
    return w


def paper_shape_den(K: int = 3022, E_target: int = 50984, B: int = 128, N: int = 700, D: int = 84) -> Workload:
    """Context workload with the sizes of the paper's denominator benchmark
    (Table 1 / Analysis section): a random graph with that many states and, on
    average, that many arcs; 128 sequences of 700 frames; 84 outputs."""
    rng = np.random.default_rng(SEED0 + 6)
    g = random_graph(rng, K, D, mean_extra_deg=E_target / K - 1.0)
    emis = _emissions(rng, B, N, D, 2.0)
    return Workload("paper_shape_den", D, emis, np.full(B, N, dtype=np.int32), den=g)


def paper_shape_lfmmi(B: int = 128, N: int = 700, D: int = 84) -> Workload:
    """Context workload with the sizes of the paper's benchmark for both graphs (Table 1 / Analysis section):
    the denominator of ``paper_shape_den`` and, for every utterance, a numerator chain the size of the largest
    alignment graph of the paper's corpus (454 states; here 151 phones = 453 states, 905 arcs); 700 frames each."""
    w = paper_shape_den(B=B, N=N, D=D)
    rng = np.random.default_rng(SEED0 + 7)
    num = chain_graphs(rng, np.full(B, 151, dtype=np.int64), D)
    return Workload("paper_shape_lfmmi", D, w.emis, w.lengths, den=w.den, num=num)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


# --------------------------------------------------------------------------
# small cases for tests
# --------------------------------------------------------------------------

def tiny_graph(seed: int, K: int, D: int, *, density: float = 0.6, parallel_arcs: bool = True) -> Graph:
    """A small irregular graph for brute-force checks: random subset of the K*K
    possible arcs (some states may have no in- or out-arc), optionally a
    duplicated arc, arbitrary negative weights, non-trivial init/final with some
    semiring zeros, many-to-one pdf map."""
    rng = np.random.default_rng(seed)
    mask = rng.random((K, K)) < density
    src, dst = np.nonzero(mask)
    if parallel_arcs and src.size:
        src = np.concatenate([src, src[:1]])
        dst = np.concatenate([dst, dst[:1]])
    order = rng.permutation(src.size)        # arcs arrive in no particular order
    src, dst = src[order].astype(np.int32), dst[order].astype(np.int32)
    logw = (-rng.exponential(size=src.size)).astype(np.float32)
    pdf = rng.integers(0, D, size=K).astype(np.int32)
    init = (-rng.exponential(size=K)).astype(np.float32)
    final = (-rng.exponential(size=K)).astype(np.float32)
    if K > 2:
        init[rng.integers(0, K)] = NEG_INF
        final[rng.integers(0, K)] = NEG_INF
    return Graph(K, src, dst, logw, pdf, init, final)


def scaled(config: int, **kw) -> Workload:
    """A configuration with some of its sizes overridden (smaller parity cases)."""
    return CONFIGS[config](**kw)
