"""fb_viterbi (the recursion in the tropical semiring) against the fp64 oracle: the score is unique and must agree;
the path need not be the oracle's, but it must be a path of the graph that attains the score.  GPU only."""
from __future__ import annotations

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
TOL_REL = 1e-4          # as for log Z


@pytest.fixture(scope="module")
def fb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2112_00709_amd as lib
    lib.lib()
    lib.POISON_NEW_BUFFERS = True   # outputs and workspaces start out as NaN
    return lib


def check(fb, g, D, emis, lengths, name, sel=None, state="auto"):
    import torch
    B, N, _ = emis.shape
    sel = list(range(B)) if sel is None else list(sel)
    print(f"[gpu-case] viterbi {name}: B={B} N={N} D={D} K={g.K} E={g.E} state={state}", flush=True)
    ref = oracle.viterbi(g, emis, lengths, sel=sel)
    G = fb.graph_from(g, D, state=state)
    score, path = fb.fb_viterbi(G, torch.from_numpy(emis).cuda(), torch.from_numpy(lengths.astype(np.int32)).cuda())
    torch.cuda.synchronize()
    score, path = score.cpu().numpy(), path.cpu().numpy()
    for i, b in enumerate(sel):
        T = int(lengths[b])
        assert np.all(path[b, T:] == -1)
        if np.isneginf(ref.score[i]):
            assert np.isneginf(score[b]) and np.all(path[b] == -1)
            continue
        assert abs(score[b] - ref.score[i]) <= TOL_REL * max(1.0, abs(ref.score[i])), (name, b, score[b], ref.score[i])
        p = path[b, :T]
        lo, hi = (g.state_off[b], g.state_off[b + 1]) if g.packed else (0, g.K)
        assert np.all((p >= lo) & (p < hi))
        got = oracle.path_score(g, emis[b], p)          # -inf if two consecutive states are not joined by an arc
        assert abs(got - ref.score[i]) <= TOL_REL * max(1.0, abs(ref.score[i])), (name, b, got, ref.score[i])
    G.destroy()
    return score, path


def test_viterbi_small_configurations(fb):
    w = wl.config1(); check(fb, w.den, w.D, w.emis, w.lengths, "config1")
    w = wl.config2(); check(fb, w.num, w.D, w.emis, w.lengths, "config2")
    w = wl.config3(B=6, N=40); check(fb, w.den, w.D, w.emis, w.lengths, "config3 B=6 N=40")
    w = wl.ctc_workload(); check(fb, w.num, w.D, w.emis, w.lengths, "ctc")


def test_viterbi_hub_graphs_with_clones(fb):
    """The longest rows are computed as clone states; a back-pointer may name a clone, the path names its state."""
    w = wl.config4(K=3500, B=3, Nmin=10, Nmax=25, D=300)
    check(fb, w.den, w.D, w.emis, w.lengths, "config4 K=3500")
    check(fb, w.den, w.D, w.emis, w.lengths, "config4 K=3500, double vectors", state="wide")
    rng = np.random.default_rng(11)
    gs = [wl.random_graph(rng, K, 64, zipf_s=1.3) for K in (2200, 1700)]
    off = np.array([0, 2200, 3900], np.int32)
    g = wl.Graph(K=3900, src=np.concatenate([gs[0].src, gs[1].src + 2200]).astype(np.int32),
                 dst=np.concatenate([gs[0].dst, gs[1].dst + 2200]).astype(np.int32),
                 logw=np.concatenate([gs[0].logw, gs[1].logw]), pdf=np.concatenate([gs[0].pdf, gs[1].pdf]),
                 init=np.concatenate([gs[0].init, gs[1].init]), final=np.concatenate([gs[0].final, gs[1].final]), state_off=off)
    emis = (rng.standard_normal((2, 14, 64)) * 2).astype(np.float32)
    check(fb, g, 64, emis, np.array([14, 9], np.int32), "packed hub graphs with clones")


def test_viterbi_config4_full_size_sampled(fb):
    w = wl.config4()
    order = np.argsort(w.lengths, kind="stable")
    sel = sorted(int(order[i]) for i in np.unique(np.linspace(0, w.B - 1, 32).round().astype(int)))
    check(fb, w.den, w.D, w.emis, w.lengths, "config4 full", sel=sel)


def test_viterbi_edge_cases(fb):
    rng = np.random.default_rng(3)
    g = wl.chain_graphs(rng, np.array([2, 3, 2]), 11)
    lengths = np.array([6, 8, 9], np.int32)                           # the second chain cannot finish
    emis = rng.normal(size=(3, 9, 11)).astype(np.float32)
    emis[2, 4, :] = -np.inf
    s, p = check(fb, g, 11, emis, lengths, "infeasible chains")
    assert np.isneginf(s[1]) and np.isneginf(s[2]) and np.isfinite(s[0])
    g1 = wl.Graph(1, np.array([0], np.int32), np.array([0], np.int32), np.array([-0.25], np.float32),
                  np.array([2], np.int32), np.array([-0.5], np.float32), np.array([-1.0], np.float32))
    e1 = rng.normal(size=(3, 4, 5)).astype(np.float32)
    check(fb, g1, 5, e1, np.array([1, 4, 2], np.int32), "one state")
    g2 = wl.tiny_graph(9, 6, 4)
    e2 = rng.normal(size=(2, 7, 4)).astype(np.float32)
    check(fb, g2, 4, e2, np.array([7, 5], np.int32), "tiny graph with -inf entries")
