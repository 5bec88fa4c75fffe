"""CPU oracle (fp64) of the "leaky-HMM" denominator -- TEST INFRASTRUCTURE, like the rest of this package.

The paper names the leaky-HMM only as the approximation its comparison system makes in the probability domain
(Python and Julia recipes section; Analysis section, Table 1) and refers to the LF-MMI paper of Povey et al. (2016)
for it.  The reading taken here, stated as a model so that it has a plain definition: before every transition a
fraction ``leak`` of the total probability is handed out again over the states in proportion to the initial
distribution pi = exp(init) / sum exp(init).  With T the transition matrix of the graph this is the ordinary hidden
Markov model with the transition matrix

    T' = (I + leak * 1 pi^T) T,

the same initial and final weights and the same emissions; forward and backward variables, log Z and posteriors are
those of Eq. 13-15 for T'.  leak = 0 gives the graph itself.

Two routes, independent of one another:
  * ``leaky_graph``: T' written out as a dense arc list, to be handed to the exact oracle (fb_oracle.c) - the
    definition itself, only feasible for small K;
  * ``forward_backward``: the same quantities with the rank-one term kept apart (T'^T a = T^T (a + leak * sum(a) * pi)),
    in the probability domain with every frame's vector rescaled to sum 1 and the logarithms of the scales added up,
    all in float64 - feasible at any size.
``tests/test_leaky_pins.py`` pins the second to the first, both to leak = 0, to a closed form and to invariants.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np


def _pi(init: np.ndarray) -> np.ndarray:
    init = np.asarray(init, dtype=np.float64)
    m = init.max()
    if not np.isfinite(m):
        raise ValueError("leaky-HMM: no state has an initial weight above zero")
    p = np.exp(init - m)
    return p / p.sum()


def leaky_graph(g, leak: float):
    """The graph whose transition matrix is T' = (I + leak 1 pi^T) T, as a dense arc list (a shared graph only).
    Returns an object with the fields of ``workloads.Graph`` (K, src, dst, logw, pdf, init, final, state_off)."""
    if getattr(g, "state_off", None) is not None:
        raise ValueError("leaky-HMM: shared graphs only")
    K = int(g.K)
    T = np.zeros((K, K), dtype=np.float64)
    np.add.at(T, (np.asarray(g.src), np.asarray(g.dst)), np.exp(np.asarray(g.logw, dtype=np.float64)))
    u = _pi(g.init) @ T                      # u[j] = sum_k pi[k] T[k, j]
    Tp = T + leak * u[None, :]
    src, dst = np.nonzero(Tp > 0.0)

    class _G:
        pass
    out = _G()
    out.K = K
    out.src = src.astype(np.int32)
    out.dst = dst.astype(np.int32)
    out.logw = np.log(Tp[src, dst]).astype(np.float32)
    out.pdf = np.asarray(g.pdf, dtype=np.int32)
    out.init = np.asarray(g.init, dtype=np.float32)
    out.final = np.asarray(g.final, dtype=np.float32)
    out.state_off = None
    out.packed = False
    out.E = int(src.shape[0])
    return out


@dataclass
class LeakyResult:
    logz: np.ndarray            # [nsel]
    gamma: list                 # per selected sequence [T_b, K]
    rho: np.ndarray             # [nsel, N, D], zero on padded frames


def forward_backward(g, emis: np.ndarray, lengths: np.ndarray, leak: float,
                     sel: Optional[Sequence[int]] = None) -> LeakyResult:
    """log Z, state and pdf posteriors of the leaky-HMM of a shared graph, sequence by sequence."""
    if getattr(g, "state_off", None) is not None:
        raise ValueError("leaky-HMM: shared graphs only")
    emis = np.asarray(emis)
    B, N, D = emis.shape
    sel = list(range(B)) if sel is None else [int(b) for b in sel]
    K = int(g.K)
    src, dst = np.asarray(g.src, dtype=np.int64), np.asarray(g.dst, dtype=np.int64)
    w = np.exp(np.asarray(g.logw, dtype=np.float64))
    pdf = np.asarray(g.pdf, dtype=np.int64)
    pi = _pi(g.init)
    init = np.exp(np.asarray(g.init, dtype=np.float64))
    fin = np.exp(np.asarray(g.final, dtype=np.float64))
    logz = np.full(len(sel), -np.inf)
    gammas = []
    rho = np.zeros((len(sel), N, D), dtype=np.float64)
    for i, b in enumerate(sel):
        T = int(lengths[b])
        gam = np.zeros((T, K), dtype=np.float64)
        gammas.append(gam)
        if T <= 0:
            continue
        e = emis[b, :T].astype(np.float64)
        shift = np.where(np.isfinite(e.max(axis=1)), e.max(axis=1), 0.0)    # per frame, any scale serves
        v = np.exp(e - shift[:, None])[:, pdf]                               # [T, K], the emission factors
        # forward: a[n] = alpha_n / its sum, logs of the sums added up
        a = np.zeros((T, K))
        log_scale = float(shift.sum())
        x = init * v[0]
        ok = True
        for n in range(T):
            if n > 0:
                spread = a[n - 1] + leak * a[n - 1].sum() * pi               # (I + leak pi 1^T) alpha_{n-1}
                x = np.zeros(K)
                np.add.at(x, dst, w * spread[src])                           # T^T ...
                x *= v[n]
            s = x.sum()
            if not s > 0.0:
                ok = False
                break
            a[n] = x / s
            log_scale += np.log(s)
        if not ok:
            continue
        zl = float((a[T - 1] * fin).sum())
        if not zl > 0.0:
            continue
        logz[i] = log_scale + np.log(zl)
        # backward: bt = beta_n up to a factor (the posteriors are normalised frame by frame)
        bt = fin.copy()
        for n in range(T - 1, -1, -1):
            if n < T - 1:
                y = np.zeros(K)
                np.add.at(y, src, w * (v[n + 1] * bt)[dst])                  # T (v_{n+1} o beta_{n+1})
                bt = y + leak * float(pi @ y)                                # (I + leak 1 pi^T) ...
                bt = bt / bt.sum()
            p = a[n] * bt
            gam[n] = p / p.sum()
            np.add.at(rho[i, n], pdf, gam[n])
    return LeakyResult(logz, gammas, rho)
