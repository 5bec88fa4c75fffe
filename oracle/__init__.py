"""CPU oracle (fp64) for the forward-backward / LF-MMI path -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP library
and never calls it.  ``fb_oracle.c`` holds the arithmetic (the definitions of
the paper's Algorithm section written out in double precision); this file only
marshals numpy arrays into it.  ``layout.py`` holds the integer graph-layout
oracle (stable sorts).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fb_oracle.c")
_LIB = os.path.join(_HERE, "libfb_oracle.so")
_VSRC = os.path.join(_HERE, "viterbi_oracle.c")
_VLIB = os.path.join(_HERE, "libviterbi_oracle.so")
_lib = None
_vlib = None


def build(force: bool = False) -> str:
    """Compile fb_oracle.c with gcc (plain -O2, no fast-math) into libfb_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    if force or not os.path.exists(_VLIB) or os.path.getmtime(_VLIB) < os.path.getmtime(_VSRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-shared", "-fPIC", "-o", _VLIB, _VSRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.fbo_forward_backward.restype = ctypes.c_int
        _lib.fbo_lfmmi.restype = ctypes.c_int
        _lib.fbo_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().fbo_num_threads())


def set_num_threads(n: int) -> None:
    _load().fbo_set_num_threads(ctypes.c_int(n))


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def _graph_args(g):
    """(K, E, src, dst, logw, pdf, init, final, state_off, arc_off); packed arcs
    are regrouped by sequence (stable, so the order inside a sequence is kept)."""
    src, dst, logw = _c(g.src, np.int32), _c(g.dst, np.int32), _c(g.logw, np.float32)
    state_off = arc_off = None
    if g.state_off is not None:
        state_off = _c(g.state_off, np.int32)
        B = state_off.shape[0] - 1
        seq = np.searchsorted(state_off, src, side="right") - 1
        assert np.array_equal(seq, np.searchsorted(state_off, dst, side="right") - 1), \
            "an arc joins two packed graphs"
        order = np.argsort(seq, kind="stable")
        src, dst, logw = src[order], dst[order], logw[order]
        arc_off = np.zeros(B + 1, dtype=np.int64)
        np.cumsum(np.bincount(seq, minlength=B), out=arc_off[1:])
    keep = (src, dst, logw, _c(g.pdf, np.int32), _c(g.init, np.float32), _c(g.final, np.float32),
            state_off, arc_off)
    return keep


@dataclass
class FBResult:
    """Per selected sequence: alpha, beta, gamma [T_b, K_b]; rho [N, D]; logz."""
    alpha: list
    beta: list
    gamma: list
    rho: Optional[np.ndarray]
    logz: np.ndarray


def forward_backward(g, emis: np.ndarray, lengths: np.ndarray, sel: Optional[Sequence[int]] = None,
                     want_gamma: bool = True, want_rho: bool = True) -> FBResult:
    """alpha, beta, posteriors and log Z of the selected sequences (all by default)."""
    lib = _load()
    emis = _c(emis, np.float32)
    lengths = _c(lengths, np.int32)
    B, N, D = emis.shape
    sel = np.arange(B, dtype=np.int32) if sel is None else _c(sel, np.int32)
    src, dst, logw, pdf, init, fin, state_off, arc_off = _graph_args(g)
    if pdf.size and (pdf.min() < 0 or pdf.max() >= D):
        raise ValueError("pdf id outside [0, D)")
    if src.size and (min(src.min(), dst.min()) < 0 or max(src.max(), dst.max()) >= g.K):
        raise ValueError("arc endpoint outside [0, K)")
    Kb = np.array([(state_off[b + 1] - state_off[b]) if state_off is not None else g.K for b in sel],
                  dtype=np.int64)
    sizes = Kb * lengths[sel].astype(np.int64)
    ooff = np.zeros(sel.shape[0] + 1, dtype=np.int64)
    np.cumsum(sizes, out=ooff[1:])
    alpha = np.empty(int(ooff[-1]), dtype=np.float64)
    beta = np.empty_like(alpha)
    gamma = np.empty_like(alpha) if want_gamma else None
    rho = np.empty((sel.shape[0], N, D), dtype=np.float64) if want_rho else None
    logz = np.empty(sel.shape[0], dtype=np.float64)
    rc = lib.fbo_forward_backward(
        ctypes.c_int32(g.K), ctypes.c_int64(src.shape[0]), _p(src), _p(dst), _p(logw), _p(pdf), _p(init), _p(fin),
        _p(state_off), _p(arc_off), _p(emis), _p(lengths), ctypes.c_int32(B), ctypes.c_int32(N), ctypes.c_int32(D),
        _p(sel), ctypes.c_int32(sel.shape[0]), _p(ooff), _p(alpha), _p(beta), _p(gamma), _p(rho), _p(logz))
    if rc == -1:
        raise ValueError("oracle: malformed argument")
    if rc != 0:
        raise FloatingPointError("oracle: NaN log-likelihood")

    def split(a):
        return None if a is None else [a[ooff[i]:ooff[i + 1]].reshape(int(lengths[sel[i]]), int(Kb[i]))
                                       for i in range(sel.shape[0])]
    return FBResult(split(alpha), split(beta), split(gamma), rho, logz)


@dataclass
class LFMMIResult:
    logz_num: np.ndarray
    logz_den: np.ndarray
    grad: np.ndarray            # [nsel, N, D]

    @property
    def loss(self) -> float:
        return float(np.sum(self.logz_num - self.logz_den))


def lfmmi(den, num, emis: np.ndarray, lengths: np.ndarray, sel: Optional[Sequence[int]] = None) -> LFMMIResult:
    """LF-MMI objective terms and derivative for the selected sequences."""
    lib = _load()
    emis = _c(emis, np.float32)
    lengths = _c(lengths, np.int32)
    B, N, D = emis.shape
    sel = np.arange(B, dtype=np.int32) if sel is None else _c(sel, np.int32)
    d = _graph_args(den)
    n = _graph_args(num)
    if d[6] is not None or n[6] is None:
        raise ValueError("den must be a shared graph and num packed graphs")
    for g, a in ((den, d), (num, n)):
        if a[3].min() < 0 or a[3].max() >= D:
            raise ValueError("pdf id outside [0, D)")
        if a[0].size and (min(a[0].min(), a[1].min()) < 0 or max(a[0].max(), a[1].max()) >= g.K):
            raise ValueError("arc endpoint outside [0, K)")
    zn = np.empty(sel.shape[0], dtype=np.float64)
    zd = np.empty_like(zn)
    grad = np.empty((sel.shape[0], N, D), dtype=np.float64)
    rc = lib.fbo_lfmmi(
        ctypes.c_int32(den.K), ctypes.c_int64(d[0].shape[0]), _p(d[0]), _p(d[1]), _p(d[2]), _p(d[3]), _p(d[4]), _p(d[5]),
        ctypes.c_int32(num.K), ctypes.c_int64(n[0].shape[0]), _p(n[0]), _p(n[1]), _p(n[2]), _p(n[3]), _p(n[4]), _p(n[5]),
        _p(n[6]), _p(n[7]), _p(emis), _p(lengths), ctypes.c_int32(B), ctypes.c_int32(N), ctypes.c_int32(D),
        _p(sel), ctypes.c_int32(sel.shape[0]), _p(zn), _p(zd), _p(grad))
    if rc != 0:
        raise ValueError("oracle: malformed argument")
    return LFMMIResult(zn, zd, grad)


@dataclass
class ViterbiResult:
    score: np.ndarray           # [nsel] best-path score (tropical-semiring "log Z")
    path: np.ndarray            # [nsel, N] int32: state per frame (global numbering), -1 on padded frames


def viterbi(g, emis: np.ndarray, lengths: np.ndarray, sel: Optional[Sequence[int]] = None) -> ViterbiResult:
    """Best path (tropical semiring) of the selected sequences; see viterbi_oracle.c."""
    global _vlib
    if _vlib is None:
        build()
        _vlib = ctypes.CDLL(_VLIB)
        _vlib.vto_viterbi.restype = ctypes.c_int
    emis = _c(emis, np.float32)
    lengths = _c(lengths, np.int32)
    B, N, D = emis.shape
    sel = np.arange(B, dtype=np.int32) if sel is None else _c(sel, np.int32)
    src, dst, logw, pdf, init, fin, state_off, arc_off = _graph_args(g)
    score = np.empty(sel.shape[0], dtype=np.float64)
    path = np.empty((sel.shape[0], N), dtype=np.int32)
    rc = _vlib.vto_viterbi(
        ctypes.c_int32(g.K), ctypes.c_int64(src.shape[0]), _p(src), _p(dst), _p(logw), _p(pdf), _p(init), _p(fin),
        _p(state_off), _p(arc_off), _p(emis), _p(lengths), ctypes.c_int32(B), ctypes.c_int32(N), ctypes.c_int32(D),
        _p(sel), ctypes.c_int32(sel.shape[0]), _p(score), _p(path))
    if rc != 0:
        raise ValueError("oracle: malformed argument")
    return ViterbiResult(score, path)


def path_score(g, emis_b: np.ndarray, path: np.ndarray) -> float:
    """Score of a given state sequence in double precision: init + emissions + the best arc between consecutive
    states (parallel arcs: the largest weight) + final; -inf if an arc is missing.  Used to check that a path
    returned by anybody is valid and attains a score."""
    T = int(path.shape[0])
    s = float(g.init[path[0]]) + float(emis_b[0, g.pdf[path[0]]])
    for n in range(1, T):
        m = (g.src == path[n - 1]) & (g.dst == path[n])
        if not m.any():
            return float("-inf")
        s += float(np.max(g.logw[m])) + float(emis_b[n, g.pdf[path[n]]])
    return s + float(g.final[path[T - 1]])
